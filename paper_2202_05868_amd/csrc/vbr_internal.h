// Internal layout of a built VBR matrix: the index arrays of the format, the packed values in
// the order the MFMA kernel reads them, and the workgroup schedule.  Host and device code of the
// library share this header; nothing outside the library includes it.
#pragma once

#include <cstdint>
#include <vector>

#include "vbr_spmm.h"

namespace vbrk {

constexpr int kSlabRows = 16;       // rows of one MFMA slab
constexpr int kStepK = 32;          // B rows consumed per K-step (one 16x16x32 MFMA deep)
constexpr int kMaxSlabs = 8;        // slabs per workgroup tile (128 rows)
constexpr int kFragElems = kSlabRows * kStepK;   // 512 16-bit values = 1 KiB per (slab, K-step)
constexpr int kTileN = 256;         // C columns per workgroup of the tile kernel
constexpr int kPanelN = 128;        // C columns per workgroup of the panel kernel
constexpr int kXcd = 8;             // L2 domains; workgroup i runs on domain i % 8

// One workgroup tile: up to kMaxSlabs slabs of ONE row group, walked over the group's K-steps.
struct TileDesc {
    int32_t ks_begin;    // first K-step of the tile's group (global K-step number)
    int32_t n_ks;        // K-steps of the group
    int64_t a_off;       // first value of the tile, in units of 8 values (16 bytes)
    int32_t row_begin;   // position in perm of the tile's first row
    int32_t n_rows;      // rows of the tile, 1 .. 16 * n_slabs
    int32_t n_slabs;     // ceil(n_rows / 16)
    int32_t group;       // row group the tile belongs to
};
static_assert(sizeof(TileDesc) == 32, "TileDesc is read by the kernel as 2 x 16 bytes");

// Position inside a (slab, K-step) fragment of the value at slab row m and K-step-local column
// kk (0..31 = row of the staged B panel), for a slab that stores `rows` rows (16, or fewer for the
// last slab of a tile: padding rows are not stored).  Lane l = m + 16 q of the wave holds 8 values
// (slots 0..7) of slab row m; a fragment is laid out [q][m][slot], so it takes rows * 32 values.
// The K order inside the step is permuted so that the four B rows a 16-lane group reads with one
// transposed LDS read, together with those of its neighbour group, fall into distinct LDS banks:
//   kk = 8 u + 4 v + e  ->  q = 2 (u / 2) + v,  slot = 4 (u % 2) + e.
inline int frag_index(int m, int kk, int rows)
{
    int u = kk >> 3, v = (kk >> 2) & 1, e = kk & 3;
    int q = 2 * (u >> 1) + v;
    int slot = 4 * (u & 1) + e;
    return ((q * rows + m) << 3) + slot;
}

// Values per K-step of a tile: full slabs take 512, the last slab rows_last * 32.
inline int64_t tile_kstep_stride(int32_t n_rows, int32_t n_slabs)
{
    int rows_last = n_rows - (n_slabs - 1) * kSlabRows;
    return (int64_t)(n_slabs - 1) * kFragElems + (int64_t)rows_last * kStepK;
}

// One workgroup panel: a few slabs (8) cut from the rows of SHORT row groups (height < 16) in
// permuted order, whatever group they belong to, walked over the union of the column blocks of
// those groups.  A B row panel is loaded once per K-step for all slabs; a slab only multiplies
// where its own groups store a block (mask bit), its fragment then follows in the value stream.
struct PanelDesc {
    int32_t ks_begin;    // first physical K-step of the panel (index into the host's pk_mask / pk_row)
    int32_t n_ks;        // physical K-steps
    int64_t a_off;       // first value of the panel, in units of 8 values (16 bytes)
    int32_t row_begin;   // first row of the panel in the panel-row list
    int32_t n_rows;      // rows of the panel, 1 .. 16 * slabs per panel
    int32_t meta_begin;  // first record of the panel in the device's K-step stream (pk_meta)
    int32_t pad;
};
static_assert(sizeof(PanelDesc) == 32, "PanelDesc is read by the kernel as 2 x 16 bytes");

constexpr int kPanelMaxFrags = 8;    // fragments per physical K-step (one load per wave); more -> the step is split
constexpr int kPanelMetaPad = 12;    // records appended to a panel's K-step stream, so that the kernel's look-ahead needs no bound checks

// Byte offsets of the sections inside the device buffer (each 256-byte aligned).
struct DeviceLayout {
    int64_t zeros_off = 0, tiles_off = 0, krow_off = 0, perm_off = 0, vals_off = 0, total = 0;
    int64_t panels_off = 0, pk_meta_off = 0, prow_off = 0;
    int64_t gcol_off = 0;      // (the column-gathered tiles follow the other tiles in the tiles section)
};

}  // namespace vbrk

struct vbr {
    int64_t n_rows = 0, n_cols = 0, nnz = 0;
    int32_t col_block = 0, dtype = 0;
    int32_t n_groups = 0;
    // the VBR index (bit-exact part of the format)
    std::vector<int32_t> perm, row_groups;
    std::vector<int64_t> blk_ptr, blk_off;
    std::vector<int32_t> blk_col;
    // kernel-side data
    int32_t lg_gran = 0;                 // log2 of the B-row gather granularity (rows per krow entry)
    std::vector<int64_t> ks_ptr;         // [n_groups+1] first global K-step of each group
    std::vector<int32_t> krow;           // first B row of each granule of each K-step, -1 = padding
    std::vector<vbrk::TileDesc> tiles;    // sorted by slab class, then by falling work
    int32_t class_begin[5] = {0, 0, 0, 0, 0};  // tiles of slab class c (1,2,4,8 slabs) are [class_begin[c], class_begin[c+1])
    std::vector<int64_t> group_first_tile;      // [n_groups+1] tiles of a group in creation order (for unpack)
    std::vector<int32_t> tile_of_group_order;   // creation order -> index in `tiles`
    std::vector<uint16_t> vals;          // packed fragments: tiles first, then panels, then 1 KiB of zeros
    // Rows of groups of height < 16 ("low rows") are collected in permuted order (prow) and cut into
    // chunks of 128 rows = 8 slabs.  A chunk is packed either as ONE PANEL (its slabs share the B rows
    // of the union of their column blocks) or as 8 COLUMN-GATHERED TILES (each slab gathers exactly
    // the B rows of the columns its own rows touch), whichever needs fewer loads.
    int32_t panel_slabs = 0;             // slabs per chunk (8); 0 = the matrix has no low rows
    std::vector<int32_t> prow;           // original row of every low row, in permuted order
    std::vector<int32_t> group_prow;     // [n_groups] first low-row position of a low group, -1 for the others
    std::vector<uint8_t> chunk_gather;   // [n_chunks] 1 = packed as column-gathered tiles, 0 = as a panel
    std::vector<int32_t> chunk_index;    // [n_chunks] index of its panel in `panels`, or of its first tile in `gtiles`
    std::vector<vbrk::TileDesc> gtiles;   // column-gathered tiles in creation order: row_begin = position in prow; group = -1 for
                                         // a slab of low rows, -2 - g for a tile of the tall group g (1 .. 8 slabs)
    std::vector<vbrk::TileDesc> gtiles_dev;      // the same tiles as the device holds them: by slab class, heaviest first
    int32_t gclass_begin[5] = {0, 0, 0, 0, 0};   // gathered tiles of slab class c are gtiles_dev[gclass_begin[c] .. gclass_begin[c+1])
    std::vector<int32_t> group_gt_first;         // [n_groups] first gathered tile of a tall group packed that way, -1 otherwise
    std::vector<int32_t> gcol;           // per K-step of a gathered tile 32 columns of A (= rows of B), ascending, -1 = padding
    std::vector<vbrk::PanelDesc> panels;
    std::vector<int32_t> pk_row;         // host only: first B row of each granule of each physical K-step, -1 = padding
    std::vector<uint32_t> pk_mask;       // host only: slabs present in each physical K-step
    std::vector<int32_t> pk_meta;        // device: per physical K-step one record {mask, granule rows...}; each panel's
                                         // records are followed by kPanelMetaPad records {0, rows of its last step}
    std::vector<int32_t> pk_logical;     // host only: K-step number inside the panel's union (a split step repeats it)
    std::vector<int64_t> pk_frag;        // host only: ordinal of the step's first fragment inside its panel
    std::vector<int64_t> p_union_ptr;    // host only: [n_panels+1] into p_union
    std::vector<int32_t> p_union;        // host only: ascending union of the column blocks of each panel
    vbrk::DeviceLayout lay;
    void *dev = nullptr;                 // uploaded buffer (caller-owned)
    // A multiply of several launches forks them over side streams and joins them on the caller's
    // stream (they write disjoint rows of C).  Created by vbr_upload on the device current then,
    // released through `release_dev` by vbr_free; all opaque to the host-only translation units.
    static constexpr int kSideStreams = 3;
    void *side_stream[kSideStreams] = {nullptr, nullptr, nullptr};
    void *ev_fork = nullptr;
    void *ev_join[kSideStreams] = {nullptr, nullptr, nullptr};
    void (*release_dev)(vbr *) = nullptr;
};
