// VBR construction on the host: index arrays of the format (section 2 and the last paragraph of
// section 3.1 of the paper), values packed as MFMA fragments, and the workgroup schedule.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "vbr_host.h"

namespace vbrk {
namespace {

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

inline int slab_class(int n_slabs)   // kernels exist for 1, 2, 4 and 8 slabs
{
    return n_slabs <= 1 ? 0 : n_slabs <= 2 ? 1 : n_slabs <= 4 ? 2 : 3;
}

// Rows of groups shorter than a slab go into panels when the block width allows the scalar
// gather path and there are enough of them to give every CU a panel or two (a panel is one long
// running workgroup per 128 columns; a handful of them would leave most of the chip idle).
// 8 slabs per panel: measured against 16, twice the workgroups (two resident per CU) gain more
// than the B rows shared by fewer slabs cost (noisy planted matrix 271 -> 185 us, others within 2 %).
constexpr int kPanelSlabs = 8;
constexpr int64_t kPanelMinRows = 4096;
inline bool use_panels(int lg_gran, int64_t short_rows) { return lg_gran >= 3 && short_rows >= kPanelMinRows; }
// Load instructions per K-step and 256 columns of C: a panel brings 32 B rows x 128 columns (8 loads)
// and up to 8 fragments (8 loads) per 128 columns; a one-slab tile 32 B rows x 256 columns (16 loads)
// and one fragment.  The direct-to-LDS load instruction is the unit of cost of both kernels.
constexpr int64_t kPanelStepCost = 32, kTileStepCost = 17;
constexpr int64_t kTileMaxGatherSteps = 64;  // K-steps a column-gathered tile of several slabs may walk before it is cut in two
constexpr int64_t kSlabMaxCols = 1024;       // columns a slab of low rows gathers before the next group starts a new slab

int build_impl(const vbr_csr_t *csr, const int32_t *perm, const int32_t *row_groups, int32_t G,
               int32_t col_block, vbr *v)
{
    const int64_t M = csr->n_rows;
    const int64_t KB = csr->n_cols / col_block;
    v->n_rows = M;
    v->n_cols = csr->n_cols;
    v->nnz = csr->nnz;
    v->col_block = col_block;
    v->dtype = csr->dtype;
    v->n_groups = G;
    v->perm.assign(perm, perm + M);
    v->row_groups.assign(row_groups, row_groups + G + 1);

    // B rows are gathered in granules of 2^lg_gran consecutive rows: the largest power of two
    // that divides the block width, at most one K-step.
    int lg = 0;
    while (lg < 5 && col_block % (2 << lg) == 0) ++lg;
    v->lg_gran = lg;
    const int gran = 1 << lg;
    const int per_step = kStepK >> lg;   // krow entries per K-step
    int64_t short_rows = 0;
    for (int32_t g = 0; g < G; ++g)
        if (row_groups[g + 1] - row_groups[g] < kSlabRows) short_rows += row_groups[g + 1] - row_groups[g];
    const bool panels_on = use_panels(lg, short_rows);

    v->blk_ptr.assign((size_t)G + 1, 0);
    v->blk_off.assign(1, 0);
    v->ks_ptr.assign((size_t)G + 1, 0);
    v->group_first_tile.assign((size_t)G + 1, 0);
    v->group_prow.assign((size_t)std::max<int32_t>(G, 1), -1);
    std::vector<int32_t> pos_of_block((size_t)std::max<int64_t>(KB, 1), -1);
    std::vector<int32_t> blocks;
    std::vector<int32_t> low_groups;            // groups lower than a slab, in group order
    std::vector<int32_t> tall_gathered;         // taller groups whose tiles gather single columns
    std::vector<int64_t> col_stamp((size_t)std::max<int64_t>(csr->n_cols, 1), -1);
    int64_t col_stamp_id = 0;
    std::vector<TileDesc> tiles;
    int64_t a_units = 0;   // running size of the packed values, in units of 8 values

    // pass 1: the VBR index arrays; K-step gather lists and tiles of the tall groups; the row list
    // of the short groups
    for (int32_t g = 0; g < G; ++g) {
        const int64_t r0 = row_groups[g], r1 = row_groups[g + 1];
        const int64_t h = r1 - r0;
        blocks.clear();
        for (int64_t q = r0; q < r1; ++q) {
            const int64_t r = perm[q];
            int64_t last = -1;
            for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p) {
                const int64_t j = csr->col_idx[p] / col_block;
                if (j != last) {
                    if (pos_of_block[j] < 0) { pos_of_block[j] = 0; blocks.push_back((int32_t)j); }
                    last = j;
                }
            }
        }
        std::sort(blocks.begin(), blocks.end());
        for (int32_t j : blocks) pos_of_block[j] = -1;
        const int64_t nb = (int64_t)blocks.size();
        for (int64_t t = 0; t < nb; ++t) {
            v->blk_col.push_back(blocks[t]);
            v->blk_off.push_back(v->blk_off.back() + h * col_block);
        }
        v->blk_ptr[g + 1] = v->blk_ptr[g] + nb;
        v->ks_ptr[g + 1] = v->ks_ptr[g];
        v->group_first_tile[g + 1] = v->group_first_tile[g];

        if (h < kSlabRows) {                        // low group: its rows join the low rows (ordered below)
            low_groups.push_back(g);
            continue;
        }

        const int64_t Kg = nb * col_block;
        const int64_t n_ks = (Kg + kStepK - 1) / kStepK;
        const int64_t slabs = (h + kSlabRows - 1) / kSlabRows;
        const int64_t nt = (slabs + kMaxSlabs - 1) / kMaxSlabs;
        // Blocks with much fill-in hold many columns without a single entry.  When the columns the
        // rows of the group's tiles actually touch need at most two thirds of the K-steps of its whole
        // blocks, the tiles gather those columns instead (a gathered load costs the load path about
        // a third more than a load of whole blocks); they are packed after the low rows, below.
        {
            int64_t gather_ks = 0, row = 0;
            for (int64_t t = 0; t < nt; ++t) {
                const int64_t s = slabs / nt + (t < slabs % nt ? 1 : 0);
                const int64_t n_rows = std::min<int64_t>(s * kSlabRows, h - row);
                ++col_stamp_id;
                int64_t cols_t = 0;
                for (int64_t q = r0 + row; q < r0 + row + n_rows; ++q)
                    for (int64_t p = csr->row_ptr[perm[q]]; p < csr->row_ptr[perm[q] + 1]; ++p)
                        if (col_stamp[csr->col_idx[p]] != col_stamp_id) { col_stamp[csr->col_idx[p]] = col_stamp_id; ++cols_t; }
                gather_ks += (cols_t + kStepK - 1) / kStepK;
                row += n_rows;
            }
            if (3 * gather_ks <= 2 * nt * n_ks) {
                tall_gathered.push_back(g);
                continue;
            }
        }
        if (v->ks_ptr[g] + n_ks > INT32_MAX / 64) return VBR_EINVAL;
        v->ks_ptr[g + 1] = v->ks_ptr[g] + n_ks;
        for (int64_t e = 0; e < n_ks * per_step; ++e) {
            const int64_t k = e * gran;
            if (k < Kg) v->krow.push_back((int32_t)((int64_t)blocks[k / col_block] * col_block + k % col_block));
            else v->krow.push_back(-1);
        }

        v->group_first_tile[g + 1] = v->group_first_tile[g] + nt;
        int64_t row = 0;
        for (int64_t t = 0; t < nt; ++t) {
            const int64_t s = slabs / nt + (t < slabs % nt ? 1 : 0);
            TileDesc td;
            td.ks_begin = (int32_t)v->ks_ptr[g];
            td.n_ks = (int32_t)n_ks;
            td.a_off = a_units;
            td.row_begin = (int32_t)(r0 + row);
            td.n_rows = (int32_t)std::min<int64_t>(s * kSlabRows, h - row);
            td.n_slabs = (int32_t)s;
            td.group = g;
            a_units += n_ks * tile_kstep_stride(td.n_rows, td.n_slabs) / 8;
            row += td.n_rows;
            tiles.push_back(td);
        }
    }

    // The order of the low groups in the low-row list is free (C is written through the row list).
    // Slabs cut from a list in which groups with similar block patterns follow each other gather
    // far fewer B rows, so the list is built cluster by cluster: the first group not yet placed
    // leads a cluster and takes with it every later group that shares at least half of the smaller
    // of the two block sets with the LEADER (overlap coefficient >= 1/2, which unlike the Jaccard
    // similarity does not fade when both sets carry noise blocks of their own; no pattern update:
    // this only orders the packing, the blocking is the caller's).  Candidates come from an index column block -> low groups.  When
    // the first 512 leaders find next to nothing (unstructured matrices), the rest keeps its order.
    {
        const int64_t n_low = (int64_t)low_groups.size();
        std::vector<int32_t> order, cluster_first;      // cluster_first: index in `order` of every cluster's leader
        order.reserve((size_t)n_low);
        std::vector<int64_t> inv_ptr((size_t)KB + 1, 0);
        for (const int32_t g : low_groups)
            for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b) inv_ptr[v->blk_col[b] + 1]++;
        for (int64_t b = 0; b < KB; ++b) inv_ptr[b + 1] += inv_ptr[b];
        std::vector<int32_t> inv((size_t)inv_ptr[KB]);
        {
            std::vector<int64_t> fill(inv_ptr.begin(), inv_ptr.end() - 1);
            for (int64_t i = 0; i < n_low; ++i) {
                const int32_t g = low_groups[i];
                for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b) inv[fill[v->blk_col[b]]++] = (int32_t)i;
            }
        }
        std::vector<int64_t> first(inv_ptr.begin(), inv_ptr.end() - 1);
        std::vector<uint8_t> placed((size_t)n_low, 0);
        std::vector<int32_t> cnt((size_t)n_low, 0), hit;
        int64_t leaders = 0, followers = 0;
        bool clustering = true;
        for (int64_t i = 0; i < n_low; ++i) {
            if (placed[i]) continue;
            placed[i] = 1;
            cluster_first.push_back((int32_t)order.size());
            order.push_back((int32_t)i);
            if (!clustering) continue;
            const int32_t g = low_groups[i];
            const int64_t li = v->blk_ptr[g + 1] - v->blk_ptr[g];
            hit.clear();
            for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b) {
                const int32_t blk = v->blk_col[b];
                int64_t &f = first[blk];
                while (f < inv_ptr[blk + 1] && inv[f] <= i) ++f;
                for (int64_t e = f; e < inv_ptr[blk + 1]; ++e) {
                    const int32_t j = inv[e];
                    if (!placed[j] && cnt[j]++ == 0) hit.push_back(j);
                }
            }
            // the followers join in rising order; only they are sorted (the candidates are thousands per
            // leader on an unstructured matrix, the followers few)
            size_t n_pass = 0;
            for (const int32_t j : hit) {
                const int32_t gj = low_groups[j];
                const int64_t I = cnt[j], lj = v->blk_ptr[gj + 1] - v->blk_ptr[gj];
                cnt[j] = 0;
                if (2 * I >= std::min(li, lj)) hit[n_pass++] = j;
            }
            std::sort(hit.begin(), hit.begin() + (std::ptrdiff_t)n_pass);
            for (size_t k = 0; k < n_pass; ++k) { placed[hit[k]] = 1; order.push_back(hit[k]); ++followers; }
            if (++leaders == 512 && followers < 64) clustering = false;
        }
        // A cluster of two slabs' worth of rows or more begins and ends on a slab boundary (the list is
        // padded with -1: positions without a row), so that no slab mixes it with its neighbours.  And no
        // slab gathers more than kSlabMaxCols columns if it can be helped: a group whose columns would
        // take the slab beyond that starts a new slab (unrelated rows add up their columns, and the
        // longest slab of a launch, one workgroup per column tile, is what the launch waits for).
        cluster_first.push_back((int32_t)order.size());
        std::vector<int64_t> col_slab((size_t)std::max<int64_t>(csr->n_cols, 1), -1);   // slab that last counted the column
        int64_t slab_id = 0, slab_cols = 0;
        auto pad_to_slab = [&]() {
            while (v->prow.size() % kSlabRows != 0) v->prow.push_back(-1);
            ++slab_id;
            slab_cols = 0;
        };
        for (size_t c = 0; c + 1 < cluster_first.size(); ++c) {
            int64_t rows = 0;
            for (int32_t o = cluster_first[c]; o < cluster_first[c + 1]; ++o)
                rows += row_groups[low_groups[order[o]] + 1] - row_groups[low_groups[order[o]]];
            const bool align = rows >= 2 * kSlabRows;
            if (align) pad_to_slab();
            for (int32_t o = cluster_first[c]; o < cluster_first[c + 1]; ++o) {
                const int32_t g = low_groups[order[o]];
                int64_t fresh = 0;                      // columns of the group the current slab does not hold yet
                for (int64_t q = row_groups[g]; q < row_groups[g + 1]; ++q)
                    for (int64_t p = csr->row_ptr[perm[q]]; p < csr->row_ptr[perm[q] + 1]; ++p)
                        fresh += col_slab[csr->col_idx[p]] != slab_id;
                if (v->prow.size() % kSlabRows != 0 && slab_cols + fresh > kSlabMaxCols) pad_to_slab();
                v->group_prow[g] = (int32_t)v->prow.size();
                for (int64_t q = row_groups[g]; q < row_groups[g + 1]; ++q) {
                    if (v->prow.size() % kSlabRows == 0) { ++slab_id; slab_cols = 0; }      // a new slab begins here
                    for (int64_t p = csr->row_ptr[perm[q]]; p < csr->row_ptr[perm[q] + 1]; ++p)
                        if (col_slab[csr->col_idx[p]] != slab_id) { col_slab[csr->col_idx[p]] = slab_id; ++slab_cols; }
                    v->prow.push_back(perm[q]);
                }
            }
            if (align) pad_to_slab();
        }
    }

    // pass 2: the low rows, in chunks of 8 slabs.
    const int64_t n_prows = (int64_t)v->prow.size();
    std::vector<int32_t> prow_group((size_t)n_prows, -1);     // -1: a padding position
    for (int32_t g = 0; g < G; ++g)
        if (v->group_prow[g] >= 0)
            for (int64_t i = 0; i < row_groups[g + 1] - row_groups[g]; ++i) prow_group[v->group_prow[g] + i] = g;
    const int R = kPanelSlabs;
    v->panel_slabs = n_prows > 0 ? R : 0;
    const int max_frags = kPanelMaxFrags;
    const int64_t panel_rows = (int64_t)R * kSlabRows;
    const int64_t n_panels = (n_prows + panel_rows - 1) / panel_rows;       // chunks
    v->p_union_ptr.assign(1, 0);
    std::vector<uint32_t> blk_mask;            // per union block: slabs that store it
    std::vector<int64_t> frag_of;              // [logical step][slab] -> fragment ordinal in the panel, -1
    std::vector<int64_t> fill_dst, fill_src;   // low-row values: position in vals <- position in csr->vals
    std::vector<int32_t> pos_of_col((size_t)std::max<int64_t>(csr->n_cols, 1), -1);
    std::vector<int32_t> cols;
    v->chunk_gather.assign((size_t)n_panels, 0);
    v->chunk_index.assign((size_t)n_panels, 0);
    int64_t g_ks = 0;                          // K-steps of the gathered tiles so far

    auto emit_panel = [&](int64_t pn) -> int {
        v->chunk_index[pn] = (int32_t)v->panels.size();
        const int64_t i0 = pn * panel_rows, i1 = std::min(n_prows, i0 + panel_rows);
        // union of blocks, and per block the slabs that hold it
        blocks.clear();
        for (int64_t i = i0; i < i1; ++i) {
            const int32_t g = prow_group[i];
            if (g < 0 || (i > i0 && prow_group[i - 1] == g)) continue;
            for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b)
                if (pos_of_block[v->blk_col[b]] < 0) { pos_of_block[v->blk_col[b]] = 0; blocks.push_back(v->blk_col[b]); }
        }
        std::sort(blocks.begin(), blocks.end());
        const int64_t nu = (int64_t)blocks.size();
        for (int64_t u = 0; u < nu; ++u) pos_of_block[blocks[u]] = (int32_t)u;
        blk_mask.assign((size_t)nu, 0u);
        for (int64_t i = i0; i < i1; ++i) {
            const int32_t g = prow_group[i];
            if (g < 0) continue;
            const uint32_t bit = 1u << ((i - i0) / kSlabRows);
            for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b) blk_mask[pos_of_block[v->blk_col[b]]] |= bit;
        }
        v->p_union.insert(v->p_union.end(), blocks.begin(), blocks.end());
        v->p_union_ptr.push_back((int64_t)v->p_union.size());

        PanelDesc pd;
        pd.ks_begin = (int32_t)v->pk_mask.size();
        pd.a_off = a_units;
        pd.row_begin = (int32_t)i0;
        pd.n_rows = (int32_t)(i1 - i0);
        pd.pad = 0;
        pd.meta_begin = (int32_t)(v->pk_meta.size() / (size_t)(1 + per_step));
        const int64_t Ku = nu * col_block;
        const int64_t T = (Ku + kStepK - 1) / kStepK;
        frag_of.assign((size_t)(T * R), -1);
        int64_t n_frags = 0;
        for (int64_t t = 0; t < T; ++t) {
            uint32_t m = 0;
            for (int64_t u = (t * kStepK) / col_block; u <= std::min(nu - 1, (t * kStepK + kStepK - 1) / col_block); ++u) m |= blk_mask[u];
            // a physical K-step carries at most max_frags fragments: split the rest into repeats
            while (m != 0) {
                uint32_t part = 0;
                int cnt = 0;
                for (int s = 0; s < R && cnt < max_frags; ++s)
                    if (m >> s & 1) { part |= 1u << s; frag_of[(size_t)(t * R + s)] = n_frags + cnt; ++cnt; }
                m &= ~part;
                v->pk_mask.push_back(part);
                v->pk_logical.push_back((int32_t)t);
                v->pk_frag.push_back(n_frags);
                n_frags += cnt;
                for (int e = 0; e < per_step; ++e) {
                    const int64_t k = t * kStepK + (int64_t)e * gran;
                    v->pk_row.push_back(k < Ku ? (int32_t)((int64_t)blocks[k / col_block] * col_block + k % col_block) : -1);
                }
            }
        }
        pd.n_ks = (int32_t)v->pk_mask.size() - pd.ks_begin;
        if ((int64_t)v->pk_mask.size() > INT32_MAX / 64) return VBR_EINVAL;
        // the device's K-step stream: one record per physical step, then the look-ahead padding
        for (int64_t ph = pd.ks_begin; ph < pd.ks_begin + pd.n_ks + (pd.n_ks > 0 ? kPanelMetaPad : 0); ++ph) {
            const int64_t src_ph = std::min<int64_t>(ph, pd.ks_begin + pd.n_ks - 1);
            v->pk_meta.push_back(ph < pd.ks_begin + pd.n_ks ? (int32_t)v->pk_mask[ph] : 0);
            for (int e = 0; e < per_step; ++e) v->pk_meta.push_back(v->pk_row[(size_t)src_ph * per_step + e]);
        }
        // values: one full 16 x 32 fragment per (physical step, present slab).  Only the target
        // position of every entry is noted here; the value array is allocated once, at its final
        // size, after the last panel.
        for (int64_t i = i0; i < i1; ++i) {
            const int64_t r = v->prow[i];
            if (r < 0) continue;
            const int s = (int)((i - i0) / kSlabRows), mrow = (int)((i - i0) % kSlabRows);
            for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p) {
                const int64_t c = csr->col_idx[p];
                const int64_t k = (int64_t)pos_of_block[c / col_block] * col_block + c % col_block;
                fill_dst.push_back(a_units * 8 + frag_of[(size_t)((k / kStepK) * R + s)] * kFragElems +
                                   frag_index(mrow, (int)(k % kStepK), kSlabRows));
                fill_src.push_back(p);
            }
        }
        a_units += n_frags * (kFragElems / 8);
        for (int64_t u = 0; u < nu; ++u) pos_of_block[blocks[u]] = -1;
        v->panels.push_back(pd);
        return VBR_OK;
    };

    // A column-gathered tile over the positions [s0, s1) of the low-row list (up to 8 slabs): its K
    // dimension is the ascending list of the columns its rows touch, cut into K-steps of 32.
    auto emit_gather_tile = [&](int64_t s0, int64_t s1, int32_t group_code) -> int {
        cols.clear();
        for (int64_t i = s0; i < s1; ++i) {
            const int64_t r = v->prow[i];
            if (r < 0) continue;
            for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p)
                if (pos_of_col[csr->col_idx[p]] < 0) { pos_of_col[csr->col_idx[p]] = 0; cols.push_back(csr->col_idx[p]); }
        }
        std::sort(cols.begin(), cols.end());
        for (size_t k = 0; k < cols.size(); ++k) pos_of_col[cols[k]] = (int32_t)k;
        const int64_t n_ks = ((int64_t)cols.size() + kStepK - 1) / kStepK;
        if (g_ks + n_ks > INT32_MAX / 64) return VBR_EINVAL;
        TileDesc td;
        td.ks_begin = (int32_t)g_ks;
        td.n_ks = (int32_t)n_ks;
        td.a_off = a_units;
        td.row_begin = (int32_t)s0;
        td.n_rows = (int32_t)(s1 - s0);
        td.n_slabs = (int32_t)((s1 - s0 + kSlabRows - 1) / kSlabRows);
        td.group = group_code;
        const int64_t stride = tile_kstep_stride(td.n_rows, td.n_slabs);
        const int rows_last = td.n_rows - (td.n_slabs - 1) * kSlabRows;
        for (int64_t i = s0; i < s1; ++i) {
            const int64_t r = v->prow[i];
            if (r < 0) continue;
            const int slab = (int)((i - s0) / kSlabRows), m = (int)((i - s0) % kSlabRows);
            const int rows = slab == td.n_slabs - 1 ? rows_last : kSlabRows;
            for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p) {
                const int64_t k = pos_of_col[csr->col_idx[p]];
                fill_dst.push_back(a_units * 8 + (k / kStepK) * stride + (int64_t)slab * kFragElems + frag_index(m, (int)(k % kStepK), rows));
                fill_src.push_back(p);
            }
        }
        for (int64_t k = 0; k < n_ks * kStepK; ++k) v->gcol.push_back(k < (int64_t)cols.size() ? cols[k] : -1);
        for (const int32_t c : cols) pos_of_col[c] = -1;
        a_units += n_ks * stride / 8;
        g_ks += n_ks;
        v->gtiles.push_back(td);
        return VBR_OK;
    };
    // the slabs of a chunk of low rows as column-gathered tiles
    auto emit_gather = [&](int64_t pn) -> int {
        const int64_t i0 = pn * panel_rows, i1 = std::min(n_prows, i0 + panel_rows);
        v->chunk_gather[pn] = 1;
        v->chunk_index[pn] = (int32_t)v->gtiles.size();
        for (int64_t s0 = i0; s0 < i1; s0 += kSlabRows) {
            const int rc = emit_gather_tile(s0, std::min(i1, s0 + kSlabRows), -1);
            if (rc != VBR_OK) return rc;
        }
        return VBR_OK;
    };

    for (int64_t pn = 0; pn < n_panels; ++pn) {
        const int64_t i0 = pn * panel_rows, i1 = std::min(n_prows, i0 + panel_rows);
        bool gather = !panels_on;
        if (!gather) {
            // loads of the two packings for this chunk (per 256 columns of C)
            blocks.clear();
            int64_t cost_gather = 0;
            for (int64_t s0 = i0; s0 < i1; s0 += kSlabRows) {
                cols.clear();
                for (int64_t i = s0; i < std::min(i1, s0 + kSlabRows); ++i) {
                    const int64_t r = v->prow[i];
                    if (r < 0) continue;
                    for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p) {
                        const int32_t c = csr->col_idx[p];
                        if (pos_of_col[c] < 0) { pos_of_col[c] = 0; cols.push_back(c); }
                        const int32_t j = c / col_block;
                        if (pos_of_block[j] < 0) { pos_of_block[j] = 0; blocks.push_back(j); }
                    }
                }
                for (const int32_t c : cols) pos_of_col[c] = -1;
                cost_gather += (((int64_t)cols.size() + kStepK - 1) / kStepK) * kTileStepCost;
            }
            for (const int32_t j : blocks) pos_of_block[j] = -1;
            const int64_t cost_panel = (((int64_t)blocks.size() * col_block + kStepK - 1) / kStepK) * kPanelStepCost;
            gather = cost_gather < cost_panel;
        }
        const int rc = gather ? emit_gather(pn) : emit_panel(pn);
        if (rc != VBR_OK) return rc;
    }

    // the tiles of the tall groups that gather single columns: their rows follow the low rows in the row list
    v->group_gt_first.assign((size_t)std::max<int32_t>(G, 1), -1);
    for (const int32_t g : tall_gathered) {
        const int64_t r0 = row_groups[g], h = row_groups[g + 1] - r0;
        const int64_t slabs = (h + kSlabRows - 1) / kSlabRows;
        const int64_t nt = (slabs + kMaxSlabs - 1) / kMaxSlabs;
        v->group_gt_first[g] = (int32_t)v->gtiles.size();
        // A tile whose rows touch more than kTileMaxGatherSteps K-steps' worth of columns is cut in two
        // (at a slab boundary; a single slab into two partial ones): fewer rows share each gathered B row,
        // but the longest tile of a launch, one workgroup per column tile, is what the launch waits for.
        struct Range { int64_t q0, q1; };
        std::vector<Range> todo;
        int64_t row = 0;
        for (int64_t t = 0; t < nt; ++t) {
            const int64_t s = slabs / nt + (t < slabs % nt ? 1 : 0);
            const int64_t n_rows = std::min<int64_t>(s * kSlabRows, h - row);
            todo.push_back(Range{r0 + row, r0 + row + n_rows});
            row += n_rows;
        }
        for (size_t i = 0; i < todo.size(); ++i) {          // in row order: a cut tile is replaced by its halves in place
            const Range rg_ = todo[i];
            const int64_t n_rows = rg_.q1 - rg_.q0, n_slabs = (n_rows + kSlabRows - 1) / kSlabRows;
            if (n_rows > 1) {
                ++col_stamp_id;
                int64_t cols_t = 0;
                for (int64_t q = rg_.q0; q < rg_.q1; ++q)
                    for (int64_t p = csr->row_ptr[perm[q]]; p < csr->row_ptr[perm[q] + 1]; ++p)
                        if (col_stamp[csr->col_idx[p]] != col_stamp_id) { col_stamp[csr->col_idx[p]] = col_stamp_id; ++cols_t; }
                if (cols_t > kTileMaxGatherSteps * kStepK) {
                    const int64_t mid = n_slabs > 1 ? rg_.q0 + (n_slabs / 2) * kSlabRows : rg_.q0 + n_rows / 2;
                    todo[i] = Range{rg_.q0, mid};
                    todo.insert(todo.begin() + (int64_t)i + 1, Range{mid, rg_.q1});
                    --i;
                    continue;
                }
            }
            const int64_t s0 = (int64_t)v->prow.size();
            for (int64_t q = rg_.q0; q < rg_.q1; ++q) v->prow.push_back(perm[q]);
            const int rc = emit_gather_tile(s0, s0 + n_rows, -2 - g);
            if (rc != VBR_OK) return rc;
        }
    }

    // pass 3: the values.  One allocation: tiles' fragments, panels' fragments, and one fragment
    // of zeros behind the last value (loads that run past a panel's data stay inside, and the
    // panel kernel's filler loads read it).
    v->vals.assign((size_t)a_units * 8 + kFragElems, 0);
    const uint16_t *src = static_cast<const uint16_t *>(csr->vals);
    for (size_t e = 0; e < fill_dst.size(); ++e) v->vals[(size_t)fill_dst[e]] = src[fill_src[e]];
    for (int32_t g = 0; g < G; ++g) {
        if (v->group_first_tile[g] == v->group_first_tile[g + 1]) continue;
        for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b) pos_of_block[v->blk_col[b]] = (int32_t)(b - v->blk_ptr[g]);
        for (int64_t t = v->group_first_tile[g]; t < v->group_first_tile[g + 1]; ++t) {
            const TileDesc &td = tiles[t];
            const int64_t stride = tile_kstep_stride(td.n_rows, td.n_slabs);
            const int rows_last = td.n_rows - (td.n_slabs - 1) * kSlabRows;
            uint16_t *dst = &v->vals[(size_t)td.a_off * 8];
            for (int32_t rr = 0; rr < td.n_rows; ++rr) {
                const int64_t r = perm[td.row_begin + rr];
                const int slab = rr / kSlabRows, m = rr % kSlabRows;
                const int rows = slab == td.n_slabs - 1 ? rows_last : kSlabRows;
                for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p) {
                    const int64_t c = csr->col_idx[p];
                    const int64_t k = (int64_t)pos_of_block[c / col_block] * col_block + c % col_block;
                    dst[(k / kStepK) * stride + (int64_t)slab * kFragElems + frag_index(m, (int)(k % kStepK), rows)] = src[p];
                }
            }
        }
        for (int64_t b = v->blk_ptr[g]; b < v->blk_ptr[g + 1]; ++b) pos_of_block[v->blk_col[b]] = -1;
    }

    // schedule: tiles grouped by slab class (one kernel instantiation each), heaviest first
    const int64_t NT = (int64_t)tiles.size();
    std::vector<int32_t> order(NT);
    for (int64_t i = 0; i < NT; ++i) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        const int ca = slab_class(tiles[a].n_slabs), cb = slab_class(tiles[b].n_slabs);
        if (ca != cb) return ca < cb;
        const int64_t wa = (int64_t)tiles[a].n_ks * tiles[a].n_slabs, wb = (int64_t)tiles[b].n_ks * tiles[b].n_slabs;
        return wa > wb;
    });
    v->tiles.resize(NT);
    v->tile_of_group_order.resize(NT);
    for (int c = 0; c < 5; ++c) v->class_begin[c] = 0;
    for (int64_t i = 0; i < NT; ++i) {
        v->tiles[i] = tiles[order[i]];
        v->tile_of_group_order[order[i]] = (int32_t)i;
        v->class_begin[slab_class(tiles[order[i]].n_slabs) + 1]++;
    }
    for (int c = 0; c < 4; ++c) v->class_begin[c + 1] += v->class_begin[c];

    // the gathered tiles as the device holds them: by slab class, heaviest first
    {
        const int64_t NG = (int64_t)v->gtiles.size();
        std::vector<int32_t> gorder(NG);
        for (int64_t i = 0; i < NG; ++i) gorder[i] = (int32_t)i;
        std::stable_sort(gorder.begin(), gorder.end(), [&](int32_t a, int32_t b) {
            const int ca = slab_class(v->gtiles[a].n_slabs), cb = slab_class(v->gtiles[b].n_slabs);
            if (ca != cb) return ca < cb;
            return (int64_t)v->gtiles[a].n_ks * v->gtiles[a].n_slabs > (int64_t)v->gtiles[b].n_ks * v->gtiles[b].n_slabs;
        });
        v->gtiles_dev.resize(NG);
        for (int c = 0; c < 5; ++c) v->gclass_begin[c] = 0;
        for (int64_t i = 0; i < NG; ++i) {
            v->gtiles_dev[i] = v->gtiles[gorder[i]];
            v->gclass_begin[slab_class(v->gtiles[gorder[i]].n_slabs) + 1]++;
        }
        for (int c = 0; c < 4; ++c) v->gclass_begin[c + 1] += v->gclass_begin[c];
    }

    DeviceLayout &L = v->lay;
    L.zeros_off = 0;                   // 256 zero bytes the kernel reads for padding
    L.tiles_off = 256;
    L.krow_off = align_up(L.tiles_off + (NT + (int64_t)v->gtiles.size()) * (int64_t)sizeof(TileDesc), 256);
    L.perm_off = align_up(L.krow_off + (int64_t)v->krow.size() * 4, 256);
    L.panels_off = align_up(L.perm_off + M * 4, 256);
    L.pk_meta_off = align_up(L.panels_off + (int64_t)v->panels.size() * (int64_t)sizeof(PanelDesc), 256);
    L.prow_off = align_up(L.pk_meta_off + (int64_t)v->pk_meta.size() * 4, 256);
    L.gcol_off = align_up(L.prow_off + (int64_t)v->prow.size() * 4, 256);
    L.vals_off = align_up(L.gcol_off + (int64_t)v->gcol.size() * 4, 256);
    L.total = std::max<int64_t>(256, align_up(L.vals_off + (int64_t)v->vals.size() * 2, 256));
    return VBR_OK;
}

}  // namespace
}  // namespace vbrk

extern "C" int vbr_build(const vbr_csr_t *csr, const int32_t *perm, const int32_t *row_groups,
                         int32_t n_groups, int32_t col_block, vbr_t **out)
{
    if (!csr || !out || n_groups < 0 || col_block <= 0) return VBR_EINVAL;
    *out = nullptr;
    int rc = vbrk::validate_csr(csr, true);
    if (rc != VBR_OK) return rc;
    if (csr->n_cols % col_block != 0) return VBR_EINVAL;
    const int64_t M = csr->n_rows;
    if ((M > 0 && (!perm || !row_groups)) || !row_groups) return VBR_EINVAL;
    if (n_groups > M || (M > 0 && n_groups == 0)) return VBR_EINVAL;
    if (row_groups[0] != 0 || row_groups[n_groups] != M) return VBR_EINVAL;
    for (int32_t g = 0; g < n_groups; ++g)
        if (row_groups[g + 1] <= row_groups[g]) return VBR_EINVAL;
    try {
        std::vector<uint8_t> seen((size_t)M, 0);
        for (int64_t i = 0; i < M; ++i) {
            if (perm[i] < 0 || perm[i] >= M || seen[perm[i]]) return VBR_EINVAL;   // not a bijection
            seen[perm[i]] = 1;
        }
        vbr *v = new vbr();
        rc = vbrk::build_impl(csr, perm, row_groups, n_groups, col_block, v);
        if (rc != VBR_OK) { delete v; return rc; }
        *out = v;
        return VBR_OK;
    } catch (const std::bad_alloc &) {
        return VBR_ENOMEM;
    } catch (...) {
        return VBR_EINVAL;
    }
}

extern "C" int vbr_get_index(const vbr_t *v, const int32_t **row_groups, const int32_t **perm,
                             const int64_t **blk_ptr, const int32_t **blk_col, const int64_t **blk_off,
                             int64_t *n_groups, int64_t *n_blocks, int64_t *stored_elems)
{
    if (!v) return VBR_EINVAL;
    if (row_groups) *row_groups = v->row_groups.data();
    if (perm) *perm = v->perm.data();
    if (blk_ptr) *blk_ptr = v->blk_ptr.data();
    if (blk_col) *blk_col = v->blk_col.data();
    if (blk_off) *blk_off = v->blk_off.data();
    if (n_groups) *n_groups = v->n_groups;
    if (n_blocks) *n_blocks = (int64_t)v->blk_col.size();
    if (stored_elems) *stored_elems = v->blk_off.back();
    return VBR_OK;
}

extern "C" int vbr_unpack_block(const vbr_t *v, int64_t blk, void *dst_)
{
    using namespace vbrk;
    if (!v || !dst_ || blk < 0 || blk >= (int64_t)v->blk_col.size()) return VBR_EINVAL;
    const int32_t g = (int32_t)(std::upper_bound(v->blk_ptr.begin(), v->blk_ptr.end(), blk) - v->blk_ptr.begin() - 1);
    const int64_t pos = blk - v->blk_ptr[g];
    const int64_t cb = v->col_block;
    uint16_t *dst = static_cast<uint16_t *>(dst_);
    if (v->group_prow[g] >= 0) {
        // low group: its rows sit in one chunk of the low rows (or two), packed as a panel or as
        // column-gathered tiles
        const int64_t h = v->row_groups[g + 1] - v->row_groups[g];
        const int R = v->panel_slabs;
        const int64_t panel_rows = (int64_t)R * kSlabRows;
        for (int64_t i = 0; i < h; ++i) {
            const int64_t pi = v->group_prow[g] + i;
            const int64_t pn = pi / panel_rows;
            if (v->chunk_gather[pn]) {
                // the slab's column list is ascending up to its padding: look every column of the block up
                const TileDesc &td = v->gtiles[v->chunk_index[pn] + (pi - pn * panel_rows) / kSlabRows];
                const int m = (int)(pi - td.row_begin);
                const int32_t *cb0 = &v->gcol[(size_t)td.ks_begin * kStepK], *ce = cb0 + (size_t)td.n_ks * kStepK;
                while (ce > cb0 && ce[-1] < 0) --ce;
                const int64_t stride = tile_kstep_stride(td.n_rows, 1);
                for (int64_t c = 0; c < cb; ++c) {
                    const int32_t col = (int32_t)((int64_t)v->blk_col[blk] * cb + c);
                    const int32_t *it = std::lower_bound(cb0, ce, col);
                    if (it == ce || *it != col) { dst[i * cb + c] = 0; continue; }      // fill-in: not stored
                    const int64_t k = it - cb0;
                    dst[i * cb + c] = v->vals[(size_t)td.a_off * 8 + (size_t)((k / kStepK) * stride) + frag_index(m, (int)(k % kStepK), td.n_rows)];
                }
                continue;
            }
            const int64_t pidx = v->chunk_index[pn];
            const PanelDesc &pd = v->panels[pidx];
            const int s = (int)((pi - pd.row_begin) / kSlabRows), m = (int)((pi - pd.row_begin) % kSlabRows);
            const int32_t *ub = &v->p_union[v->p_union_ptr[pidx]], *ue = &v->p_union[0] + v->p_union_ptr[pidx + 1];
            const int64_t u = std::lower_bound(ub, ue, v->blk_col[blk]) - ub;
            for (int64_t c = 0; c < cb; ++c) {
                const int64_t k = u * cb + c;
                const int32_t t = (int32_t)(k / kStepK);
                // physical steps of logical step t are consecutive; take the one that carries slab s
                const int32_t *lb = &v->pk_logical[pd.ks_begin], *le = lb + pd.n_ks;
                int64_t ph = pd.ks_begin + (std::lower_bound(lb, le, t) - lb);
                while (!(v->pk_mask[ph] >> s & 1)) ++ph;
                const int rank = __builtin_popcount(v->pk_mask[ph] & ((1u << s) - 1u));
                dst[i * cb + c] = v->vals[(size_t)pd.a_off * 8 + (size_t)(v->pk_frag[ph] + rank) * kFragElems +
                                          frag_index(m, (int)(k % kStepK), kSlabRows)];
            }
        }
        return VBR_OK;
    }
    if (v->group_gt_first[g] >= 0) {
        // tall group whose tiles gather single columns: the tiles follow each other, each with its own column list
        const int64_t h = v->row_groups[g + 1] - v->row_groups[g];
        int64_t row = 0;
        for (int64_t t = v->group_gt_first[g]; row < h; ++t) {
            const TileDesc &td = v->gtiles[t];
            const int32_t *cb0 = &v->gcol[(size_t)td.ks_begin * kStepK], *ce = cb0 + (size_t)td.n_ks * kStepK;
            while (ce > cb0 && ce[-1] < 0) --ce;
            const int64_t stride = tile_kstep_stride(td.n_rows, td.n_slabs);
            const int rows_last = td.n_rows - (td.n_slabs - 1) * kSlabRows;
            for (int32_t rr = 0; rr < td.n_rows; ++rr, ++row) {
                const int slab = rr / kSlabRows, m = rr % kSlabRows;
                const int rows = slab == td.n_slabs - 1 ? rows_last : kSlabRows;
                for (int64_t c = 0; c < cb; ++c) {
                    const int32_t col = (int32_t)((int64_t)v->blk_col[blk] * cb + c);
                    const int32_t *it = std::lower_bound(cb0, ce, col);
                    if (it == ce || *it != col) { dst[row * cb + c] = 0; continue; }          // fill-in: not stored
                    const int64_t k = it - cb0;
                    dst[row * cb + c] = v->vals[(size_t)td.a_off * 8 + (size_t)((k / kStepK) * stride) + (size_t)slab * kFragElems +
                                                frag_index(m, (int)(k % kStepK), rows)];
                }
            }
        }
        return VBR_OK;
    }
    int64_t row = 0;
    for (int64_t t = v->group_first_tile[g]; t < v->group_first_tile[g + 1]; ++t) {
        const TileDesc &td = v->tiles[v->tile_of_group_order[t]];
        const int64_t stride = tile_kstep_stride(td.n_rows, td.n_slabs);
        const int rows_last = td.n_rows - (td.n_slabs - 1) * kSlabRows;
        const uint16_t *src = &v->vals[(size_t)td.a_off * 8];
        for (int32_t rr = 0; rr < td.n_rows; ++rr, ++row) {
            const int slab = rr / kSlabRows, m = rr % kSlabRows;
            const int rows = slab == td.n_slabs - 1 ? rows_last : kSlabRows;
            for (int64_t c = 0; c < cb; ++c) {
                const int64_t k = pos * cb + c;
                dst[row * cb + c] = src[(k / kStepK) * stride + (int64_t)slab * kFragElems + frag_index(m, (int)(k % kStepK), rows)];
            }
        }
    }
    return VBR_OK;
}

// Everything the kernels index with, checked against the sizes of what they index into: a wrong
// entry here would be a device access out of bounds, so the check is plain and complete.
extern "C" int vbr_audit(const vbr_t *v)
{
    using namespace vbrk;
    if (!v) return VBR_EINVAL;
    const int64_t M = v->n_rows, K = v->n_cols;
    const int gran = 1 << v->lg_gran, per_step = kStepK >> v->lg_gran;
    const int64_t n_vals = (int64_t)v->vals.size();
    if (n_vals < kFragElems || (int64_t)v->perm.size() != M) return VBR_EINVAL;
    for (int64_t i = 0; i < M; ++i)
        if (v->perm[i] < 0 || v->perm[i] >= M) return VBR_EINVAL;
    for (const int32_t e : v->krow)
        if (e < -1 || (e >= 0 && (int64_t)e + gran > K)) return VBR_EINVAL;
    if ((int64_t)v->krow.size() % per_step != 0) return VBR_EINVAL;
    const int64_t total_ks = (int64_t)v->krow.size() / per_step;
    if (v->class_begin[0] != 0 || v->class_begin[4] != (int32_t)v->tiles.size()) return VBR_EINVAL;
    for (int c = 0; c < 4; ++c) {
        if (v->class_begin[c + 1] < v->class_begin[c]) return VBR_EINVAL;
        for (int32_t t = v->class_begin[c]; t < v->class_begin[c + 1]; ++t) {
            const TileDesc &td = v->tiles[t];
            if (td.n_rows < 1 || td.n_slabs != (td.n_rows + kSlabRows - 1) / kSlabRows || td.n_slabs > kMaxSlabs) return VBR_EINVAL;
            if (slab_class(td.n_slabs) != c) return VBR_EINVAL;
            if (td.row_begin < 0 || (int64_t)td.row_begin + td.n_rows > M) return VBR_EINVAL;
            if (td.n_ks < 0 || td.ks_begin < 0 || (int64_t)td.ks_begin + td.n_ks > total_ks) return VBR_EINVAL;
            // the fragments of all its K-steps lie inside the values (the zero fragment at the end excluded)
            if (td.a_off < 0 || td.a_off * 8 + (int64_t)td.n_ks * tile_kstep_stride(td.n_rows, td.n_slabs) > n_vals - kFragElems) return VBR_EINVAL;
        }
    }
    const int rec = 1 + per_step;
    if ((int64_t)v->pk_meta.size() % rec != 0) return VBR_EINVAL;
    const int64_t n_rec = (int64_t)v->pk_meta.size() / rec;
    for (int64_t r = 0; r < n_rec; ++r) {
        if ((uint32_t)v->pk_meta[r * rec] >> kPanelSlabs) return VBR_EINVAL;                 // mask of at most 8 slabs
        for (int e = 0; e < per_step; ++e) {
            const int32_t row = v->pk_meta[r * rec + 1 + e];
            if (row < -1 || (row >= 0 && (int64_t)row + gran > K)) return VBR_EINVAL;
        }
    }
    for (const int32_t r : v->prow)
        if (r < -1 || r >= M) return VBR_EINVAL;          // -1: a padding position, never stored
    for (const PanelDesc &pd : v->panels) {
        if (pd.n_rows < 1 || pd.n_rows > kPanelSlabs * kSlabRows) return VBR_EINVAL;
        if (pd.row_begin < 0 || (int64_t)pd.row_begin + pd.n_rows > (int64_t)v->prow.size()) return VBR_EINVAL;
        if (pd.n_ks < 0 || pd.meta_begin < 0) return VBR_EINVAL;
        if (pd.n_ks > 0 && (int64_t)pd.meta_begin + pd.n_ks + kPanelMetaPad > n_rec) return VBR_EINVAL;
        int64_t frags = 0;
        for (int32_t k = 0; k < pd.n_ks; ++k) {
            const uint32_t m = (uint32_t)v->pk_meta[((int64_t)pd.meta_begin + k) * rec];
            const int cnt = __builtin_popcount(m);
            if (cnt < 1 || cnt > kPanelMaxFrags) return VBR_EINVAL;
            frags += cnt;
        }
        for (int32_t k = pd.n_ks; k < pd.n_ks + (pd.n_ks > 0 ? kPanelMetaPad : 0); ++k)
            if (v->pk_meta[((int64_t)pd.meta_begin + k) * rec] != 0) return VBR_EINVAL;      // look-ahead records carry no slab
        if (pd.a_off < 0 || pd.a_off * 8 + frags * kFragElems > n_vals - kFragElems) return VBR_EINVAL;
    }
    if ((int64_t)v->gcol.size() % kStepK != 0) return VBR_EINVAL;
    for (const int32_t c : v->gcol)
        if (c < -1 || c >= K) return VBR_EINVAL;
    if (v->gtiles_dev.size() != v->gtiles.size() || v->gclass_begin[0] != 0 || v->gclass_begin[4] != (int32_t)v->gtiles.size()) return VBR_EINVAL;
    for (int c = 0; c < 4; ++c)
        for (int32_t t = v->gclass_begin[c]; t < v->gclass_begin[c + 1]; ++t)
            if (slab_class(v->gtiles_dev[t].n_slabs) != c) return VBR_EINVAL;
    for (const TileDesc &td : v->gtiles_dev) {
        if (td.n_rows < 1 || td.n_slabs != (td.n_rows + kSlabRows - 1) / kSlabRows || td.n_slabs > kMaxSlabs || td.group >= 0) return VBR_EINVAL;
        if (td.row_begin < 0 || (int64_t)td.row_begin + td.n_rows > (int64_t)v->prow.size()) return VBR_EINVAL;
        if (td.n_ks < 0 || td.ks_begin < 0 || ((int64_t)td.ks_begin + td.n_ks) * kStepK > (int64_t)v->gcol.size()) return VBR_EINVAL;
        if (td.a_off < 0 || td.a_off * 8 + (int64_t)td.n_ks * tile_kstep_stride(td.n_rows, td.n_slabs) > n_vals - kFragElems) return VBR_EINVAL;
    }
    for (size_t i = v->vals.size() - kFragElems; i < v->vals.size(); ++i)
        if (v->vals[i] != 0) return VBR_EINVAL;                                               // the zero fragment
    const DeviceLayout &L = v->lay;
    const int64_t ends[9] = {L.zeros_off + 256, L.tiles_off + (int64_t)(v->tiles.size() + v->gtiles.size()) * (int64_t)sizeof(TileDesc),
                              L.krow_off + (int64_t)v->krow.size() * 4, L.perm_off + M * 4,
                              L.panels_off + (int64_t)v->panels.size() * (int64_t)sizeof(PanelDesc),
                              L.pk_meta_off + (int64_t)v->pk_meta.size() * 4, L.prow_off + (int64_t)v->prow.size() * 4,
                              L.gcol_off + (int64_t)v->gcol.size() * 4, L.vals_off + n_vals * 2};
    const int64_t begins[9] = {L.zeros_off, L.tiles_off, L.krow_off, L.perm_off, L.panels_off, L.pk_meta_off, L.prow_off,
                               L.gcol_off, L.vals_off};
    for (int i = 0; i < 9; ++i) {
        if (begins[i] % 256 != 0 || ends[i] > L.total) return VBR_EINVAL;
        if (i + 1 < 9 && ends[i] > begins[i + 1]) return VBR_EINVAL;                         // sections in this order, disjoint
    }
    return VBR_OK;
}

extern "C" int64_t vbr_device_bytes(const vbr_t *v) { return v ? v->lay.total : 0; }

namespace vbrk {

// Workgroups of a launch over T row tiles and Q column tiles: workgroups are dealt to the L2
// domains round-robin, and a domain keeps to few column tiles (the kernels undo this map).
static int64_t grid_size(int64_t T, int64_t Q)
{
    if (Q >= kXcd) return (int64_t)kXcd * ((Q + kXcd - 1) / kXcd) * T;
    return (int64_t)kXcd * ((T + (kXcd / Q) - 1) / (kXcd / Q));
}

// The panels first (they are the long-running workgroups), then either one mixed launch (several
// slab classes, none of which alone gives every CU a couple of workgroups) or one launch per slab
// class present.
int plan_launches(const vbr *v, int64_t N, Launch out[VBR_MAX_LAUNCHES])
{
    int n = 0;
    const int64_t Qt = (N + kTileN - 1) / kTileN, Qp = (N + kPanelN - 1) / kPanelN;
    if (!v->panels.empty())
        out[n++] = Launch{VBR_LAUNCH_PANEL, 0, (int32_t)v->panels.size(), grid_size((int64_t)v->panels.size(), Qp)};
    // Eight tile classes, contiguous in the device's tile array: tiles of 1, 2, 3-4, 5-8 slabs that
    // gather whole column blocks, then the same four of tiles that gather single columns.  Several
    // classes that together do not give every CU a few workgroups share one launch of the mixed
    // kernel; otherwise every class present gets a launch of its own kernel, the gathered ones first.
    // (Mixing only the small classes of a large matrix was measured and lost: the mixed kernel holds
    // the LDS of the tallest class, and the tall tiles of the graph workload, few but with long block
    // lists, ran 20 % longer in it.)
    const int32_t T_blk = v->class_begin[4];
    int classes = 0;
    for (int c = 0; c < 4; ++c) classes += (v->class_begin[c + 1] > v->class_begin[c]) + (v->gclass_begin[c + 1] > v->gclass_begin[c]);
    const int64_t T_all = (int64_t)T_blk + v->gclass_begin[4];
    if (classes > 1 && T_all * Qt < 4096) {
        out[n++] = Launch{VBR_LAUNCH_TILE_MIXED, 0, (int32_t)T_all, grid_size(T_all, Qt)};
        return n;
    }
    for (int c = 0; c < 4; ++c) {
        const int32_t T = v->gclass_begin[c + 1] - v->gclass_begin[c];
        if (T > 0) out[n++] = Launch{VBR_LAUNCH_GATHER_1 + c, T_blk + v->gclass_begin[c], T, grid_size(T, Qt)};
    }
    for (int c = 0; c < 4; ++c) {
        const int32_t T = v->class_begin[c + 1] - v->class_begin[c];
        if (T > 0) out[n++] = Launch{VBR_LAUNCH_TILE_1 + c, v->class_begin[c], T, grid_size(T, Qt)};
    }
    return n;
}

}  // namespace vbrk

extern "C" int vbr_get_launches(const vbr_t *v, int64_t N, int32_t *n_launches, int32_t *kinds, int64_t *tiles, int64_t *workgroups)
{
    if (!v || !n_launches || N < 0) return VBR_EINVAL;
    vbrk::Launch plan[VBR_MAX_LAUNCHES];
    const int n = (N == 0 || v->n_rows == 0) ? 0 : vbrk::plan_launches(v, N, plan);
    *n_launches = n;
    for (int i = 0; i < n; ++i) {
        if (kinds) kinds[i] = plan[i].kind;
        if (tiles) tiles[i] = plan[i].n_tiles;
        if (workgroups) workgroups[i] = plan[i].grid;
    }
    return VBR_OK;
}

extern "C" int vbr_get_schedule(const vbr_t *v, int64_t *n_tiles, int64_t *n_ksteps, int64_t *packed_elems)
{
    if (!v) return VBR_EINVAL;
    if (n_tiles) *n_tiles = (int64_t)v->tiles.size() + (int64_t)v->panels.size() + (int64_t)v->gtiles.size();
    if (n_ksteps) *n_ksteps = v->ks_ptr.back() + (int64_t)v->pk_mask.size() + (int64_t)v->gcol.size() / vbrk::kStepK;
    if (packed_elems) *packed_elems = (int64_t)v->vals.size();
    return VBR_OK;
}

extern "C" int64_t vbr_get_tile_ksteps(const vbr_t *v, int64_t *out, int64_t cap)
{
    if (!v) return VBR_EINVAL;
    const int64_t n = (int64_t)(v->tiles.size() + v->gtiles.size() + v->panels.size());
    if (!out) return n;
    int64_t w = 0;
    for (const vbrk::TileDesc &t : v->tiles) { if (w < cap) out[w] = t.n_ks; ++w; }
    for (const vbrk::TileDesc &t : v->gtiles) { if (w < cap) out[w] = t.n_ks; ++w; }
    for (const vbrk::PanelDesc &t : v->panels) { if (w < cap) out[w] = t.n_ks; ++w; }
    return n;
}

extern "C" void vbr_free(vbr_t *v)
{
    if (v && v->release_dev) v->release_dev(v);
    delete v;
}

extern "C" const char *vbr_strerror(int code)
{
    switch (code) {
    case VBR_OK: return "ok";
    case VBR_EINVAL: return "invalid argument";
    case VBR_ENOMEM: return "out of host memory";
    case VBR_EHIP: return "HIP runtime error";
    case VBR_ESTATE: return "call out of order";
    case VBR_EUNSUPPORTED: return "unsupported input";
    default: return "unknown error";
    }
}
