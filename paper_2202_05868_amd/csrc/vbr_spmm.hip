// vbr_spmm on gfx950: C = A.B with A in packed VBR form (section 4.4.1 of the paper: every stored
// block is multiplied as a dense product on the matrix units).  Three kernels share one scheme: a
// workgroup owns some slabs of 16 rows and a column tile of C, walks a list of K-steps of 32 B rows,
// brings the gathered B rows and the A fragments into rings of LDS slots with 128-bit direct-to-LDS
// loads, and issues v_mfma_f32_16x16x32 on them.
//   tile kernel    up to 8 slabs of ONE row group x 256 columns; K-steps = the group's column blocks
//                  (one launch per slab class, or one mixed launch for small matrices)
//   gathered tiles the same kernel with K-steps = the single columns its rows touch: slabs cut from the
//                  rows of low groups, and tiles of tall groups whose blocks are mostly fill-in
//   panel kernel   8 slabs of low groups x 128 columns walking the union of their column blocks
// The launches of one call are independent and are spread over the handle's streams (launch_all).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstdint>
#include <type_traits>

#include "vbr_host.h"

namespace vbrk {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int code) { g_last_hip_error = code; }

namespace {

constexpr int kThreads = 256;          // 4 waves
constexpr int kWaveN = 64;             // C columns per wave: 4 MFMA tiles of 16
constexpr int kRowBytes = kTileN * 2;  // one staged B row in LDS: 512 bytes, no padding
constexpr int kPanelBytes = kStepK * kRowBytes;   // 16 KiB of B per K-step
constexpr int kFragBytes = kFragElems * 2;        // 1 KiB per A fragment

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;
typedef __attribute__((address_space(3))) short8v *lds_short8_ptr;
typedef __attribute__((address_space(3))) unsigned char *lds_u8_ptr;
typedef __attribute__((address_space(4))) const int32_t *const_i32_ptr;

struct Params {
    const TileDesc *tiles;    // tiles of this launch: one slab class, all of them, or the column-gathered ones
    const int32_t *krow;
    const int32_t *perm;
    const int32_t *gcol;      // column-gathered tiles: their column lists ...
    const int32_t *prow;      // ... and the list of the low rows their row positions refer to
    int32_t b_fits32;         // the rows of B the matrix can touch span less than 4 GiB: 32-bit offsets from B suffice
    const uint16_t *vals;
    const uint16_t *zeros;    // 256 zero bytes: source of padding rows, padding lanes and columns >= N
    const uint16_t *zfrag;    // 1 KiB of zeros behind the last fragment: padding rows of the column-gathered tiles
    const uint16_t *B;
    float *C;
    int64_t ldb, ldc;
    int32_t N;
    int32_t lg_gran;
    int32_t n_tiles;          // T
    int32_t n_ntiles;         // Q = ceil(N / 256)
};

template <int DT>
__device__ __forceinline__ float4v mfma16x16x32(short8v a, short8v b, float4v c)
{
    if constexpr (DT == VBR_F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, a), __builtin_bit_cast(bf16x8v, b), c, 0, 0, 0);
}

// 16 bytes per active lane from global memory straight into LDS, no register staging: lane l's
// data lands at lds_base + 16 l (lds_base wave-uniform, passed in M0).  The load is counted in
// vmcnt like any vector load; the compiler does not see it, so the waits are placed by hand.
// Every wave must issue the same, fixed number of these per K-step (never with an empty lane mask).
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr),
                 "s"((uint32_t)__builtin_amdgcn_readfirstlane(lds_base)) : "memory");
}
// same, address = wave-uniform base + zero-extended 32-bit lane offset
__device__ __forceinline__ void dma16_base(uint32_t voff, const void *base, uint32_t lds_base)
{
    // the base has to sit in scalar registers: say so explicitly (a no-op when it already does)
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    const uint64_t sbase = ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase),
                 "s"((uint32_t)__builtin_amdgcn_readfirstlane(lds_base)) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// S  = slabs the instantiation computes (tiles of the class have S/2 < n_slabs <= S; 1 for S = 1).
// NS = slots of the LDS ring of B panels: NS-1 K-steps of B loads are in flight per workgroup.
// DA = prefetch distance of the A fragments in K-steps (ring of DA+1 slots): A is streamed from
//      beyond L2 while B mostly hits in L2, and the loads of a wave retire in order.
// The loop is bound by the instructions a wave needs per K-step, so the common case (block width a
// multiple of 8, full column tile, no padding rows in the K-step) is kept to a handful of scalar
// instructions per 1 KiB load; everything else takes the general path.
// Workgroup -> (tile, column tile).  Workgroups are dealt to the 8 L2 domains round-robin; a
// domain keeps to few column tiles so that the B columns it gathers stay in its L2.
__device__ __forceinline__ bool map_workgroup(int T, int Q, int &tile, int &ntile)
{
    const int x = blockIdx.x & (kXcd - 1), j = blockIdx.x >> 3;
    if (Q >= kXcd) {
        ntile = x + kXcd * (j / T);
        tile = j % T;
        return ntile < Q;
    }
    ntile = x % Q;
    const int member = x / Q, members = (kXcd - ntile + Q - 1) / Q;
    tile = member + members * j;
    return tile < T;
}

template <int S, int NS, int DA>
constexpr int tile_lds_bytes() { return NS * kPanelBytes + (DA + 1) * S * kFragBytes; }

// GATHER: the tile is a slab of rows of low row groups whose K dimension is the list of the single
// COLUMNS its rows touch (one gather entry per B row, krow = that list) instead of whole column
// blocks: the fill-in columns of the blocks, which hold nothing but zeros, are never loaded.
template <int DT, int S, int NS, int DA, bool GATHER = false>
__device__ __forceinline__ void tile_body(const Params &p, const TileDesc td, const int ntile, unsigned char *smem)
{
    static_assert(NS >= 2 && DA >= NS - 1, "A must be requested before the B panel of its K-step");
    constexpr int NA = S >= 4 ? S / 4 : 1;      // A loads per wave per K-step
    constexpr int NAS = DA + 1;
    constexpr int kAStage = S * kFragBytes;
    constexpr int kBRing = NS * kPanelBytes;
    // loads younger than the last B load of K-step ks when the workgroup waits for it
    constexpr int kWait = (NS - 2) * 4 + (NS - 1) * NA;
    static_assert(kWait < 64, "vmcnt is a 6-bit counter");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n0 = ntile * kTileN;
    const lds_u8_ptr sm = (lds_u8_ptr)smem;
    const uint32_t smem_base = (uint32_t)(uintptr_t)sm;      // LDS byte address, for M0
    const char *zeros = reinterpret_cast<const char *>(p.zeros);
    const char *zpad = reinterpret_cast<const char *>(p.zfrag);
    const int n_ks = td.n_ks;
    const int q = lane >> 4, s16 = lane & 15;

    float4v acc[S][4];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[s][f] = float4v{0.f, 0.f, 0.f, 0.f};

    if (n_ks > 0) {
        // ---- B staging.  Per K-step a wave issues 4 loads; load i brings rows 8 wave + 2 i (lanes
        // 0-31) and 8 wave + 2 i + 1 (lanes 32-63) of the K-step, 512 bytes each, into 1 KiB of LDS.
        // LDS chunk c' (16 bytes) of row r holds global chunk c' ^ 2 (r % 8): the XOR spreads the
        // four rows one transposed read touches over distinct banks (rows are 512 bytes apart).
        const int half = lane >> 5;
        const int lg = p.lg_gran;
        const int gmask = (1 << lg) - 1;
        const const_i32_ptr krow = (const_i32_ptr)p.krow + (int64_t)td.ks_begin * (kStepK >> lg);
        const uint32_t ldb_bytes = (uint32_t)(p.ldb * 2);          // host checked: 32 rows of B span less than 2^32 bytes
        const char *Btile = reinterpret_cast<const char *>(p.B) + (int64_t)n0 * 2;
        // In the last column tile the chunks at or beyond column N do not exist: their lanes fetch
        // the tile's last existing chunk again (the C columns it would feed are never stored, and
        // columns do not mix), so the fast path serves partial tiles too.
        const bool tile_fast = lg >= 3;
        const int last_chunk = (p.N - n0 < kTileN ? p.N - n0 : kTileN) / 8 - 1;
        uint32_t b_col[4];       // byte offset of this lane's chunk from the tile's first column
        uint32_t b_lane[4];      // fast path: offset of this lane's 16 bytes from the first row of the wave's granule
        bool b_col_ok[4];
        uint32_t b_coff[4];      // column-gathered tiles: the same, clamped to the tile's last existing chunk
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int chunk = (lane & 31) ^ (2 * (2 * i + half));
            b_col[i] = chunk * 16;
            b_col_ok[i] = chunk <= last_chunk;
            b_coff[i] = (uint32_t)(chunk <= last_chunk ? chunk : last_chunk) * 16;      // past column N: the last chunk again
            b_lane[i] = (uint32_t)((8 * wave + 2 * i + half) & gmask) * ldb_bytes + (chunk <= last_chunk ? chunk : last_chunk) * 16;
        }

        // ---- A staging.  A direct-to-LDS load costs the CU the same whatever its lane mask, so a
        // fragment is always one load: with 1 or 2 slabs the waves take turns (K-step a: wave a % 4,
        // resp. waves 2 (a % 2) + slab), with 4 or 8 slabs every wave loads S/4 fragments per K-step.
        // Lanes of rows a partial last slab does not store are masked off (their LDS bytes keep
        // whatever they held: those fragment rows only feed C rows that are never stored); a wave
        // whose slab does not exist in this tile reloads the tile's last slab instead, so that the
        // loads per wave follow a fixed pattern and no load has an empty lane mask.
        const int rows_last = td.n_rows - (td.n_slabs - 1) * kSlabRows;
        const uint32_t a_stride_bytes = (uint32_t)(((td.n_slabs - 1) * kFragElems + rows_last * kStepK) * 2);
        const char *Abase = reinterpret_cast<const char *>(p.vals) + td.a_off * 16;
        int a_slab[NA];
        uint32_t a_lane[NA];     // byte offset of this lane's 16 bytes inside a K-step of the tile
        bool a_on[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if constexpr (S == 1) a_slab[i] = 0;
            else if constexpr (S == 2) a_slab[i] = wave & 1;
            else a_slab[i] = wave + 4 * i;
            if (a_slab[i] > td.n_slabs - 1) a_slab[i] = td.n_slabs - 1;
            const int rows = (a_slab[i] == td.n_slabs - 1) ? rows_last : kSlabRows;
            a_on[i] = s16 < rows;
            a_lane[i] = (uint32_t)((a_slab[i] * kFragElems + (q * rows + s16) * 8) * 2);
        }
        // does this wave load (part of) the A fragments of K-step a?
        auto a_turn = [&](int a) -> bool {
            if constexpr (S == 1) return (a & 3) == wave;
            else if constexpr (S == 2) return (a & 1) == (wave >> 1);
            else return true;
        };

        // First B row of the granule holding this wave's 8 rows (blocks at least 8 wide), for the
        // K-step whose B loads are issued next (rb0) and the one after (rb1): scalar loads, issued
        // two iterations ahead of their use.  Narrower blocks look their rows up per lane at issue
        // time instead, with an ordinary load the compiler waits for (slow, but rare and simple).
        // Column-gathered tiles: the 8 B rows of the wave, one list entry each, as 8 scalars.
        struct Rows { int r[GATHER ? 8 : 1]; };
        Rows rb0, rb1;
        rb0.r[0] = rb1.r[0] = -1;
        auto load_rows = [&](int ks) -> Rows {
            // past the end: reload the last K-step (never computed); wave-uniform, and said so, or the
            // lookups below become vector loads, which cost the load path as much as a load of B
            const int kc = __builtin_amdgcn_readfirstlane(ks < n_ks ? ks : n_ks - 1);
            Rows out;
            if constexpr (GATHER) {
                const const_i32_ptr src = (const_i32_ptr)p.gcol + ((int64_t)td.ks_begin + kc) * kStepK + 8 * wave;
#pragma unroll
                for (int j = 0; j < 8; ++j) out.r[j] = src[j];
            } else {
                out.r[0] = lg >= 3 ? krow[(kc * kStepK + 8 * wave) >> lg] : -1;
            }
            return out;
        };
        auto issue_b = [&](int ks, int slot) {
            const uint32_t sb = smem_base + slot * kPanelBytes + 8 * wave * kRowBytes;
            if constexpr (GATHER) {
                // the two row pointers of a load are computed on the scalar unit (a padding entry points
                // at the kilobyte of zeros behind the values); a lane only selects its half's pointer and
                // adds its column offset
                if (p.b_fits32 && rb0.r[7] >= 0) {
                    // all of B lies within 4 GiB and none of the wave's 8 entries is padding (the list
                    // ascends, padding trails): scalar base + 32-bit lane offsets, the cheaper form of the load
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t o0 = (uint32_t)rb0.r[2 * i] * ldb_bytes, o1 = (uint32_t)rb0.r[2 * i + 1] * ldb_bytes;
                        dma16_base((half ? o1 : o0) + b_coff[i], Btile, sb + 2 * i * kRowBytes);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int e0 = rb0.r[2 * i], e1 = rb0.r[2 * i + 1];
                        const char *p0 = e0 >= 0 ? Btile + (uint64_t)(uint32_t)e0 * ldb_bytes : zpad;
                        const char *p1 = e1 >= 0 ? Btile + (uint64_t)(uint32_t)e1 * ldb_bytes : zpad;
                        dma16((half ? p1 : p0) + b_coff[i], sb + 2 * i * kRowBytes);
                    }
                }
            } else if (tile_fast && rb0.r[0] >= 0) {
                const char *rowptr = Btile + (uint64_t)(uint32_t)rb0.r[0] * ldb_bytes;          // scalar, 64-bit
#pragma unroll
                for (int i = 0; i < 4; ++i) dma16_base(b_lane[i], rowptr, sb + 2 * i * kRowBytes);
            } else {         // narrow blocks, padding rows or column tail: zeros come from the zero page
                const int kc = ks < n_ks ? ks : n_ks - 1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 8 * wave + 2 * i + half;
                    const int e = lg >= 3 ? rb0.r[0] : p.krow[(int64_t)td.ks_begin * (kStepK >> lg) + ((kc * kStepK + r) >> lg)];
                    const char *src = (e >= 0 && b_col_ok[i]) ? Btile + (int64_t)(e + (r & gmask)) * ldb_bytes + b_col[i] : zeros;
                    dma16(src, sb + 2 * i * kRowBytes);
                }
            }
        };
        auto issue_a = [&](int ks, int slot) {
            if (!a_turn(ks)) return;
            const int kc = ks < n_ks ? ks : n_ks - 1;
            const char *kptr = Abase + (int64_t)kc * a_stride_bytes;             // scalar
            const uint32_t sa = smem_base + kBRing + slot * kAStage;
#pragma unroll
            for (int i = 0; i < NA; ++i)
                if (a_on[i]) dma16_base(a_lane[i], kptr, sa + a_slab[i] * kFragBytes);
        };
        // wait until this wave's loads of K-step ks have landed: everything but the loads it issued
        // after the B panel of ks, i.e. in the iterations ks-NS+1 (its A part) .. ks-1
        auto wait_stage = [&](int ks) {
            if constexpr (S >= 4) {
                wait_vmcnt<kWait>();
            } else {
                int later_a = 0;
#pragma unroll
                for (int d = 1; d <= NS - 1; ++d) later_a += a_turn(ks - d + DA) ? 1 : 0;
                if (later_a == 0) wait_vmcnt<(NS - 2) * 4>();
                else if (later_a == 1) wait_vmcnt<(NS - 2) * 4 + 1>();
                else if (later_a == 2) wait_vmcnt<(NS - 2) * 4 + 2>();
                else if (later_a == 3) wait_vmcnt<(NS - 2) * 4 + 3>();
                else wait_vmcnt<(NS - 2) * 4 + 4>();
                static_assert(NS <= 5, "at most four later A loads are told apart");
            }
        };

        // B fragment of MFMA tile f, half r: lane (q, s16) reads 8 bytes of B row
        // R = 16 (q/2) + 8 r + 4 (q%2) + s16/4 at columns 64 wave + 16 f + 4 (s16%4) ..+3; the
        // transposed read hands every lane the 4 rows of ITS column (column s16 of the tile).
        uint32_t b_off[4];
        {
            const int R0 = 16 * (q >> 1) + 4 * (q & 1) + (s16 >> 2);       // r adds 8 rows: R % 8 unchanged
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int chunk = 8 * wave + 2 * f + ((s16 & 3) >> 1);
                b_off[f] = R0 * kRowBytes + ((chunk ^ (2 * (R0 & 7))) << 4) + (s16 & 1) * 8;
            }
        }
        // the LDS reads of a K-step are issued before the next loads (the inline asm keeps that
        // order), so that their latency overlaps with the address work of the loads
        short8v bfrag[4], afrag[S];
        auto read_frags = [&](int bslot, int aslot) {
            const lds_u8_ptr sb = sm + bslot * kPanelBytes;
            const lds_u8_ptr sa = sm + kBRing + aslot * kAStage;
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(sb + b_off[f]));
                const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(sb + b_off[f] + 8 * kRowBytes));
                bfrag[f] = short8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
#pragma unroll
            for (int s = 0; s < S; ++s) afrag[s] = *(lds_short8_ptr)(sa + s * kFragBytes + lane * 16);
        };
        auto multiply = [&]() {
            // operands swapped: the result tile comes out transposed, so a lane holds 4 consecutive
            // columns of one C row and stores them as one 16-byte word
#pragma unroll
            for (int s = 0; s < S; ++s)
#pragma unroll
                for (int f = 0; f < 4; ++f) acc[s][f] = mfma16x16x32<DT>(bfrag[f], afrag[s], acc[s][f]);
        };

        // ---- software pipeline over the K-steps.  Issue order, as if the loop had started NS-1
        // iterations early: A(0 .. DA-NS), then B(t), A(DA-NS+1+t) for t = 0 .. NS-2; iteration ks
        // then issues B(ks+NS-1), A(ks+DA).  The prologue re-loads the last K-step for K-steps past the
        // end of a very short tile, so that the loop always starts with the same loads in flight.
        rb0 = load_rows(0);
        rb1 = load_rows(1);
#pragma unroll
        for (int k = 0; k <= DA - NS; ++k) issue_a(k, k);
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) {
            issue_b(t, t);
            rb0 = rb1;
            rb1 = load_rows(t + 2);
            issue_a(DA - NS + 1 + t, DA - NS + 1 + t);
        }
        int bslot = 0, aslot = 0;
        for (int ks = 0; ks < n_ks; ++ks) {
            // The last iterations issue nothing for K-steps past the end (a short tile would spend a
            // tenth of its loads there); from the first iteration whose predecessors left loads out,
            // the counted wait no longer holds and the wave waits for everything it has in flight.
            if (ks + DA > n_ks) wait_vmcnt<0>();
            else wait_stage(ks);                   // this wave's loads of K-step ks have landed
            __builtin_amdgcn_s_barrier();          // ... and everybody else's; the slots of K-step ks-1 are free
            asm volatile("" ::"s"(rb0.r[0]));      // the scalar row lookup is waited for here, not behind the LDS reads
            read_frags(bslot, aslot);
            // the load path is what bounds the kernel: a wave that is about to issue its loads goes
            // ahead of the waves that are multiplying (measured: 3-4 % on the 16-row workload)
            __builtin_amdgcn_s_setprio(3);
            if (ks + NS - 1 < n_ks) issue_b(ks + NS - 1, bslot == 0 ? NS - 1 : bslot - 1);
            if (ks + DA < n_ks) issue_a(ks + DA, aslot == 0 ? NAS - 1 : aslot - 1);
            __builtin_amdgcn_s_setprio(0);
            multiply();
            rb0 = rb1;
            rb1 = load_rows(ks + NS + 1);
            bslot = bslot == NS - 1 ? 0 : bslot + 1;
            aslot = aslot == NAS - 1 ? 0 : aslot + 1;
        }
        wait_vmcnt<0>();                           // no load may still be writing LDS when the workgroup ends
    }

    // C rows go back to their original positions through perm; beta = 0
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int rr = s * kSlabRows + s16;
        const int64_t orig = rr < td.n_rows ? (GATHER ? p.prow : p.perm)[td.row_begin + rr] : -1;
        if (orig >= 0) {                 // a position of the low-row list may be padding (-1)
            float *crow = p.C + orig * p.ldc;
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int n = n0 + wave * kWaveN + 16 * f + 4 * q;
                if (n >= p.N) continue;
                // tall tiles and gathered tiles store around the caches' write allocation (measured: the
                // dense 4096 x 16384 x 4096 product 0.44 -> 0.37 ms, the graph workload 213 -> 204 us; no
                // gain, or a small loss, for the lower classes on whole column blocks)
                if constexpr (S >= 8 || GATHER) __builtin_nontemporal_store(acc[s][f], reinterpret_cast<float4v *>(crow + n));
                else *reinterpret_cast<float4v *>(crow + n) = acc[s][f];
            }
        }
    }
}

// Measured on the 16-row workload: two ring slots and four resident workgroups per CU (36 KiB of
// LDS each) beat deeper rings with fewer workgroups; the gather is bound by how many independent
// instruction streams feed the texture-address unit, not by the depth of any one of them.
template <int DT, int S, int NS, int DA, bool GATHER = false>
__global__ void __launch_bounds__(kThreads) vbr_spmm_kernel(const Params p)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[tile_lds_bytes<S, NS, DA>()];
    int tile, ntile;
    if (!map_workgroup(p.n_tiles, p.n_ntiles, tile, ntile)) return;
    tile_body<DT, S, NS, DA, GATHER>(p, p.tiles[tile], ntile, smem);
}

// All slab classes in one launch, for matrices whose classes are each too small to fill the chip:
// the workgroup picks the code of its tile's class (registers and LDS are those of the largest).
template <int DT, int NS, int DA>
__global__ void __launch_bounds__(kThreads) vbr_spmm_mixed_kernel(const Params p)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[tile_lds_bytes<8, NS, DA>()];
    int tile, ntile;
    if (!map_workgroup(p.n_tiles, p.n_ntiles, tile, ntile)) return;
    const TileDesc td = p.tiles[tile];
    if (td.group < 0) {                   // column-gathered
        if (td.n_slabs <= 1) tile_body<DT, 1, NS, DA, true>(p, td, ntile, smem);
        else if (td.n_slabs <= 2) tile_body<DT, 2, NS, DA, true>(p, td, ntile, smem);
        else if (td.n_slabs <= 4) tile_body<DT, 4, NS, DA, true>(p, td, ntile, smem);
        else tile_body<DT, 8, NS, DA, true>(p, td, ntile, smem);
    } else if (td.n_slabs <= 1) tile_body<DT, 1, NS, DA>(p, td, ntile, smem);
    else if (td.n_slabs <= 2) tile_body<DT, 2, NS, DA>(p, td, ntile, smem);
    else if (td.n_slabs <= 4) tile_body<DT, 4, NS, DA>(p, td, ntile, smem);
    else tile_body<DT, 8, NS, DA>(p, td, ntile, smem);
}

struct PanelParams {
    const PanelDesc *panels;
    const int32_t *pk_meta;   // K-step stream: records {mask, first B row of each granule}
    const int32_t *prow;
    const uint16_t *vals;
    const uint16_t *zfrag;    // 1 KiB of zeros (behind the last fragment): source of the filler loads
    const uint16_t *zeros;
    const uint16_t *B;
    float *C;
    int64_t ldb, ldc;
    int32_t N;
    int32_t lg_gran;          // >= 3
    int32_t n_panels;         // T
    int32_t n_ntiles;         // Q = ceil(N / 128)
};

// Panel kernel: one workgroup (8 waves) owns R slabs (R * 16 rows of short row groups, whatever
// group they belong to) and 128 columns of C, and walks the union of the column blocks of those
// groups.  A B row panel is brought into LDS once per K-step for all R slabs; a slab multiplies only
// in the K-steps where its own groups store a block (mask bit), and only those fragments exist in
// memory.  Waves form a 2 x 4 grid: wave (wr, wc) owns slabs [wr R/2, (wr+1) R/2) x columns
// [32 wc, 32 wc + 32).  A direct-to-LDS load costs the CU about 22 cycles whatever its lane mask, so
// the unit of cost is the load instruction: per K-step 8 for B (1 KiB each) and 8 for A (one
// fragment each; the host splits K-steps that carry more than 8 fragments).
constexpr int kPanelThreads = 512;
template <int DT, int R, int NS, int DA>
__global__ void __launch_bounds__(kPanelThreads) vbr_spmm_panel_kernel(const PanelParams p)
{
    static_assert(NS >= 2 && (NS & (NS - 1)) == 0 && DA == NS - 1, "one ring index for both rings: a power of two, A issued with its B");
    constexpr int kPN = 128;                       // C columns per workgroup
    constexpr int kPRow = kPN * 2;                 // one staged B row: 256 bytes
    constexpr int kPPanel = kStepK * kPRow;        // 8 KiB of B per K-step
    constexpr int kAStage = kPanelMaxFrags * kFragBytes;
    constexpr int NAS = NS;
    constexpr int kBRing = NS * kPPanel;
    constexpr int HS = R / 2;                      // slabs per wave
    // per K-step a wave issues one B load, then one A load; both of K-step ks must have landed
    constexpr int kWait = (NS - 2) * 2;
    static_assert(kWait < 64, "vmcnt is a 6-bit counter");
    static_assert(kPanelMaxFrags == 8, "one fragment load per wave per K-step");
    static_assert(kPanelMetaPad >= NS + 3, "look-ahead of the K-step stream");
    // 2 KiB of slack: the fragment chain reads up to two fragments past the ones it uses
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kBRing + NAS * kAStage + 2 * kFragBytes];

    int tile, ntile;
    if (!map_workgroup(p.n_panels, p.n_ntiles, tile, ntile)) return;
    const PanelDesc pd = p.panels[tile];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 2, wc = wave & 3;
    const int n0 = ntile * kPN;
    const lds_u8_ptr sm = (lds_u8_ptr)(&smem[0]);
    const uint32_t smem_base = (uint32_t)(uintptr_t)sm;
    const char *zeros = reinterpret_cast<const char *>(p.zeros);
    const int n_ks = pd.n_ks;
    const int q = lane >> 4, s16 = lane & 15;

    float4v acc[HS][2];
#pragma unroll
    for (int s = 0; s < HS; ++s)
#pragma unroll
        for (int f = 0; f < 2; ++f) acc[s][f] = float4v{0.f, 0.f, 0.f, 0.f};

    if (n_ks > 0) {
        // ---- B staging: per K-step every wave issues 1 load: rows 4 wave + (lane / 16) of the
        // K-step, 256 bytes each (16 lanes), into 1 KiB of LDS.  LDS chunk c' of row r holds
        // global chunk c' ^ 2 (r % 8), which spreads the rows of a transposed read over all banks.
        const int lg = p.lg_gran;
        const int gmask = (1 << lg) - 1;
        const int rec = 1 + (kStepK >> lg);                       // int32 per K-step record
        const const_i32_ptr meta = (const_i32_ptr)p.pk_meta + (int64_t)pd.meta_begin * rec;
        // three readers walk the stream: the row lookup of the B loads, the mask of the A loads,
        // the mask of the multiply; each is a pointer that advances by one record per K-step
        const_i32_ptr p_rb = meta + 1 + ((4 * wave) >> lg), p_ma = meta, p_mc = meta;
        const uint32_t ldb_bytes = (uint32_t)(p.ldb * 2);
        const char *Btile = reinterpret_cast<const char *>(p.B) + (int64_t)n0 * 2;
        // chunks at or beyond column N: their lanes fetch the tile's last existing chunk again
        // (the C columns it would feed are never stored, and columns do not mix)
        const int last_chunk = (p.N - n0 < kPN ? p.N - n0 : kPN) / 8 - 1;
        const int rk = 4 * wave + q;                                // this lane's row of the K-step
        const int b_chunk = s16 ^ (2 * (rk & 7));
        const uint32_t b_lane = (uint32_t)(rk & gmask) * ldb_bytes + (b_chunk <= last_chunk ? b_chunk : last_chunk) * 16;
        auto next_rows = [&]() -> int { const int v = *p_rb; p_rb += rec; return v; };
        auto next_ma = [&]() -> uint32_t { const uint32_t v = (uint32_t)*p_ma; p_ma += rec; return v; };
        auto next_mc = [&]() -> uint32_t { const uint32_t v = (uint32_t)*p_mc; p_mc += rec; return v; };
        int rb0, rb1;
        auto issue_b = [&](int slot) {
            const uint32_t sb = smem_base + slot * kPPanel + 4 * wave * kPRow;
            if (rb0 >= 0) {
                dma16_base(b_lane, Btile + (uint64_t)(uint32_t)rb0 * ldb_bytes, sb);
            } else {         // padding rows of the K-step: zeros
                dma16(zeros, sb);
            }
        };
        // ---- A staging: the fragments of a K-step follow each other in memory, one per present
        // slab in rising slab order; fragment i is loaded by wave i.  Every wave issues one load
        // per K-step whatever the count: a wave without a fragment loads 1 KiB of zeros instead.
        const char *a_next = reinterpret_cast<const char *>(p.vals) + pd.a_off * 16;
        const char *zfrag = reinterpret_cast<const char *>(p.zfrag);
        uint32_t mA0, mA1;
        auto issue_a = [&](int slot) {
            const uint32_t sa = smem_base + kBRing + slot * kAStage;
            const int cnt = __builtin_popcount(mA0);
            dma16_base(lane * 16, wave < cnt ? a_next + wave * kFragBytes : zfrag, sa + wave * kFragBytes);
            a_next += cnt * kFragBytes;
        };

        uint32_t b_off[2];
        {
            const int R0 = 16 * (q >> 1) + 4 * (q & 1) + (s16 >> 2);
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const int chunk = 4 * wc + 2 * f + ((s16 & 3) >> 1);
                b_off[f] = R0 * kPRow + ((chunk ^ (2 * (R0 & 7))) << 4) + (s16 & 1) * 8;
            }
        }
        // the LDS reads of a K-step are issued before the next loads (the inline asm keeps that
        // order): B fragments of the wave's 32 columns and the first of its A fragments
        short8v bfrag[2], a_nxt;
        lds_u8_ptr fa;
        auto read_frags = [&](int bslot, int aslot, uint32_t m) {
            const lds_u8_ptr sb = sm + bslot * kPPanel;
            fa = sm + kBRing + aslot * kAStage + __builtin_popcount(m & ((1u << (wr * HS)) - 1u)) * kFragBytes + lane * 16;
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(sb + b_off[f]));
                const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(sb + b_off[f] + 8 * kPRow));
                bfrag[f] = short8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
            a_nxt = *(lds_short8_ptr)fa;
        };
        auto multiply = [&](uint32_t mh) {
            // the fragments of this wave's present slabs follow each other: read one ahead
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                if (mh >> s & 1) {
                    const short8v a_cur = a_nxt;
                    fa += kFragBytes;
                    a_nxt = *(lds_short8_ptr)fa;
#pragma unroll
                    for (int f = 0; f < 2; ++f) acc[s][f] = mfma16x16x32<DT>(bfrag[f], a_cur, acc[s][f]);
                }
            }
        };

        // ---- software pipeline: K-steps 0 .. NS-2 are issued up front (B then A each); iteration
        // ks issues K-step ks+NS-1 into the slot K-step ks-1 has left.  K-steps past the end are
        // filler records of the stream (mask 0, rows of the last step), so the loads in flight per
        // wave never change in number.
        rb0 = next_rows();
        rb1 = next_rows();
        mA0 = next_ma();
        mA1 = next_ma();
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) {
            issue_b(t);
            issue_a(t);
            rb0 = rb1; mA0 = mA1;
            rb1 = next_rows();
            mA1 = next_ma();
        }
        uint32_t mC0 = next_mc(), mC1 = next_mc();
        for (int ks = 0; ks < n_ks; ++ks) {
            wait_vmcnt<kWait>();
            __builtin_amdgcn_s_barrier();
            // scalar lookups (issued at the end of earlier iterations) are waited for here, not behind the LDS reads
            asm volatile("" ::"s"(rb0), "s"(mA0), "s"(mC0));
            const int cur = ks & (NS - 1), fill = (ks - 1) & (NS - 1);
            const uint32_t mh = (mC0 >> (wr * HS)) & ((1u << HS) - 1u);      // this wave's slabs
            if (mh != 0) read_frags(cur, cur, mC0);
            issue_b(fill);
            issue_a(fill);
            if (mh != 0) multiply(mh);
            rb0 = rb1; mA0 = mA1; mC0 = mC1;
            rb1 = next_rows();
            mA1 = next_ma();
            mC1 = next_mc();
        }
        wait_vmcnt<0>();
    }

#pragma unroll
    for (int s = 0; s < HS; ++s) {
        const int rr = (wr * HS + s) * kSlabRows + s16;
        const int64_t orig = rr < pd.n_rows ? p.prow[pd.row_begin + rr] : -1;
        if (orig >= 0) {                 // a position of the low-row list may be padding (-1)
            float *crow = p.C + orig * p.ldc;
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                const int n = n0 + wc * 32 + 16 * f + 4 * q;
                if (n < p.N) *reinterpret_cast<float4v *>(crow + n) = acc[s][f];
            }
        }
    }
}

constexpr int kStages = 2;      // LDS ring of B panels
constexpr int kStagesTall = 3;  // the same for tiles of 5 to 8 slabs (80 KiB of LDS, two workgroups per CU): measured 3 % (K = 16 384)
                                // to 14 % (K = 8 192) faster than 2 on dense matrices; slower than 2 for every lower class
constexpr int kADistance = 3;   // K-steps the A fragments are requested ahead

template <int DT>
int launch_all(const vbr *v, const Params &base, const PanelParams &pp, hipStream_t caller)
{
    Launch plan[VBR_MAX_LAUNCHES];
    const int n = plan_launches(v, base.N, plan);
    for (int i = 0; i < n; ++i)
        if (plan[i].grid > INT32_MAX) return VBR_EINVAL;
    // Several launches write disjoint rows of C and are independent of each other: the first stays on
    // the caller's stream, the others go to the side streams behind an event recorded on the caller's
    // stream, and the caller's stream waits for each side stream's last launch.
    static const bool serial = getenv("VBR_SPMM_SERIAL") != nullptr;
    const bool fork = n > 1 && v->ev_fork && !serial;
    if (fork) {
        hipError_t e = hipEventRecord((hipEvent_t)v->ev_fork, caller);
        for (int k = 0; e == hipSuccess && k < std::min(n - 1, (int)vbr::kSideStreams); ++k)
            e = hipStreamWaitEvent((hipStream_t)v->side_stream[k], (hipEvent_t)v->ev_fork, 0);
        if (e != hipSuccess) { set_last_hip_error((int)e); return VBR_EHIP; }
    }
    for (int i = 0; i < n; ++i) {
        const Launch &L = plan[i];
        hipStream_t stream = fork && i > 0 ? (hipStream_t)v->side_stream[(i - 1) % vbr::kSideStreams] : caller;
        Params p = base;
        p.tiles = base.tiles + L.first_tile;
        p.n_tiles = L.n_tiles;
        const dim3 grid((unsigned)L.grid);
        switch (L.kind) {
        case VBR_LAUNCH_PANEL:
            hipLaunchKernelGGL((vbr_spmm_panel_kernel<DT, 8, 4, 3>), grid, dim3(kPanelThreads), 0, stream, pp);
            break;
        case VBR_LAUNCH_TILE_MIXED:
            hipLaunchKernelGGL((vbr_spmm_mixed_kernel<DT, kStages, kADistance>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_GATHER_1:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 1, kStages, kADistance, true>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_GATHER_2:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 2, kStages, kADistance, true>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_GATHER_4:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 4, kStages, kADistance, true>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_GATHER_8:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 8, kStagesTall, kADistance, true>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_TILE_1:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 1, kStages, kADistance>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_TILE_2:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 2, kStages, kADistance>), grid, dim3(kThreads), 0, stream, p);
            break;
        case VBR_LAUNCH_TILE_4:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 4, kStages, kADistance>), grid, dim3(kThreads), 0, stream, p);
            break;
        default:
            hipLaunchKernelGGL((vbr_spmm_kernel<DT, 8, kStagesTall, kADistance>), grid, dim3(kThreads), 0, stream, p);
            break;
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) { set_last_hip_error((int)e); return VBR_EHIP; }
    }
    if (fork) {
        for (int k = 0; k < std::min(n - 1, (int)vbr::kSideStreams); ++k) {
            hipError_t e = hipEventRecord((hipEvent_t)v->ev_join[k], (hipStream_t)v->side_stream[k]);
            if (e == hipSuccess) e = hipStreamWaitEvent(caller, (hipEvent_t)v->ev_join[k], 0);
            if (e != hipSuccess) { set_last_hip_error((int)e); return VBR_EHIP; }
        }
    }
    return VBR_OK;
}

// Streams and events of the forked launches; vbr_free calls this through the handle.
void release_device_objects(vbr *v)
{
    for (int k = 0; k < vbr::kSideStreams; ++k) {
        if (v->ev_join[k]) (void)hipEventDestroy((hipEvent_t)v->ev_join[k]);
        if (v->side_stream[k]) (void)hipStreamDestroy((hipStream_t)v->side_stream[k]);
        v->ev_join[k] = v->side_stream[k] = nullptr;
    }
    if (v->ev_fork) (void)hipEventDestroy((hipEvent_t)v->ev_fork);
    v->ev_fork = nullptr;
    v->release_dev = nullptr;
}

int create_device_objects(vbr *v)
{
    if (v->ev_fork) return VBR_OK;
    // a matrix with one kind of work is one launch whatever N is: nothing to spread
    int kinds = v->panels.empty() ? 0 : 1;
    for (int c = 0; c < 4; ++c)
        kinds += (v->class_begin[c + 1] > v->class_begin[c]) + (v->gclass_begin[c + 1] > v->gclass_begin[c]);
    if (kinds <= 1) return VBR_OK;
    v->release_dev = release_device_objects;
    hipEvent_t ev;
    hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e == hipSuccess) v->ev_fork = ev;
    for (int k = 0; e == hipSuccess && k < vbr::kSideStreams; ++k) {
        hipStream_t st;
        e = hipStreamCreateWithFlags(&st, hipStreamNonBlocking);       // default priority
        if (e != hipSuccess) break;
        v->side_stream[k] = st;
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e == hipSuccess) v->ev_join[k] = ev;
    }
    if (e != hipSuccess) { release_device_objects(v); set_last_hip_error((int)e); return VBR_EHIP; }
    return VBR_OK;
}

}  // namespace
}  // namespace vbrk

extern "C" int vbr_last_hip_error(void) { return vbrk::g_last_hip_error; }

extern "C" int vbr_upload(vbr_t *v, void *buf_dev, void *hip_stream)
{
    if (!v || !buf_dev || (reinterpret_cast<uintptr_t>(buf_dev) & 255) != 0) return VBR_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *d = static_cast<char *>(buf_dev);
    const vbrk::DeviceLayout &L = v->lay;
    struct Part { int64_t off; const void *src; size_t bytes; };
    static const unsigned char kZeros[256] = {0};
    const Part parts[10] = {
        {L.tiles_off + (int64_t)(v->tiles.size() * sizeof(vbrk::TileDesc)), v->gtiles_dev.data(), v->gtiles_dev.size() * sizeof(vbrk::TileDesc)},
        {L.gcol_off, v->gcol.data(), v->gcol.size() * 4},
        {L.panels_off, v->panels.data(), v->panels.size() * sizeof(vbrk::PanelDesc)},
        {L.pk_meta_off, v->pk_meta.data(), v->pk_meta.size() * 4},
        {L.prow_off, v->prow.data(), v->prow.size() * 4},
        {L.zeros_off, kZeros, sizeof(kZeros)},
        {L.tiles_off, v->tiles.data(), v->tiles.size() * sizeof(vbrk::TileDesc)},
        {L.krow_off, v->krow.data(), v->krow.size() * 4},
        {L.perm_off, v->perm.data(), v->perm.size() * 4},
        {L.vals_off, v->vals.data(), v->vals.size() * 2},
    };
    for (const Part &pt : parts) {
        if (pt.bytes == 0) continue;
        hipError_t e = hipMemcpyAsync(d + pt.off, pt.src, pt.bytes, hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) { vbrk::set_last_hip_error((int)e); return VBR_EHIP; }
    }
    hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) { vbrk::set_last_hip_error((int)e); return VBR_EHIP; }
    v->dev = buf_dev;
    return vbrk::create_device_objects(v);
}

extern "C" int vbr_spmm(const vbr_t *v, const void *B_dev, int64_t ldb, float *C_dev, int64_t ldc,
                        int64_t N, void *hip_stream)
{
    if (!v) return VBR_EINVAL;
    if (!v->dev) return VBR_ESTATE;
    if (N < 0 || N % 8 != 0 || N > (int64_t)INT32_MAX - 1024) return VBR_EINVAL;
    if (N == 0 || v->n_rows == 0) return VBR_OK;
    if (!B_dev || !C_dev || ldb < N || ldc < N || ldb % 8 != 0 || ldc % 4 != 0) return VBR_EINVAL;
    if (ldb >= ((int64_t)1 << 26)) return VBR_EUNSUPPORTED;   // a lane's offset inside a 32-row granule of B is 32 bits
    if ((reinterpret_cast<uintptr_t>(B_dev) & 15) != 0 || (reinterpret_cast<uintptr_t>(C_dev) & 15) != 0) return VBR_EINVAL;
    const char *d = static_cast<const char *>(v->dev);
    vbrk::Params p;
    p.tiles = reinterpret_cast<const vbrk::TileDesc *>(d + v->lay.tiles_off);
    p.krow = reinterpret_cast<const int32_t *>(d + v->lay.krow_off);
    p.perm = reinterpret_cast<const int32_t *>(d + v->lay.perm_off);
    p.vals = reinterpret_cast<const uint16_t *>(d + v->lay.vals_off);
    p.zeros = reinterpret_cast<const uint16_t *>(d + v->lay.zeros_off);
    p.B = static_cast<const uint16_t *>(B_dev);
    p.C = C_dev;
    p.ldb = ldb;
    p.ldc = ldc;
    p.N = (int32_t)N;
    p.lg_gran = v->lg_gran;
    p.n_tiles = 0;
    p.n_ntiles = (int32_t)((N + vbrk::kTileN - 1) / vbrk::kTileN);
    vbrk::PanelParams pp;
    pp.panels = reinterpret_cast<const vbrk::PanelDesc *>(d + v->lay.panels_off);
    pp.pk_meta = reinterpret_cast<const int32_t *>(d + v->lay.pk_meta_off);
    pp.zfrag = p.vals + (v->vals.size() - vbrk::kFragElems);
    pp.prow = reinterpret_cast<const int32_t *>(d + v->lay.prow_off);
    pp.vals = p.vals;
    pp.zeros = p.zeros;
    pp.B = p.B;
    pp.C = C_dev;
    pp.ldb = ldb;
    pp.ldc = ldc;
    pp.N = (int32_t)N;
    pp.lg_gran = v->lg_gran;
    pp.n_panels = (int32_t)v->panels.size();
    pp.n_ntiles = (int32_t)((N + 127) / 128);
    p.gcol = reinterpret_cast<const int32_t *>(d + v->lay.gcol_off);
    p.zfrag = pp.zfrag;
    p.b_fits32 = (v->n_cols * ldb * 2 + N * 2) < ((int64_t)1 << 32) ? 1 : 0;
    p.prow = pp.prow;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return v->dtype == VBR_F16 ? vbrk::launch_all<VBR_F16>(v, p, pp, stream) : vbrk::launch_all<VBR_BF16>(v, p, pp, stream);
}
