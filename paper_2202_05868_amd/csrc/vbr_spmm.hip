// vbr_spmm on gfx950: C = A.B with A in packed VBR form (section 4.4.1 of the paper: every stored
// block is multiplied as a dense product on the matrix units).  One launch per slab class; each
// workgroup owns up to 8 slabs of 16 rows of ONE row group and a 256-column tile of C, walks the
// group's block list in K-steps of 32 B rows, stages the gathered B rows and the A fragments in
// LDS (double buffered, 128-bit global loads), and issues v_mfma_f32_16x16x32 on them.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "vbr_host.h"

namespace vbrk {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int code) { g_last_hip_error = code; }

namespace {

constexpr int kThreads = 256;          // 4 waves
constexpr int kTileN = 256;            // C columns per workgroup
constexpr int kWaveN = 64;             // C columns per wave: 4 MFMA tiles of 16
constexpr int kLdsRow = kTileN + 16;   // 16-bit values per staged B row; the 32-byte pad shifts
                                       // consecutive rows by 8 LDS banks
constexpr int kXcd = 8;                // L2 domains; workgroup i runs on domain i % 8

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;

struct Params {
    const TileDesc *tiles;    // tiles of this launch's slab class
    const int32_t *krow;
    const int32_t *perm;
    const uint16_t *vals;
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

// S = slabs the instantiation computes (tiles of the class have S/2 < n_slabs <= S, n_slabs = 1 for S = 1).
template <int DT, int S>
__global__ void __launch_bounds__(kThreads) vbr_spmm_kernel(const Params p)
{
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][kStepK * kLdsRow];
    __shared__ __attribute__((aligned(16))) uint16_t As[2][S * kFragElems];

    // Workgroup -> (tile, column tile).  Workgroups are dealt to the 8 L2 domains round-robin;
    // a domain keeps to few column tiles so that the B columns it gathers stay in its L2.
    const int T = p.n_tiles, Q = p.n_ntiles;
    const int x = blockIdx.x & (kXcd - 1), j = blockIdx.x >> 3;
    int tile, ntile;
    if (Q >= kXcd) {
        ntile = x + kXcd * (j / T);
        tile = j % T;
        if (ntile >= Q) return;
    } else {
        ntile = x % Q;
        const int member = x / Q, members = (kXcd - ntile + Q - 1) / Q;
        tile = member + members * j;
        if (tile >= T) return;
    }
    const TileDesc td = p.tiles[tile];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = ntile * kTileN;

    // staging role for B: 16-byte column chunk bc of rows br, br+8, br+16, br+24 of the K-step
    const int bc = tid & 31, br = tid >> 5;
    const bool col_ok = n0 + bc * 8 < p.N;
    const uint16_t *Bcol = p.B + n0 + bc * 8;
    const int gmask = (1 << p.lg_gran) - 1;
    // staging role for A: fragment lane `lane` of slabs wave, wave+4
    constexpr int NA = (S + 3) / 4;
    const int rows_last = td.n_rows - (td.n_slabs - 1) * kSlabRows;
    const int64_t a_stride = (int64_t)(td.n_slabs - 1) * kFragElems + (int64_t)rows_last * kStepK;
    const uint16_t *Abase = p.vals + td.a_off * 8;
    int a_src[NA];      // offset of this thread's 16 bytes inside a K-step of the tile, -1 = padding
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int s = wave + 4 * i, m = lane & 15, q = lane >> 4;
        const int rows = (s == td.n_slabs - 1) ? rows_last : kSlabRows;
        a_src[i] = (s < td.n_slabs && s < S && m < rows) ? s * kFragElems + (q * rows + m) * 8 : -1;
    }

    float4v acc[S][4];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[s][f] = float4v{0.f, 0.f, 0.f, 0.f};

    int rowidx[4];
    uint4 breg[4], areg[NA];
    auto load_rows = [&](int ks) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = br + 8 * i;
            const int base = p.krow[((td.ks_begin + ks) * kStepK + r) >> p.lg_gran];
            rowidx[i] = base < 0 ? -1 : base + (r & gmask);
        }
    };
    auto load_tiles = [&](int ks) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            breg[i] = uint4{0u, 0u, 0u, 0u};
            if (rowidx[i] >= 0 && col_ok) breg[i] = *reinterpret_cast<const uint4 *>(Bcol + (int64_t)rowidx[i] * p.ldb);
        }
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            areg[i] = uint4{0u, 0u, 0u, 0u};
            if (a_src[i] >= 0) areg[i] = *reinterpret_cast<const uint4 *>(Abase + (int64_t)ks * a_stride + a_src[i]);
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint4 *>(&Bs[buf][(br + 8 * i) * kLdsRow + bc * 8]) = breg[i];
#pragma unroll
        for (int i = 0; i < NA; ++i)
            if (wave + 4 * i < S) *reinterpret_cast<uint4 *>(&As[buf][(wave + 4 * i) * kFragElems + lane * 8]) = areg[i];
    };

    const int n_ks = td.n_ks;
    if (n_ks > 0) {
        load_rows(0);
        load_tiles(0);
        if (n_ks > 1) load_rows(1);
        store_tiles(0);
    }
    __syncthreads();

    // B fragment of MFMA tile f, half r: lane (q, s16) reads 4 values of B row
    // 8 (2 (q/2) + r) + 4 (q%2) + s16/4 at column 64 wave + 16 f + 4 (s16 % 4); the transposed
    // read hands every lane the 4 rows of ITS column (column s16 of the tile).
    const int q = lane >> 4, s16 = lane & 15;
    const int b_base = (16 * (q >> 1) + 4 * (q & 1) + (s16 >> 2)) * kLdsRow + wave * kWaveN + 4 * (s16 & 3);

    for (int ks = 0; ks < n_ks; ++ks) {
        const int cur = ks & 1;
        const bool more = ks + 1 < n_ks;
        if (more) {
            load_tiles(ks + 1);
            if (ks + 2 < n_ks) load_rows(ks + 2);
        }
        short8v bfrag[4];
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(&Bs[cur][b_base + 16 * f]));
            const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(&Bs[cur][b_base + 16 * f + 8 * kLdsRow]));
            bfrag[f] = short8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const short8v afrag = *reinterpret_cast<const short8v *>(&As[cur][s * kFragElems + lane * 8]);
            // operands swapped: the result tile comes out transposed, so a lane holds 4 consecutive
            // columns of one C row and stores them as one 16-byte word
#pragma unroll
            for (int f = 0; f < 4; ++f) acc[s][f] = mfma16x16x32<DT>(bfrag[f], afrag, acc[s][f]);
        }
        if (more) store_tiles(cur ^ 1);
        __syncthreads();
    }

    // C rows go back to their original positions through perm; beta = 0
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int rr = s * kSlabRows + s16;
        if (rr < td.n_rows) {
            const int64_t orig = p.perm[td.row_begin + rr];
            float *crow = p.C + orig * p.ldc;
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int n = n0 + wave * kWaveN + 16 * f + 4 * q;
                if (n < p.N) *reinterpret_cast<float4v *>(crow + n) = acc[s][f];
            }
        }
    }
}

template <int DT, int S>
int launch_class(const vbr *v, const Params &base, int cls, hipStream_t stream)
{
    const int T = v->class_begin[cls + 1] - v->class_begin[cls];
    if (T == 0) return VBR_OK;
    Params p = base;
    p.tiles = base.tiles + v->class_begin[cls];
    p.n_tiles = T;
    const int64_t Q = p.n_ntiles;
    int64_t grid;
    if (Q >= kXcd) grid = (int64_t)kXcd * ((Q + kXcd - 1) / kXcd) * T;
    else grid = (int64_t)kXcd * ((T + (kXcd / Q) - 1) / (kXcd / Q));
    if (grid > INT32_MAX) return VBR_EINVAL;
    hipLaunchKernelGGL((vbr_spmm_kernel<DT, S>), dim3((unsigned)grid), dim3(kThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_last_hip_error((int)e); return VBR_EHIP; }
    return VBR_OK;
}

template <int DT>
int launch_all(const vbr *v, const Params &p, hipStream_t stream)
{
    int rc = launch_class<DT, 1>(v, p, 0, stream);
    if (rc == VBR_OK) rc = launch_class<DT, 2>(v, p, 1, stream);
    if (rc == VBR_OK) rc = launch_class<DT, 4>(v, p, 2, stream);
    if (rc == VBR_OK) rc = launch_class<DT, 8>(v, p, 3, stream);
    return rc;
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
    const Part parts[4] = {
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
    return VBR_OK;
}

extern "C" int vbr_spmm(const vbr_t *v, const void *B_dev, int64_t ldb, float *C_dev, int64_t ldc,
                        int64_t N, void *hip_stream)
{
    if (!v) return VBR_EINVAL;
    if (!v->dev) return VBR_ESTATE;
    if (N < 0 || N % 8 != 0 || N > (int64_t)INT32_MAX - 1024) return VBR_EINVAL;
    if (N == 0 || v->n_rows == 0) return VBR_OK;
    if (!B_dev || !C_dev || ldb < N || ldc < N || ldb % 8 != 0 || ldc % 4 != 0) return VBR_EINVAL;
    if ((reinterpret_cast<uintptr_t>(B_dev) & 15) != 0 || (reinterpret_cast<uintptr_t>(C_dev) & 15) != 0) return VBR_EINVAL;
    const char *d = static_cast<const char *>(v->dev);
    vbrk::Params p;
    p.tiles = reinterpret_cast<const vbrk::TileDesc *>(d + v->lay.tiles_off);
    p.krow = reinterpret_cast<const int32_t *>(d + v->lay.krow_off);
    p.perm = reinterpret_cast<const int32_t *>(d + v->lay.perm_off);
    p.vals = reinterpret_cast<const uint16_t *>(d + v->lay.vals_off);
    p.B = static_cast<const uint16_t *>(B_dev);
    p.C = C_dev;
    p.ldb = ldb;
    p.ldc = ldc;
    p.N = (int32_t)N;
    p.lg_gran = v->lg_gran;
    p.n_tiles = 0;
    p.n_ntiles = (int32_t)((N + vbrk::kTileN - 1) / vbrk::kTileN);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return v->dtype == VBR_F16 ? vbrk::launch_all<VBR_F16>(v, p, stream) : vbrk::launch_all<VBR_BF16>(v, p, stream);
}
