// Comparator kernel: C = A.B straight from CSR (the role the sparse-library routine plays in
// section 4.4.2 of the paper).  One wave per row and 512-column tile: the lanes hold 8 consecutive
// columns each in fp32, the row's entries are walked with wave-uniform (scalar) loads of column
// index and value, and every entry costs one 16-byte load of B per lane.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "vbr_host.h"

struct csr_dev {
    int64_t n_rows = 0, n_cols = 0, nnz = 0;
    int32_t dtype = 0;
    std::vector<int64_t> row_ptr;
    std::vector<int32_t> col_idx;
    std::vector<uint16_t> vals;
    int64_t col_off = 0, val_off = 0, total = 256;
    void *dev = nullptr;
};

namespace vbrk {
namespace {

constexpr int kCsrThreads = 256;     // 4 waves = 4 rows per workgroup
constexpr int kCsrTileN = 512;       // 64 lanes x 8 columns

typedef short short8v __attribute__((ext_vector_type(8)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ float to_f32(short x)
{
    if constexpr (DT == VBR_F16) return (float)__builtin_bit_cast(_Float16, x);
    else return __builtin_bit_cast(float, (uint32_t)(uint16_t)x << 16);
}

template <int DT>
__global__ void __launch_bounds__(kCsrThreads) csr_spmm_kernel(const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                                               const uint16_t *__restrict__ vals, const uint16_t *__restrict__ B,
                                                               float *__restrict__ C, int64_t ldb, int64_t ldc, int64_t n_rows, int32_t N)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    const int n = blockIdx.y * kCsrTileN + lane * 8;
    if (row >= n_rows || n >= N) return;
    const int64_t p0 = row_ptr[row], p1 = row_ptr[row + 1];
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    const uint16_t *Bn = B + n;
    int64_t p = p0;
    for (; p + 4 <= p1; p += 4) {        // four independent B loads in flight
        short8v b[4];
        float a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            b[u] = *reinterpret_cast<const short8v *>(Bn + (int64_t)col_idx[p + u] * ldb);
            a[u] = to_f32<DT>((short)vals[p + u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(a[u], to_f32<DT>(b[u][i]), acc[i]);
    }
    for (; p < p1; ++p) {
        const short8v b = *reinterpret_cast<const short8v *>(Bn + (int64_t)col_idx[p] * ldb);
        const float a = to_f32<DT>((short)vals[p]);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(a, to_f32<DT>(b[i]), acc[i]);
    }
    float *c = C + row * ldc + n;
    *reinterpret_cast<float4v *>(c) = float4v{acc[0], acc[1], acc[2], acc[3]};
    *reinterpret_cast<float4v *>(c + 4) = float4v{acc[4], acc[5], acc[6], acc[7]};
}

inline int64_t align_up256(int64_t x) { return (x + 255) / 256 * 256; }

}  // namespace
}  // namespace vbrk

extern "C" int csr_spmm_create(const vbr_csr_t *csr, csr_dev_t **out)
{
    if (!csr || !out) return VBR_EINVAL;
    *out = nullptr;
    const int rc = vbrk::validate_csr(csr, true);
    if (rc != VBR_OK) return rc;
    try {
        csr_dev *h = new csr_dev();
        h->n_rows = csr->n_rows;
        h->n_cols = csr->n_cols;
        h->nnz = csr->nnz;
        h->dtype = csr->dtype;
        h->row_ptr.assign(csr->row_ptr, csr->row_ptr + csr->n_rows + 1);
        h->col_idx.assign(csr->col_idx, csr->col_idx + csr->nnz);
        const uint16_t *v = static_cast<const uint16_t *>(csr->vals);
        h->vals.assign(v, v + csr->nnz);
        h->col_off = vbrk::align_up256((csr->n_rows + 1) * 8);
        h->val_off = vbrk::align_up256(h->col_off + csr->nnz * 4);
        h->total = vbrk::align_up256(h->val_off + csr->nnz * 2 + 256);
        *out = h;
        return VBR_OK;
    } catch (const std::bad_alloc &) {
        return VBR_ENOMEM;
    } catch (...) {
        return VBR_EINVAL;
    }
}

extern "C" int64_t csr_device_bytes(const csr_dev_t *h) { return h ? h->total : 0; }

extern "C" int csr_upload(csr_dev_t *h, void *buf_dev, void *hip_stream)
{
    if (!h || !buf_dev || (reinterpret_cast<uintptr_t>(buf_dev) & 255) != 0) return VBR_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *d = static_cast<char *>(buf_dev);
    struct Part { int64_t off; const void *src; size_t bytes; };
    const Part parts[3] = {
        {0, h->row_ptr.data(), h->row_ptr.size() * 8},
        {h->col_off, h->col_idx.data(), h->col_idx.size() * 4},
        {h->val_off, h->vals.data(), h->vals.size() * 2},
    };
    for (const Part &pt : parts) {
        if (pt.bytes == 0) continue;
        hipError_t e = hipMemcpyAsync(d + pt.off, pt.src, pt.bytes, hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) { vbrk::set_last_hip_error((int)e); return VBR_EHIP; }
    }
    hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) { vbrk::set_last_hip_error((int)e); return VBR_EHIP; }
    h->dev = buf_dev;
    return VBR_OK;
}

extern "C" int csr_spmm(const csr_dev_t *h, const void *B_dev, int64_t ldb, float *C_dev, int64_t ldc,
                        int64_t N, void *hip_stream)
{
    if (!h) return VBR_EINVAL;
    if (!h->dev) return VBR_ESTATE;
    if (N < 0 || N % 8 != 0 || N > (int64_t)INT32_MAX - 1024) return VBR_EINVAL;
    if (N == 0 || h->n_rows == 0) return VBR_OK;
    if (!B_dev || !C_dev || ldb < N || ldc < N || ldb % 8 != 0 || ldc % 4 != 0) return VBR_EINVAL;
    if ((reinterpret_cast<uintptr_t>(B_dev) & 15) != 0 || (reinterpret_cast<uintptr_t>(C_dev) & 15) != 0) return VBR_EINVAL;
    const int64_t gx = (h->n_rows + 3) / 4, gy = (N + vbrk::kCsrTileN - 1) / vbrk::kCsrTileN;
    if (gx > INT32_MAX || gy > 65535) return VBR_EUNSUPPORTED;
    const char *d = static_cast<const char *>(h->dev);
    const int64_t *row_ptr = reinterpret_cast<const int64_t *>(d);
    const int32_t *col_idx = reinterpret_cast<const int32_t *>(d + h->col_off);
    const uint16_t *vals = reinterpret_cast<const uint16_t *>(d + h->val_off);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)gx, (unsigned)gy), block(vbrk::kCsrThreads);
    if (h->dtype == VBR_F16)
        hipLaunchKernelGGL((vbrk::csr_spmm_kernel<VBR_F16>), grid, block, 0, stream, row_ptr, col_idx, vals,
                           static_cast<const uint16_t *>(B_dev), C_dev, ldb, ldc, h->n_rows, (int32_t)N);
    else
        hipLaunchKernelGGL((vbrk::csr_spmm_kernel<VBR_BF16>), grid, block, 0, stream, row_ptr, col_idx, vals,
                           static_cast<const uint16_t *>(B_dev), C_dev, ldb, ldc, h->n_rows, (int32_t)N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { vbrk::set_last_hip_error((int)e); return VBR_EHIP; }
    return VBR_OK;
}

extern "C" void csr_free(csr_dev_t *h) { delete h; }
