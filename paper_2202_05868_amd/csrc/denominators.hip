// Measured denominators of the blocked multiply on gfx950: small loops that exercise one unit of
// the compute unit each, at the occupancy the kernels of vbr_spmm.hip run at.  They are what the
// kernel's measured time is priced against beside the published peaks: the issue rate of the three
// matrix instructions the kernels could use, the rate at which operands leave LDS (transposed 64-bit
// reads, plain 64- and 128-bit reads), the rate of 128-bit direct-to-LDS loads from cache-resident
// memory (the gather of B rows), and a streaming copy through HBM.  Not part of the path: nothing
// in vbr_spmm calls these.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "vbr_host.h"

namespace vbrk {
namespace {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;
typedef __attribute__((address_space(3))) short8v *lds_short8_ptr;
typedef __attribute__((address_space(3))) unsigned char *lds_u8_ptr;

constexpr int kProbeThreads = 256;     // 4 waves, one per SIMD

// ---- matrix instruction issue rate: four independent accumulator chains per wave
template <int KIND>
__global__ void __launch_bounds__(kProbeThreads) probe_mfma(float *out, int iters)
{
    half8v a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(threadIdx.x * 0.001f + i); b[i] = (_Float16)(i * 0.5f); }
    const half4v a4 = {a[0], a[1], a[2], a[3]}, b4 = {b[0], b[1], b[2], b[3]};
    float4v c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    float16v d0 = {0}, d1 = {0};
    for (int it = 0; it < iters; ++it) {
        if constexpr (KIND == VBR_PROBE_MFMA_16X16X32) {
            c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c3, 0, 0, 0);
        } else if constexpr (KIND == VBR_PROBE_MFMA_16X16X16) {
            c0 = __builtin_amdgcn_mfma_f32_16x16x16f16(a4, b4, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_16x16x16f16(a4, b4, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_16x16x16f16(a4, b4, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_16x16x16f16(a4, b4, c3, 0, 0, 0);
        } else {
            d0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, d0, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, d1, 0, 0, 0);
            d0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, d0, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, d1, 0, 0, 0);
        }
    }
    const float s = c0[0] + c1[1] + c2[2] + c3[3] + d0[0] + d1[5];
    if (s == 12345.678f) out[0] = s;      // never true: keeps the chains alive
}

// ---- LDS -> register operand rate: 8 reads per iteration per wave out of a 32 KiB region, with the
// address pattern the kernels use (transposed reads: 16 rows of 256 bytes, 16-byte chunks XOR-ed
// with the row; plain reads: consecutive lanes, consecutive addresses)
template <int KIND>
__global__ void __launch_bounds__(kProbeThreads) probe_lds(int *out, int iters)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[32768];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 32768 / 4; i += kProbeThreads) ((int *)smem)[i] = i;
    __syncthreads();
    const lds_u8_ptr sm = (lds_u8_ptr)(&smem[0]);
    const int q = lane >> 4, s16 = lane & 15;
    uint32_t off[8];
    for (int f = 0; f < 8; ++f) {
        if (KIND == VBR_PROBE_LDS_TR_B64) {
            const int r = 4 * q + (s16 >> 2);
            const int chunk = 2 * f + ((s16 & 3) >> 1);
            off[f] = r * 256 + ((chunk ^ (2 * (r & 7))) << 4) + (s16 & 1) * 8;
        } else if (KIND == VBR_PROBE_LDS_B64) {
            off[f] = f * 512 + lane * 8;
        } else {
            off[f] = f * 1024 + lane * 16;
        }
    }
    int acc = 0;
    for (int it = 0; it < iters; ++it) {
        const lds_u8_ptr base = sm + ((it + wave) & 3) * (KIND == VBR_PROBE_LDS_B128 ? 8192 : 4096);
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            if constexpr (KIND == VBR_PROBE_LDS_TR_B64) {
                const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(base + off[f]));
                acc += v[0] + v[3];
            } else if constexpr (KIND == VBR_PROBE_LDS_B64) {
                const short4v v = *(lds_short4_ptr)(base + off[f]);
                acc += v[0] + v[3];
            } else {
                const short8v v = *(lds_short8_ptr)(base + off[f]);
                acc += v[0] + v[7];
            }
        }
    }
    if (acc == 0x7fffffff) out[0] = acc;
}

// ---- direct-to-LDS loads, 16 bytes per lane (1 KiB per instruction), from a region of `span`
// bytes that stays cache-resident: every wave issues 8 loads, waits, repeats
__global__ void __launch_bounds__(kProbeThreads) probe_dma(const unsigned char *src, uint32_t span_mask, int *out, int iters)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[32768];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8_ptr)(&smem[0]) + wave * 8192;
    uint32_t pos = (blockIdx.x * 4 + wave) * 8192u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            const unsigned char *g = src + ((pos + f * 1024u) & span_mask) + lane * 16;
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g),
                         "s"((uint32_t)__builtin_amdgcn_readfirstlane(lds0 + f * 1024)) : "memory");
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        pos += 8192u * 1031u;        // another 8 KiB block of the region
    }
    __syncthreads();
    if (((int *)smem)[tid] == 0x7fffffff && iters < 0) out[0] = 1;
}

// ---- streaming copy, 16 bytes per lane per step
__global__ void __launch_bounds__(kProbeThreads) probe_copy(const float4v *__restrict__ src, float4v *__restrict__ dst, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kProbeThreads;
    for (; i < n; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace vbrk

extern "C" int vbr_probe_launch(int32_t kind, void *buf_dev, int64_t buf_bytes, int32_t iters, void *hip_stream,
                                double *work)
{
    using namespace vbrk;
    if (!buf_dev || !work || iters <= 0 || (reinterpret_cast<uintptr_t>(buf_dev) & 255) != 0) return VBR_EINVAL;
    if (buf_bytes < ((int64_t)1 << 20)) return VBR_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus <= 0) { set_last_hip_error((int)e); return VBR_EHIP; }
    const int blocks = cus * 4;          // four workgroups of four waves per compute unit
    const double waves = (double)blocks * 4;
    switch (kind) {
    case VBR_PROBE_MFMA_16X16X32:
        hipLaunchKernelGGL(probe_mfma<VBR_PROBE_MFMA_16X16X32>, dim3(blocks), dim3(kProbeThreads), 0, stream, (float *)buf_dev, iters);
        *work = waves * iters * 4 * 2.0 * 16 * 16 * 32;
        break;
    case VBR_PROBE_MFMA_16X16X16:
        hipLaunchKernelGGL(probe_mfma<VBR_PROBE_MFMA_16X16X16>, dim3(blocks), dim3(kProbeThreads), 0, stream, (float *)buf_dev, iters);
        *work = waves * iters * 4 * 2.0 * 16 * 16 * 16;
        break;
    case VBR_PROBE_MFMA_32X32X16:
        hipLaunchKernelGGL(probe_mfma<VBR_PROBE_MFMA_32X32X16>, dim3(blocks), dim3(kProbeThreads), 0, stream, (float *)buf_dev, iters);
        *work = waves * iters * 4 * 2.0 * 32 * 32 * 16;
        break;
    case VBR_PROBE_LDS_TR_B64:
        hipLaunchKernelGGL(probe_lds<VBR_PROBE_LDS_TR_B64>, dim3(blocks), dim3(kProbeThreads), 0, stream, (int *)buf_dev, iters);
        *work = waves * iters * 8 * 64.0 * 8;
        break;
    case VBR_PROBE_LDS_B64:
        hipLaunchKernelGGL(probe_lds<VBR_PROBE_LDS_B64>, dim3(blocks), dim3(kProbeThreads), 0, stream, (int *)buf_dev, iters);
        *work = waves * iters * 8 * 64.0 * 8;
        break;
    case VBR_PROBE_LDS_B128:
        hipLaunchKernelGGL(probe_lds<VBR_PROBE_LDS_B128>, dim3(blocks), dim3(kProbeThreads), 0, stream, (int *)buf_dev, iters);
        *work = waves * iters * 8 * 64.0 * 16;
        break;
    case VBR_PROBE_LDS_DMA: {
        // the region the loads walk: the largest power of two inside the buffer, at most 2 MiB
        // (stays in every L2), behind the first 256 bytes (the result word)
        uint32_t span = 1u << 20;
        while (span < (2u << 20) && (int64_t)span * 2 + 8192 + 256 <= buf_bytes) span *= 2;
        if ((int64_t)span + 8192 + 256 + 1024 > buf_bytes) return VBR_EINVAL;
        hipLaunchKernelGGL(probe_dma, dim3(blocks), dim3(kProbeThreads), 0, stream,
                           (const unsigned char *)buf_dev + 256, span - 1, (int *)buf_dev, iters);
        *work = waves * iters * 8 * 1024.0;
        break;
    }
    case VBR_PROBE_HBM_COPY: {
        const int64_t half = (buf_bytes / 2) & ~(int64_t)255;
        hipLaunchKernelGGL(probe_copy, dim3(cus * 8), dim3(kProbeThreads), 0, stream,
                           (const float4v *)buf_dev, (float4v *)((char *)buf_dev + half), half / 16);
        *work = 2.0 * (double)half;      // bytes read + bytes written
        break;
    }
    default:
        return VBR_EINVAL;
    }
    e = hipGetLastError();
    if (e != hipSuccess) { set_last_hip_error((int)e); return VBR_EHIP; }
    return VBR_OK;
}
