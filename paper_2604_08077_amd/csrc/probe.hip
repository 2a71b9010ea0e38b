// Two measurement probes for the benchmark: what this GPU actually sustains, to set next to the datasheet peaks.
//   probe_copy  a plain streaming copy (16 bytes per lane and trip, grid-stride): the HBM rate a kernel with nothing
//               else to do reaches, reads and writes together;
//   probe_mfma  back-to-back mfma_f32_16x16x32_bf16 on eight independent accumulators per wavefront, two wavefronts
//               per SIMD on every CU: the rate of the instruction the attention and FFN kernels are built from.
// Neither is part of the method; they touch only the buffers they are given.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/adaspark.h"

namespace {

typedef unsigned int probe_u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_copy_kernel(probe_u32x4 *__restrict__ dst, const probe_u32x4 *__restrict__ src,
                                                         size_t chunks)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < chunks; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

constexpr int PROBE_MFMA_THREADS = 512;  // two wavefronts per SIMD
constexpr int PROBE_MFMA_PER_TRIP = 16;

__global__ __launch_bounds__(PROBE_MFMA_THREADS) void probe_mfma_kernel(float *__restrict__ out, int trips)
{
    probe_bf16x8 a, b;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        a[t] = (__bf16)1.0f;
        b[t] = (__bf16)(0.001f * (float)(threadIdx.x & 63));
    }
    probe_f32x4 c[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) c[t] = probe_f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < trips; ++i) {
#pragma unroll
        for (int r = 0; r < PROBE_MFMA_PER_TRIP / 8; ++r)
#pragma unroll
            for (int t = 0; t < 8; ++t) c[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[t], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) s += c[t][0] + c[t][1] + c[t][2] + c[t][3];
    // one value per workgroup, so that the accumulators are live; out has room for gridDim.x floats
    if (threadIdx.x == 0) out[blockIdx.x] = s;
}

}  // namespace

extern "C" {

int adaspark_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (dst == nullptr || src == nullptr || (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u) ||
        bytes == 0 || (bytes & 15u))
        return ADASPARK_EINVAL;
    const uintptr_t d0 = reinterpret_cast<uintptr_t>(dst), s0 = reinterpret_cast<uintptr_t>(src);
    if (d0 < s0 + bytes && s0 < d0 + bytes) return ADASPARK_EINVAL;  // the buffers must not overlap
    hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<probe_u32x4 *>(dst), static_cast<const probe_u32x4 *>(src), bytes / 16);
    return hipGetLastError() == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

int adaspark_probe_mfma(float *out, int32_t workgroups, int32_t trips, double *flops, void *stream)
{
    if (out == nullptr || (reinterpret_cast<uintptr_t>(out) & 15u) || workgroups <= 0 || workgroups > 65536 || trips <= 0 ||
        trips > (1 << 24))
        return ADASPARK_EINVAL;
    if (flops != nullptr)  // 16 x 16 x 32 multiply-adds per instruction and wavefront
        *flops = 2.0 * 16 * 16 * 32 * PROBE_MFMA_PER_TRIP * (double)trips * (PROBE_MFMA_THREADS / 64) * (double)workgroups;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)workgroups), dim3(PROBE_MFMA_THREADS), 0,
                       static_cast<hipStream_t>(stream), out, trips);
    return hipGetLastError() == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

}  // extern "C"
