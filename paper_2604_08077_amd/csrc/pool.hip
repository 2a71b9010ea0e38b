// Cube mean keys (Eq. 1: k-bar_j = Mean(k in K_j)).
//
// One workgroup per cube.  A token's KV heads are contiguous in memory
// (Hkv*D bf16), so the workgroup reads whole token rows: thread = (token slot,
// 16-byte chunk of the row); slots stride over the cube's tokens, the partial
// sums of the slots are combined through LDS in a fixed order (the result does
// not depend on scheduling).  HBM-bound: K is read exactly once.
#include "geom.h"

namespace adaspark {

constexpr int POOL_THREADS = 1024;  // 16 wavefronts: one workgroup (one cube) per CU has to keep that CU's share of HBM busy

__global__ __launch_bounds__(POOL_THREADS) void cube_pool_kernel(Geom g, const uint16_t *__restrict__ K,
                                                                 float *__restrict__ kbar)
{
    __shared__ float part[POOL_THREADS * 8];
    const int c = blockIdx.x;
    const CubeBox box = cube_box(g, c);
    const int size = box.size();
    const int row_elems = g.Hkv * g.D;  // elements per token row
    const int chunks = row_elems / 8;   // 16-byte chunks per row

    for (int chunk0 = 0; chunk0 < chunks; chunk0 += POOL_THREADS) {
        const int lanes = min(chunks - chunk0, POOL_THREADS);  // chunks handled in this sweep
        const int slots = POOL_THREADS / lanes;                // token slots working in parallel
        const int slot = threadIdx.x / lanes, col = threadIdx.x % lanes;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        if (slot < slots) {
            // eight independent 16-byte loads in flight per thread: a cube is read by one workgroup, so the
            // memory-level parallelism has to come from inside it
            constexpr int UNROLL = 8;
            for (int r0 = slot; r0 < size; r0 += slots * UNROLL) {
                uint4 v[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const int r = r0 + u * slots;
                    v[u] = make_uint4(0, 0, 0, 0);
                    if (r < size) {
                        const int n = token_of(g, box, r);
                        v[u] = *reinterpret_cast<const uint4 *>(K + (size_t)n * row_elems + (size_t)(chunk0 + col) * 8);
                    }
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[2 * e] += __uint_as_float(w[e] << 16);
                        acc[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
                    }
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) part[threadIdx.x * 8 + e] = acc[e];
        __syncthreads();
        if (threadIdx.x < lanes) {
            float sum[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] = 0.f;
            for (int s2 = 0; s2 < slots; ++s2)
#pragma unroll
                for (int e = 0; e < 8; ++e) sum[e] += part[(s2 * lanes + threadIdx.x) * 8 + e];
            float *dst = kbar + (size_t)c * row_elems + (size_t)(chunk0 + threadIdx.x) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e] = sum[e] / (float)size;
        }
        __syncthreads();
    }
}

hipError_t launch_cube_pool(const Geom &g, const uint16_t *K, float *kbar, hipStream_t st)
{
    hipLaunchKernelGGL(cube_pool_kernel, dim3(g.N), dim3(POOL_THREADS), 0, st, g, K, kbar);
    return hipGetLastError();
}

}  // namespace adaspark
