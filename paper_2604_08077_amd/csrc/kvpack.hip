// Cube-major packed copy of K and V (Alg. 1 "Reshape K,V into Cubes").
//
// kv_pack_kernel gathers K and V from raster token order into a cube-major tiled copy in the workspace, one
// 64-key tile per workgroup (layout and swizzle: kvtile.h).  Ranks beyond a (clipped) cube's size are
// zero-filled; the attention kernel masks them.  A table of the cubes' sizes follows the two copies.  The natural
// copy of K is stored as fp16, the form the score products take it in (attn_tile.h).  HBM-bound:
// K and V are read once and written once.
#include "attn_tile.h"

namespace adaspark {

// F16: the natural copy (the first operand's) is written as fp16 -- the score operand of the attention kernels
// (attn_tile.h: exact within fp16's range, saturating beyond it); otherwise as the bf16 it is.
template <int D, bool F16>
__global__ __launch_bounds__(256) void kv_pack_kernel(Geom g, const uint16_t *__restrict__ K,
                                                      const uint16_t *__restrict__ V, uint16_t *__restrict__ Kp,
                                                      uint16_t *__restrict__ Vt, int32_t *__restrict__ csize)
{
    constexpr int CPR = D / 8;  // 16-byte chunks per key row
    __shared__ __attribute__((aligned(16))) uint16_t vs[KEY_TILE][D + 8];
    const int t = blockIdx.x, c = blockIdx.y, kv = blockIdx.z;
    const CubeBox box = cube_box(g, c);
    const int size = box.size();
    if (t == 0 && kv == 0 && threadIdx.x == 0) csize[c] = size;  // table of (clipped) cube sizes for the readers
    const size_t tile_base = ((((size_t)kv * g.N + c) * g.TPC) + t) * (size_t)(KEY_TILE * D);

    for (int x = threadIdx.x; x < KEY_TILE * CPR; x += 256) {
        const int k = x / CPR, col = x % CPR;
        const int rank = KEY_TILE * t + k;
        uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (rank < size) {
            const int n = token_of(g, box, rank);
            const size_t src = ((size_t)n * g.Hkv + kv) * D + col * 8;
            kk = *reinterpret_cast<const uint4 *>(K + src);
            vv = *reinterpret_cast<const uint4 *>(V + src);
        }
        if (F16) kk = __builtin_bit_cast(uint4, score_operand(__builtin_bit_cast(bf16x8, kk), 1.0f));
        *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Kp + tile_base) + k_tile_off<D>(k, col)) = kk;
        *reinterpret_cast<uint4 *>(&vs[k][col * 8]) = vv;
    }
    __syncthreads();
    for (int x = threadIdx.x; x < D * (KEY_TILE / 8); x += 256) {
        const int d = x / (KEY_TILE / 8), kc = x % (KEY_TILE / 8);
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)vs[kc * 8 + 2 * e][d] | ((uint32_t)vs[kc * 8 + 2 * e + 1][d] << 16);
        *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Vt + tile_base) + vt_tile_off(d, kc)) =
            make_uint4(w[0], w[1], w[2], w[3]);
    }
}

size_t attn_workspace_bytes(const Geom &g)
{
    // Kp and Vt: [Hkv][N][TPC][64][D] bf16 each, then the cube sizes: int32 [N], then 16 bytes of scratch for the
    // attention entries (kernel choice flag)
    return 2 * (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * g.D * sizeof(uint16_t) + (((size_t)g.N * 4 + 15) / 16) * 16 + 16;
}

template <int D, bool F16>
static hipError_t launch_pack_d(const Geom &g, const uint16_t *K, const uint16_t *V, void *ws, hipStream_t st)
{
    uint16_t *Kp = reinterpret_cast<uint16_t *>(ws);
    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    uint16_t *Vt = Kp + half_elems;
    int32_t *csize = reinterpret_cast<int32_t *>(Vt + half_elems);
    hipLaunchKernelGGL((kv_pack_kernel<D, F16>), dim3(g.TPC, g.N, g.Hkv), dim3(256), 0, st, g, K, V, Kp, Vt, csize);
    return hipGetLastError();
}

hipError_t launch_kv_pack(const Geom &g, const uint16_t *K, const uint16_t *V, void *ws, bool natural_f16, hipStream_t st)
{
    if (g.D == 64) return natural_f16 ? launch_pack_d<64, true>(g, K, V, ws, st) : launch_pack_d<64, false>(g, K, V, ws, st);
    return natural_f16 ? launch_pack_d<128, true>(g, K, V, ws, st) : launch_pack_d<128, false>(g, K, V, ws, st);
}

}  // namespace adaspark
