// Sparse (Eq. 3 + own-cube rule, Sec. 3.2) and dense causal attention.
//
// Pass 1 (kv_pack_kernel): K and V are gathered from raster token order into a
// cube-major tiled copy in the workspace, one 64-key tile at a time:
//     Kp[kv][cube][tile][64 keys][D]      keys in rank order, rows as in K
//     Vt[kv][cube][tile][D][64 keys]      transposed, so a PV operand is 16 contiguous bytes
// Ranks beyond a (clipped) cube's size are zero-filled and masked in pass 2.
//
// Pass 2 (attn_kernel): flash attention with the query tile stationary.  A
// workgroup owns 128 consecutive ranks of one query cube for one query head
// (4 wavefronts x 32 rows).  It walks the key cubes j <= i; for j < i a row
// takes part only if bit j of its selection mask is set (dense mode: always),
// for j == i the causal mask inside the cube applies.  Per 64-key tile a
// wavefront computes S^T = K.Q^T with 32x32x16 bf16 MFMA (keys on the M side,
// query rows on the N side, so a lane owns one query row and the softmax
// statistics need one cross-half exchange), keeps fp32 online-softmax state
// per row, rounds P to bf16 and accumulates O^T = V^T.P^T with the same MFMA.
#include "geom.h"

namespace adaspark {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int ATTN_THREADS = 256;
constexpr int ROWS_PER_WAVE = 32;
constexpr int ROWS_PER_BLOCK = 128;
constexpr int MAX_MASK_WORDS = ADASPARK_MAX_CUBES / 32;

// ------------------------------------------------------------------------------------------------ pass 1
template <int D>
__global__ __launch_bounds__(256) void kv_pack_kernel(Geom g, const uint16_t *__restrict__ K,
                                                      const uint16_t *__restrict__ V, uint16_t *__restrict__ Kp,
                                                      uint16_t *__restrict__ Vt)
{
    constexpr int CPR = D / 8;  // 16-byte chunks per key row
    __shared__ __attribute__((aligned(16))) uint16_t vs[KEY_TILE][D + 8];
    const int t = blockIdx.x, c = blockIdx.y, kv = blockIdx.z;
    const CubeBox box = cube_box(g, c);
    const int size = box.size();
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
        *reinterpret_cast<uint4 *>(Kp + tile_base + (size_t)k * D + col * 8) = kk;
        *reinterpret_cast<uint4 *>(&vs[k][col * 8]) = vv;
    }
    __syncthreads();
    for (int x = threadIdx.x; x < D * (KEY_TILE / 8); x += 256) {
        const int d = x / (KEY_TILE / 8), kc = x % (KEY_TILE / 8);
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)vs[kc * 8 + 2 * e][d] | ((uint32_t)vs[kc * 8 + 2 * e + 1][d] << 16);
        *reinterpret_cast<uint4 *>(Vt + tile_base + (size_t)d * KEY_TILE + kc * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// ------------------------------------------------------------------------------------------------ pass 2
// Exchange between lane l and lane l^32: returns the partner's value.
__device__ inline float other_half(float x)
{
    return __shfl_xor(x, 32, 64);
}

// MFMA M-row m (0..31) of an S^T tile carries key kappa(m) of the 32-key group, chosen so that after the
// MFMA a lane's registers 8s..8s+7 hold keys 16s+8h..16s+8h+7 (h = lane/32): exactly the operand order the
// P.V MFMA wants, with no shuffle.  kappa swaps bits 2 and 3 of m.
__device__ inline int kappa(int m) { return (m & 0x13) | ((m & 8) >> 1) | ((m & 4) << 1); }

template <int D, bool SPARSE>
__global__ __launch_bounds__(ATTN_THREADS) void attn_kernel(Geom g, const uint16_t *__restrict__ Q,
                                                            const uint16_t *__restrict__ Kp,
                                                            const uint16_t *__restrict__ Vt,
                                                            const uint32_t *__restrict__ sel_mask,
                                                            uint16_t *__restrict__ O, float *__restrict__ lse)
{
    constexpr int KROW = D + 8;         // padded LDS row of the K tile (bf16 elements)
    constexpr int VROW = KEY_TILE + 8;  // padded LDS row of the V^T tile
    constexpr int KSTEPS = D / 16;      // MFMA k-steps of S^T
    constexpr int DTILES = D / 32;      // 32-wide output tiles of O^T
    __shared__ __attribute__((aligned(16))) uint16_t k_lds[KEY_TILE * KROW];
    __shared__ __attribute__((aligned(16))) uint16_t v_lds[D * VROW];
    __shared__ uint32_t union_mask[SPARSE ? MAX_MASK_WORDS : 1];

    // workgroup -> (query cube, query head, 128-rank chunk); late (long) cubes are scheduled first
    const int chunks_per_cube = (g.Cmax + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    int bid = blockIdx.x;
    const int chunk = bid % chunks_per_cube;
    bid /= chunks_per_cube;
    const int a = bid % g.Hq;
    bid /= g.Hq;
    const int i = g.N - 1 - bid;
    const int kv = a / g.G;
    const CubeBox qbox = cube_box(g, i);
    const int qsize = qbox.size();
    if (chunk * ROWS_PER_BLOCK >= qsize) return;  // uniform for the workgroup

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n32 = lane & 31, h = lane >> 5;
    const int wave_min_rank = chunk * ROWS_PER_BLOCK + wave * ROWS_PER_WAVE;
    const int wave_max_rank = wave_min_rank + ROWS_PER_WAVE - 1;
    const int block_max_rank = min(chunk * ROWS_PER_BLOCK + ROWS_PER_BLOCK, qsize) - 1;
    const int rank = wave_min_rank + n32;
    const bool row_ok = rank < qsize;
    const int tok = token_of(g, qbox, row_ok ? rank : 0);
    const size_t row = (size_t)tok * g.Hq + a;
    const uint32_t *mrow = SPARSE ? sel_mask + row * g.words : nullptr;

    if (SPARSE) {
        for (int w = threadIdx.x; w < g.words; w += ATTN_THREADS) union_mask[w] = 0;
        __syncthreads();
        if (row_ok && h == 0)
            for (int w = 0; w < g.words; ++w) {
                const uint32_t bits = mrow[w];
                if (bits) atomicOr(&union_mask[w], bits);
            }
        __syncthreads();
    }

    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int c = 0; c < KSTEPS; ++c) qf[c] = *reinterpret_cast<const bf16x8 *>(Q + row * D + 16 * c + 8 * h);

    f32x16 o[DTILES];
#pragma unroll
    for (int e = 0; e < DTILES; ++e)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[e][v] = 0.f;
    float m_run = -1e30f, l_run = 0.f;
    const float c2 = 1.44269504088896340736f / sqrtf((float)D);

    const int krow_sel = kappa(n32);

    for (int j = 0; j <= i; ++j) {
        const bool own = (j == i);
        if (SPARSE && !own && !((union_mask[j >> 5] >> (j & 31)) & 1u)) continue;  // no row here selected cube j
        const int jsize = own ? qsize : cube_box(g, j).size();
        bool sel = row_ok;
        if (SPARSE && !own) sel = sel && ((mrow[j >> 5] >> (j & 31)) & 1u);
        const bool wave_active = __ballot(sel) != 0ull;
        // last key rank this row may see in cube j (-1: none)
        const int lim = !sel ? -1 : (own ? min(rank, jsize - 1) : jsize - 1);
        int ntiles = (jsize + KEY_TILE - 1) / KEY_TILE;
        if (own) ntiles = min(ntiles, block_max_rank / KEY_TILE + 1);
        const size_t cube_base = (((size_t)kv * g.N + j) * g.TPC) * (size_t)(KEY_TILE * D);

        for (int t = 0; t < ntiles; ++t) {
            __syncthreads();  // previous tile fully consumed
            {
                const uint16_t *ksrc = Kp + cube_base + (size_t)t * (KEY_TILE * D);
                const uint16_t *vsrc = Vt + cube_base + (size_t)t * (KEY_TILE * D);
#pragma unroll
                for (int x = threadIdx.x; x < KEY_TILE * D / 8; x += ATTN_THREADS) {
                    const int kr = x / (D / 8), kc = x % (D / 8);
                    *reinterpret_cast<uint4 *>(&k_lds[kr * KROW + kc * 8]) = *reinterpret_cast<const uint4 *>(ksrc + x * 8);
                    const int vr = x / (KEY_TILE / 8), vc = x % (KEY_TILE / 8);
                    *reinterpret_cast<uint4 *>(&v_lds[vr * VROW + vc * 8]) = *reinterpret_cast<const uint4 *>(vsrc + x * 8);
                }
            }
            __syncthreads();
            if (!wave_active) continue;
            const int key0 = KEY_TILE * t;
            if (own && key0 > wave_max_rank) continue;

            // S^T = K . Q^T for 64 keys x 32 rows
            f32x16 s[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) s[mt][v] = 0.f;
                const uint16_t *kb = &k_lds[(32 * mt + krow_sel) * KROW + 8 * h];
#pragma unroll
                for (int c = 0; c < KSTEPS; ++c) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8 *>(kb + 16 * c);
                    s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, qf[c], s[mt], 0, 0, 0);
                }
            }
            // register v = 8*sl + tt of s[mt] holds key rank key0 + 32*mt + 16*sl + 8*h + tt
            const bool need_mask = __ballot(lim < key0 + KEY_TILE - 1) != 0ull;
            if (need_mask) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int kr = key0 + 32 * mt + 16 * (v >> 3) + 8 * h + (v & 7);
                        if (kr > lim) s[mt][v] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[mt][v]);
            mx = fmaxf(mx, other_half(mx));
            const float m_new = fmaxf(m_run, mx * c2);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            float rs = 0.f;
            bf16x8 pf[4];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[mt][v], c2, -m_new));
                    rs += p;
                    pf[2 * mt + (v >> 3)][v & 7] = (__bf16)p;
                }
            rs += other_half(rs);
            l_run = l_run * alpha + rs;
            m_run = m_new;
#pragma unroll
            for (int e = 0; e < DTILES; ++e)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[e][v] *= alpha;
            // O^T += V^T . P^T
#pragma unroll
            for (int e = 0; e < DTILES; ++e) {
                const uint16_t *vb = &v_lds[(32 * e + n32) * VROW + 8 * h];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8 *>(vb + 16 * ks);
                    o[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pf[ks], o[e], 0, 0, 0);
                }
            }
        }
    }

    if (row_ok) {
        const float inv = 1.0f / l_run;
        uint16_t *orow = O + row * D;
#pragma unroll
        for (int e = 0; e < DTILES; ++e)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                // registers 4b..4b+3 of tile e hold d = 32e + 8b + 4h + (0..3)
                uint32_t w0 = (uint32_t)float_to_bf16_bits(o[e][4 * b] * inv) |
                              ((uint32_t)float_to_bf16_bits(o[e][4 * b + 1] * inv) << 16);
                uint32_t w1 = (uint32_t)float_to_bf16_bits(o[e][4 * b + 2] * inv) |
                              ((uint32_t)float_to_bf16_bits(o[e][4 * b + 3] * inv) << 16);
                *reinterpret_cast<uint2 *>(orow + 32 * e + 8 * b + 4 * h) = make_uint2(w0, w1);
            }
        if (lse != nullptr && h == 0) lse[row] = (m_run + log2f(l_run)) * 0.69314718055994530942f;
    }
}

size_t attn_workspace_bytes(const Geom &g)
{
    // Kp and Vt: [Hkv][N][TPC][64][D] bf16 each
    return 2 * (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * g.D * sizeof(uint16_t);
}

template <int D>
static hipError_t launch_pack_d(const Geom &g, const uint16_t *K, const uint16_t *V, void *ws, hipStream_t st)
{
    uint16_t *Kp = reinterpret_cast<uint16_t *>(ws);
    uint16_t *Vt = Kp + (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    hipLaunchKernelGGL((kv_pack_kernel<D>), dim3(g.TPC, g.N, g.Hkv), dim3(256), 0, st, g, K, V, Kp, Vt);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_attn_d(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                                uint16_t *O, float *lse, hipStream_t st)
{
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const uint16_t *Vt = Kp + (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const int chunks_per_cube = (g.Cmax + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    const dim3 grid((unsigned)((size_t)g.N * g.Hq * chunks_per_cube));
    if (sel_mask != nullptr)
        hipLaunchKernelGGL((attn_kernel<D, true>), grid, dim3(ATTN_THREADS), 0, st, g, Q, Kp, Vt, sel_mask, O, lse);
    else
        hipLaunchKernelGGL((attn_kernel<D, false>), grid, dim3(ATTN_THREADS), 0, st, g, Q, Kp, Vt, sel_mask, O, lse);
    return hipGetLastError();
}

hipError_t launch_kv_pack(const Geom &g, const uint16_t *K, const uint16_t *V, void *ws, hipStream_t st)
{
    if (g.D == 64) return launch_pack_d<64>(g, K, V, ws, st);
    return launch_pack_d<128>(g, K, V, ws, st);
}

hipError_t launch_attn(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask, uint16_t *O,
                       float *lse, hipStream_t st)
{
    if (g.D == 64) return launch_attn_d<64>(g, Q, packed, sel_mask, O, lse, st);
    return launch_attn_d<128>(g, Q, packed, sel_mask, O, lse, st);
}

}  // namespace adaspark
