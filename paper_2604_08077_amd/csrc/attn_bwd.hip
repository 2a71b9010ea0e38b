// Backward pass of cube-selective attention (Eq. 3 differentiated; the selected sets are constants).
//
// For a row r with attended keys A_r, scale c = 1/sqrt(D):  p = softmax(c q.k),  delta = dO.O,
//     dV_j += p_j dO,   dS_j = p_j (dO.v_j - delta),   dQ = c sum_j dS_j k_j,   dK_j += c dS_j q.
// p is rebuilt from the forward's log-sum-exp, so nothing of the forward's size is stored.  Three MFMA kernels, none
// of which needs a transposition in registers or an atomic:
//   attn_bwd_dq_kernel   row-stationary (like the forward's masked walk): a wavefront keeps Q and dO of 32 rows as
//                        MFMA B operands, walks the key tiles of every cube up to its own, and accumulates dQ^T.
//                        S^T = K.Q^T, dP^T = V.dO^T, dQ^T += K^T.dS^T.
//   attn_bwd_dkv_kernel  key-stationary: a wavefront keeps K (and V) of 32 keys as B operands, walks the 64-row
//                        tiles of every later cube and its own, and accumulates dV^T (WHICH = 0: S = Q.K^T,
//                        dV^T += dO^T.P) or dK^T (WHICH = 1: S, dP = dO.V^T, dK^T += Q^T.dS).  Two passes because the
//                        two accumulators together with both operand sets do not fit the register file.
// In both, a row's selection bit for the key cube acts as a mask (dense work, like the forward's masked walk).
// Streamed tiles come from packed, pre-swizzled copies (kvtile.h layouts) straight into LDS: K natural / V natural
// / K transposed per 64 keys (two runs of the forward's pack kernel), Q, dO natural and transposed per 64 rows in
// (cube, rank, head of the group) order (bwd_pack_rows_kernel).
// The score products take Q and K as they are (bf16 x bf16 -> fp32: exact products, so the rebuilt probabilities
// carry nothing but their own rounding, whatever the size of the scores) and their accumulators start from
// -lse * sqrt(D), -inf for a row that did not select the key cube: the accumulator times the softmax scale in base
// 2 is then the exponent of the probability, and the selection costs no instruction per score.  The dP accumulators
// start from minus delta.  bwd_pack_rows_kernel leaves both start values per packed row.
#include <algorithm>
#include <type_traits>

#include "attn_tile.h"

namespace adaspark {

constexpr int BWD_THREADS = 512;
constexpr int BWD_ROWS = 256;   // rows (dQ kernel) or keys (dK/dV kernel) per workgroup: 8 wavefronts x 2 x 16
constexpr float BWD_LOG2E = 1.44269504088896340736f;

struct BwdWorkspace {
    void *packA;             // launch_kv_pack(K, V): natural K first (its V^T half is not used here)
    void *packB;             // launch_kv_pack(V, K): natural V, then K transposed
    uint16_t *Qn, *Qt, *dOn, *dOt;  // [Hkv][N][tpcr][64 * D]
    // -lse * sqrt(D) and -delta per packed row (what the score and dP products start from)
    float *lse2, *delta;     // [Hkv][N][tpcr * 64]; padding rows: -inf, 0
    unsigned long long *colmask;  // [Hkv][N (key cube j)][N (row cube i)][tpcr]: bit k = row 64 t + k of cube i selects j
    int tpcr;                // 64-row tiles per cube = ceil(Cmax * G / 64)
    size_t bytes;
};

BwdWorkspace bwd_workspace(const Geom &g, void *ws)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    BwdWorkspace w;
    unsigned char *p = static_cast<unsigned char *>(ws);
    w.tpcr = (g.Cmax * g.G + 63) / 64;
    const size_t tile_elems = (size_t)g.Hkv * g.N * w.tpcr * 64 * g.D;
    size_t off = 0;
    w.packA = p + off; off = up(off + attn_workspace_bytes(g));
    w.packB = p + off; off = up(off + attn_workspace_bytes(g));
    w.Qn = reinterpret_cast<uint16_t *>(p + off); off = up(off + tile_elems * 2);
    w.Qt = reinterpret_cast<uint16_t *>(p + off); off = up(off + tile_elems * 2);
    w.dOn = reinterpret_cast<uint16_t *>(p + off); off = up(off + tile_elems * 2);
    w.dOt = reinterpret_cast<uint16_t *>(p + off); off = up(off + tile_elems * 2);
    w.lse2 = reinterpret_cast<float *>(p + off); off = up(off + (size_t)g.Hkv * g.N * w.tpcr * 64 * 4);
    w.delta = reinterpret_cast<float *>(p + off); off = up(off + (size_t)g.Hkv * g.N * w.tpcr * 64 * 4);
    w.colmask = reinterpret_cast<unsigned long long *>(p + off); off = up(off + (size_t)g.Hkv * g.N * g.N * w.tpcr * 8);
    w.bytes = off;
    return w;
}

size_t attn_bwd_workspace_bytes(const Geom &g) { return bwd_workspace(g, nullptr).bytes; }

// Workgroup -> (KV head, slot among the head's workgroups).  Consecutive workgroups go to different XCDs, each with
// its own L2; the workgroups of one KV head stream the same tiles, so where the head count allows a head's
// workgroups stay on as few XCDs as possible.  bwd_grid is the matching launch size.
__host__ __device__ inline bool bwd_head_slot(int b, int Hkv, int per_head, int &kv, int &slot)
{
    if (Hkv <= 8 && 8 % Hkv == 0) {
        const int x = b & 7, idx = b >> 3, share = 8 / Hkv;
        kv = x % Hkv;
        slot = idx * share + x / Hkv;
    } else if (Hkv % 8 == 0) {
        const int x = b & 7, idx = b >> 3, m = Hkv / 8;
        kv = x + 8 * (idx % m);
        slot = idx / m;
    } else {
        kv = b % Hkv;
        slot = b / Hkv;
    }
    return slot < per_head;
}
inline unsigned bwd_grid(int Hkv, int per_head)
{
    if (Hkv <= 8 && 8 % Hkv == 0) return (unsigned)((per_head + 8 / Hkv - 1) / (8 / Hkv) * 8);
    return (unsigned)per_head * (unsigned)Hkv;
}

// One wavefront copies 64 dwords from global memory straight into LDS: lane l moves the 4 bytes at sbase + voff to
// lds_addr + 4*l.
__device__ __forceinline__ void dma_dword_s(uint32_t lds_addr, const void *sbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Row r of cube c in the packed row order: rank r / G, head r % G of the group.
// Q, dO natural and transposed per 64-row tile; deltap = -dO.O; lse2p = -lse * sqrt(D) (-inf for padding rows).
template <int D>
__global__ __launch_bounds__(256) void bwd_pack_rows_kernel(Geom g, const uint16_t *__restrict__ Q,
                                                            const uint16_t *__restrict__ dO,
                                                            const uint16_t *__restrict__ O, const float *__restrict__ lse,
                                                            int tpcr, uint16_t *__restrict__ Qn, uint16_t *__restrict__ Qt,
                                                            uint16_t *__restrict__ dOn, uint16_t *__restrict__ dOt,
                                                            float *__restrict__ lse2p, float *__restrict__ deltap)
{
    constexpr int CPR = D / 8;
    __shared__ __attribute__((aligned(16))) uint16_t qs[64][D + 8];
    __shared__ __attribute__((aligned(16))) uint16_t gs[64][D + 8];
    const int t = blockIdx.x, c = blockIdx.y, kv = blockIdx.z;
    const CubeBox box = cube_box(g, c);
    const int mrows = box.size() * g.G;
    const size_t tile = (((size_t)kv * g.N + c) * tpcr) + t;
    const size_t tile_base = tile * (size_t)(64 * D);
    for (int x = threadIdx.x; x < 64 * CPR; x += 256) {
        const int k = x / CPR, col = x % CPR;
        const int r = 64 * t + k;
        uint4 qq = make_uint4(0, 0, 0, 0), gg = make_uint4(0, 0, 0, 0);
        float part = 0.f, l2 = INFINITY;  // (padding rows: minus its log-sum-exp is -inf, its probabilities 0)
        if (r < mrows) {
            const int n = token_of(g, box, r / g.G);
            const size_t rowid = (size_t)n * g.Hq + kv * g.G + r % g.G;
            const size_t src = rowid * D + col * 8;
            qq = *reinterpret_cast<const uint4 *>(Q + src);
            gg = *reinterpret_cast<const uint4 *>(dO + src);
            const uint4 oo = *reinterpret_cast<const uint4 *>(O + src);
            const uint32_t gw[4] = {gg.x, gg.y, gg.z, gg.w}, ow[4] = {oo.x, oo.y, oo.z, oo.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                part = fmaf(__uint_as_float(gw[e] << 16), __uint_as_float(ow[e] << 16), part);
                part = fmaf(__uint_as_float(gw[e] & 0xffff0000u), __uint_as_float(ow[e] & 0xffff0000u), part);
            }
            l2 = lse[rowid] * sqrtf((float)D);  // = (lse in base 2) / (softmax scale in base 2)
        }
#pragma unroll
        for (int d = CPR / 2; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
        if (col == 0) {  // both with the sign the MFMA accumulators of the key-stationary kernels start from
            lse2p[tile * 64 + k] = -l2;
            deltap[tile * 64 + k] = -part;
        }
        *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Qn + tile_base) + k_tile_off<D>(k, col)) = qq;
        *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(dOn + tile_base) + k_tile_off<D>(k, col)) = gg;
        *reinterpret_cast<uint4 *>(&qs[k][col * 8]) = qq;
        *reinterpret_cast<uint4 *>(&gs[k][col * 8]) = gg;
    }
    __syncthreads();
    for (int x = threadIdx.x; x < D * 8; x += 256) {
        const int d = x / 8, kc = x % 8;
        uint32_t wq[4], wg[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            wq[e] = (uint32_t)qs[kc * 8 + 2 * e][d] | ((uint32_t)qs[kc * 8 + 2 * e + 1][d] << 16);
            wg[e] = (uint32_t)gs[kc * 8 + 2 * e][d] | ((uint32_t)gs[kc * 8 + 2 * e + 1][d] << 16);
        }
        *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Qt + tile_base) + vt_tile_off(d, kc)) =
            make_uint4(wq[0], wq[1], wq[2], wq[3]);
        *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(dOt + tile_base) + vt_tile_off(d, kc)) =
            make_uint4(wg[0], wg[1], wg[2], wg[3]);
    }
}

// The selection bits transposed for the key-stationary kernels: one wavefront per (KV head, row cube i, row tile t);
// lane k holds row 64 t + k's mask words, a ballot per cube turns 64 rows' bits into one 64-bit word.
__global__ __launch_bounds__(64) void bwd_colmask_kernel(Geom g, const uint32_t *__restrict__ sel_mask, int tpcr,
                                                        unsigned long long *__restrict__ colmask)
{
    const int t = blockIdx.x, i = blockIdx.y, kv = blockIdx.z;
    const int lane = threadIdx.x;
    const CubeBox box = cube_box(g, i);
    const int r = 64 * t + lane;
    const bool valid = r < box.size() * g.G;
    const size_t rowid = valid ? (size_t)token_of(g, box, r / g.G) * g.Hq + kv * g.G + r % g.G : 0;
    for (int jw = 0; jw < g.words; ++jw) {
        const uint32_t word = valid ? sel_mask[rowid * g.words + jw] : 0u;
        unsigned long long mine = 0ull;
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            const unsigned long long bal = __ballot((word >> b) & 1u);
            if (lane == b) mine = bal;
        }
        const int j = 32 * jw + lane;
        if (lane < 32 && j < g.N) colmask[(((size_t)kv * g.N + j) * g.N + i) * tpcr + t] = mine;
    }
}

// Half H of qk_tile: the products of a natural tile's rows 32 H .. 32 H + 31 with the B operands of NS slabs (OP:
// the operand type, bf16x8).  acc[s][k2][v] belongs to tile row 32 H + 8 q4 + 4 k2 + v.
// Working a tile in two halves keeps half as many accumulators alive.  The accumulators of slab s start from bias[s],
// a value of the slab's row (the lane's column): the products come out with it added.
template <int D, int NS, int H, typename OP>
__device__ __forceinline__ void nat_half_bias(const unsigned char *kt, int n16, int q4, const OP (&bf)[NS][D / 32],
                                              const float (&bias)[NS], f32x4 (&acc)[NS][2])
{
    f32x4 init[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) init[s] = f32x4{bias[s], bias[s], bias[s], bias[s]};
#pragma unroll
    for (int c = 0; c < D / 32; ++c)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            const int krow = 32 * H + 8 * (n16 >> 2) + 4 * k2 + (n16 & 3);
            const OP af = *reinterpret_cast<const OP *>(kt + k_tile_off<D>(krow, 4 * c + q4));
#pragma unroll
            for (int s = 0; s < NS; ++s) acc[s][k2] = mfma16(af, bf[s][c], c == 0 ? init[s] : acc[s][k2]);
        }
}

// The same with the accumulators started from init[k2]: four values, one per tile row 32 H + 8 q4 + 4 k2 + v, shared by
// the slabs (minus a tile row's log-sum-exp or delta: the products then come out with it subtracted).
template <int D, int NS, int H, typename OP>
__device__ __forceinline__ void nat_half_from(const unsigned char *kt, int n16, int q4, const OP (&bf)[NS][D / 32],
                                              const f32x4 (&init)[2], f32x4 (&acc)[NS][2])
{
#pragma unroll
    for (int c = 0; c < D / 32; ++c)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            const int krow = 32 * H + 8 * (n16 >> 2) + 4 * k2 + (n16 & 3);
            const OP af = *reinterpret_cast<const OP *>(kt + k_tile_off<D>(krow, 4 * c + q4));
#pragma unroll
            for (int s = 0; s < NS; ++s) acc[s][k2] = mfma16(af, bf[s][c], c == 0 ? init[k2] : acc[s][k2]);
        }
}

// acc^T[d, n] += T[d, 0..63] . B[0..63, n] for slabs 0..NS-1: T a transposed tile in LDS (rows = head-dim), B in
// registers in the operand order qk_tile's outputs pack into (bf[s][half] = entities 32*half + 8*q4 + 0..7).
template <int D, int NS>
__device__ __forceinline__ void tn_tile(const unsigned char *tt, int n16, int q4, const bf16x8 (&bf)[NS][2],
                                        f32x4 (&acc)[NS][D / 16])
{
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int e = 0; e < D / 16; ++e) {
            const bf16x8 af = *reinterpret_cast<const bf16x8 *>(tt + vt_tile_off(16 * e + n16, 4 * sl + q4));
#pragma unroll
            for (int s = 0; s < NS; ++s)
                acc[s][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bf[s][sl], acc[s][e], 0, 0, 0);
        }
}

// ---------------------------------------------------------------------------------------------------------------
// dQ: workgroup = 256 rows (packed row order) of one (cube i, KV head); late cubes (the long walks) first.
// ---------------------------------------------------------------------------------------------------------------
template <int D, bool MASKED>
__global__ __launch_bounds__(BWD_THREADS) void attn_bwd_dq_kernel(Geom g, const uint16_t *__restrict__ Q,
                                                                  const uint16_t *__restrict__ dO,
                                                                  const uint16_t *__restrict__ Kn,
                                                                  const uint16_t *__restrict__ Vn,
                                                                  const uint16_t *__restrict__ Kt,
                                                                  const int32_t *__restrict__ csize,
                                                                  float *__restrict__ lse2p,
                                                                  const float *__restrict__ deltap, int tpcr,
                                                                  const uint32_t *__restrict__ sel_mask,
                                                                  uint16_t *__restrict__ dQ)
{
    constexpr int NS = 2, KSTEPS = D / 32;
    constexpr int TILE = 64 * D * 2;       // bytes of one tile
    constexpr int STAGE = 3 * TILE;        // K natural, V natural, K transposed
    constexpr int PIECES = TILE / 1024;    // 1 KB pieces per tile
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];

    const int nblk = (g.Cmax * g.G + BWD_ROWS - 1) / BWD_ROWS;
    int kv, slot;
    if (!bwd_head_slot(blockIdx.x, g.Hkv, g.N * nblk, kv, slot)) return;
    const int blk = slot % nblk;
    const int i = g.N - 1 - slot / nblk;
    const CubeBox box = cube_box(g, i);
    const int mrows = box.size() * g.G;
    if (blk * BWD_ROWS >= mrows) return;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n16 = lane & 15, q4 = lane >> 4;

    // the wavefront's rows
    int rr[NS], rank[NS];
    size_t rowid[NS];
    bool valid[NS];
    bf16x8 qf[NS][KSTEPS], gf[NS][KSTEPS];
    float lse2[NS], delta[NS], psum[NS];
    size_t prow[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        psum[s] = 0.f;
        const int r = blk * BWD_ROWS + wave * 32 + s * 16 + n16;
        valid[s] = r < mrows;
        rr[s] = valid[s] ? r : mrows - 1;
        rank[s] = rr[s] / g.G;
        rowid[s] = (size_t)token_of(g, box, rank[s]) * g.Hq + kv * g.G + rr[s] % g.G;
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) {
            qf[s][c] = *reinterpret_cast<const bf16x8 *>(Q + rowid[s] * D + 32 * c + 8 * q4);
            gf[s][c] = *reinterpret_cast<const bf16x8 *>(dO + rowid[s] * D + 32 * c + 8 * q4);
        }
        prow[s] = ((size_t)kv * g.N + i) * tpcr * 64 + rr[s];
        lse2[s] = lse2p[prow[s]];    // -lse * sqrt(D): what the score products start from
        delta[s] = deltap[prow[s]];  // minus delta: what the dP products start from
    }

    const float c2 = BWD_LOG2E / sqrtf((float)D);  // softmax scale in base 2

    // tile stream: cubes 0..i, the tiles of each that hold keys
    const size_t head_tiles = (size_t)kv * g.N * g.TPC;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    auto issue = [&](int stage, int j, int t) __attribute__((always_inline)) {
        const size_t toff = (head_tiles + (size_t)j * g.TPC + t) * (size_t)TILE;
        // every wavefront moves its eighth of each of the three tiles (the tile is a compile-time index: a run-time
        // choice among kernel arguments would be made through a table in scratch memory)
#pragma unroll
        for (int which = 0; which < 3; ++which)
#pragma unroll
            for (int u = 0; u < PIECES / 8; ++u) {
                const int sub = wave * (PIECES / 8) + u;
                const unsigned char *src =
                    reinterpret_cast<const unsigned char *>(which == 0 ? Kn : which == 1 ? Vn : Kt) + toff + sub * 1024;
                dma_1k_s(__builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(stage * STAGE + which * TILE + sub * 1024)),
                         uniform_ptr(src), (uint32_t)(lane * 16));
            }
    };
    auto tiles_of = [&](int j) { return (csize[j] + 63) >> 6; };

    f32x4 acc[NS][D / 16];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int e = 0; e < D / 16; ++e) acc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};

    int ij = 0, it = 0, int_ = tiles_of(0);  // next tile to issue
    issue(0, 0, 0);
    if (++it == int_) { ++ij; it = 0; int_ = ij <= i ? tiles_of(ij) : 0; }
    int stage = 0;
    uint32_t mw[NS] = {0u, 0u};
    for (int j = 0; j <= i; ++j) {
        const int nt = tiles_of(j);
        const int size_j = csize[j];
        // What the score products start from: minus the row's log-sum-exp; -inf for a row that did not select cube
        // j, which then takes no part (probabilities 0)
        float le[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            le[s] = lse2[s];
            if (MASKED && j < i) {
                if ((j & 31) == 0) mw[s] = sel_mask[rowid[s] * g.words + (j >> 5)];
                if (!((mw[s] >> (j & 31)) & 1u)) le[s] = -INFINITY;
            }
        }
        for (int t = 0; t < nt; ++t) {
            tile_barrier();
            if (ij <= i) {
                issue(stage ^ 1, ij, it);
                if (++it == int_) { ++ij; it = 0; int_ = ij <= i ? tiles_of(ij) : 0; }
            }
            const unsigned char *kt = smem + stage * STAGE, *vt = kt + TILE, *ktt = vt + TILE;
            const bool edge = j == i || 64 * t + 64 > size_j;  // the own cube's causal edge, padding keys: few tiles
            bf16x8 ds[NS][2];
            auto half = [&](auto hc) __attribute__((always_inline)) {
                constexpr int H = decltype(hc)::value;
                f32x4 sacc[NS][2], pacc[NS][2];
                nat_half_bias<D, NS, H>(kt, n16, q4, qf, le, sacc);
                nat_half_bias<D, NS, H>(vt, n16, q4, gf, delta, pacc);
                if (edge) {
                    int kb = 64 * t + 32 * H + 8 * q4;
                    asm volatile("" : "+v"(kb));
#pragma unroll
                    for (int s = 0; s < NS; ++s)
#pragma unroll
                        for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const int key = kb + 4 * k2 + v;
                                if (key >= size_j || (j == i && key > rank[s])) sacc[s][k2][v] = -INFINITY;
                            }
                }
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const float p = __builtin_amdgcn_exp2f(sacc[s][k2][v] * c2);
                            psum[s] += p;
                            ds[s][H][4 * k2 + v] = (__bf16)(p * pacc[s][k2][v]);
                        }
            };
            half(std::integral_constant<int, 0>{});
            half(std::integral_constant<int, 1>{});
            tn_tile<D, NS>(ktt, n16, q4, ds, acc);
            stage ^= 1;
        }
    }
    // The probabilities above were built from the caller's log-sum-exp, which the forward kernels give to about
    // 1e-3; their sum over the row says by how much it is off.  dQ is linear in them, so it is divided by the sum
    // here, and the packed log-sum-exp is corrected for the dK / dV kernel that runs next.
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const float total = quad_sum(psum[s]);
        if (!valid[s]) continue;
        if (q4 == 0) lse2p[prow[s]] = lse2[s] - log2f(total) / c2;
        const float scale = 1.0f / (sqrtf((float)D) * total);
#pragma unroll
        for (int e = 0; e < D / 16; ++e) {
            bf16x2 a, b;
            a[0] = (__bf16)(acc[s][e][0] * scale); a[1] = (__bf16)(acc[s][e][1] * scale);
            b[0] = (__bf16)(acc[s][e][2] * scale); b[1] = (__bf16)(acc[s][e][3] * scale);
            uint2 o;
            o.x = *reinterpret_cast<uint32_t *>(&a);
            o.y = *reinterpret_cast<uint32_t *>(&b);
            *reinterpret_cast<uint2 *>(dQ + rowid[s] * D + 16 * e + 4 * q4) = o;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// dV (WHICH = 0) / dK (WHICH = 1): workgroup = 256 keys of one (cube j, KV head); walks the row tiles of cube j
// and of every later cube, from the last one down.  Early cubes (the long walks) first.
// ---------------------------------------------------------------------------------------------------------------
template <int D, int WHICH, bool MASKED>
__global__ __launch_bounds__(BWD_THREADS) void attn_bwd_dkv_kernel(Geom g, const uint16_t *__restrict__ K,
                                                                   const uint16_t *__restrict__ V,
                                                                   const uint16_t *__restrict__ Qn,
                                                                   const uint16_t *__restrict__ Qt,
                                                                   const uint16_t *__restrict__ dOn,
                                                                   const uint16_t *__restrict__ dOt,
                                                                   const float *__restrict__ lse2p,
                                                                   const float *__restrict__ deltap, int tpcr,
                                                                   const int32_t *__restrict__ csize,
                                                                   const unsigned long long *__restrict__ colmask,
                                                                   uint16_t *__restrict__ dOut)
{
    constexpr int NS = 2, KSTEPS = D / 32;
    constexpr int TILE = 64 * D * 2;
    constexpr int NT = WHICH == 0 ? 2 : 3;   // dV: Q natural, dO transposed; dK: Q natural, dO natural, Q transposed
    constexpr int VEC = NT * TILE;           // per row tile: then 64 floats lse2, 64 floats delta
    constexpr int SLOT = VEC + 2 * 256;
    constexpr int TPS = WHICH == 0 ? 2 : 1;  // row tiles per step (per barrier): as many as two stages of them fit
    constexpr int STAGE = TPS * SLOT;
    constexpr int PIECES = TILE / 1024;
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];

    const int nkb = (g.Cmax + BWD_ROWS - 1) / BWD_ROWS;
    int kv, slot;
    if (!bwd_head_slot(blockIdx.x, g.Hkv, g.N * nkb, kv, slot)) return;
    const int kb = slot % nkb;
    const int j = slot / nkb;
    const CubeBox box = cube_box(g, j);
    const int size_j = box.size();
    if (kb * BWD_ROWS >= size_j) return;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n16 = lane & 15, q4 = lane >> 4;

    // the wavefront's keys (B operands)
    int key[NS];
    bool valid[NS];
    size_t krow[NS];
    bf16x8 kf[NS][KSTEPS], vf[NS][KSTEPS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        key[s] = kb * BWD_ROWS + wave * 32 + s * 16 + n16;
        valid[s] = key[s] < size_j;
        krow[s] = ((size_t)token_of(g, box, valid[s] ? key[s] : size_j - 1) * g.Hkv + kv) * D;
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) {
            kf[s][c] = *reinterpret_cast<const bf16x8 *>(K + krow[s] + 32 * c + 8 * q4);
            if (WHICH == 1) vf[s][c] = *reinterpret_cast<const bf16x8 *>(V + krow[s] + 32 * c + 8 * q4);
        }
    }
    const float c2 = BWD_LOG2E / sqrtf((float)D);  // softmax scale in base 2

    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    const size_t head_tiles = (size_t)kv * g.N * tpcr;
    const size_t cm_base = ((size_t)kv * g.N + j) * g.N;
    // row tile t of cube i into slot `slot` of `stage`: the tiles by all wavefronts, the two per-row vectors by
    // wavefront 0
    auto issue_tile = [&](int stage, int slot, int i, int t) __attribute__((always_inline)) {
        const size_t tile = head_tiles + (size_t)i * tpcr + t;
        stage = stage * TPS + slot;  // in units of SLOT
#pragma unroll
        for (int which = 0; which < NT; ++which)
#pragma unroll
            for (int u = 0; u < PIECES / 8; ++u) {
                const int sub = wave * (PIECES / 8) + u;
                const uint16_t *base = WHICH == 0 ? (which == 0 ? Qn : dOt) : (which == 0 ? Qn : which == 1 ? dOn : Qt);
                const unsigned char *src = reinterpret_cast<const unsigned char *>(base) + tile * (size_t)TILE + sub * 1024;
                dma_1k_s(__builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(stage * SLOT + which * TILE + sub * 1024)),
                         uniform_ptr(src), (uint32_t)(lane * 16));
            }
        if (wave == 0) {
            const uint32_t vec = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(stage * SLOT + VEC));
            dma_dword_s(vec, uniform_ptr(lse2p + tile * 64), (uint32_t)(lane * 4));
            dma_dword_s(vec + 256, uniform_ptr(deltap + tile * 64), (uint32_t)(lane * 4));
        }
    };
    auto tiles_of = [&](int i) { return (csize[i] * g.G + 63) >> 6; };
    // the TPS tiles t .. t + TPS - 1 of cube i, as far as the cube has them (nt tiles)
    auto issue = [&](int stage, int i, int t, int nt) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < TPS; ++u)
            if (t + u < nt) issue_tile(stage, u, i, t + u);
    };

    f32x4 acc[NS][D / 16];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int e = 0; e < D / 16; ++e) acc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Row cubes from the last one down to the own cube: workgroups that start together then stream the same tiles at
    // the same time, whatever their key cube, and one copy in L2 serves them all.
    int ii = g.N - 1, it = 0, int_ = tiles_of(g.N - 1);
    issue(0, ii, 0, int_);
    if ((it += TPS) >= int_) { --ii; it = 0; int_ = ii >= j ? tiles_of(ii) : 0; }
    int stage = 0;
    for (int i = g.N - 1; i >= j; --i) {
        const int nt = tiles_of(i);
        for (int tb = 0; tb < nt; tb += TPS) {
            tile_barrier();
            if (ii >= j) {
                issue(stage ^ 1, ii, it, int_);
                if ((it += TPS) >= int_) { --ii; it = 0; int_ = ii >= j ? tiles_of(ii) : 0; }
            }
            auto tile_work = [&](int slot) __attribute__((always_inline)) {
            const int t = tb + slot;
            const unsigned char *t0 = smem + stage * STAGE + slot * SLOT;
            const float *lv = reinterpret_cast<const float *>(t0 + VEC);
            const float *dv = lv + 64;
            // bit k: row k of the tile selected cube j (rows of the own cube attend it by rule)
            unsigned long long cm = ~0ull;
            if (MASKED && i > j) cm = colmask[(cm_base + i) * tpcr + t];
            // S[row, key]: the streamed rows take the place the keys have in the forward (qk_tile's row order)
            bf16x8 pf[NS][2];
            auto half = [&](auto hc) __attribute__((always_inline)) {
                constexpr int H = decltype(hc)::value;
                f32x4 sacc[NS][2], pacc[NS][2];
                const int rb = 32 * H + 8 * q4;  // the lane's eight rows of this half: rb .. rb + 7
                const uint32_t bits = (uint32_t)(cm >> rb);  // their selection bits
                // What the products start from: -lse * sqrt(D) of the row (times the softmax scale in base 2 the
                // accumulator is then the exponent of the probability), -inf for a row that did not select this key
                // cube (probabilities 0); and minus the row's delta for dP.
                f32x4 sinit[2], pinit[2];
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    sinit[k2] = *reinterpret_cast<const f32x4 *>(lv + rb + 4 * k2);
                    if (MASKED) {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (!((bits >> (4 * k2 + v)) & 1u)) sinit[k2][v] = -INFINITY;
                    }
                    if (WHICH == 1) pinit[k2] = *reinterpret_cast<const f32x4 *>(dv + rb + 4 * k2);
                }
                nat_half_from<D, NS, H>(t0, n16, q4, kf, sinit, sacc);
                if (WHICH == 1) nat_half_from<D, NS, H>(t0 + TILE, n16, q4, vf, pinit, pacc);
                if (i == j) {  // causal edge inside the own cube: a row attends keys up to its own rank
                    int r0 = 64 * t + rb;
                    asm volatile("" : "+v"(r0));
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int rrank = (r0 + 4 * k2 + v) / g.G;
#pragma unroll
                            for (int s = 0; s < NS; ++s)
                                if (key[s] > rrank) sacc[s][k2][v] = -INFINITY;
                        }
                }
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int s = 0; s < NS; ++s) {
                            const float p = __builtin_amdgcn_exp2f(sacc[s][k2][v] * c2);
                            pf[s][H][4 * k2 + v] = (__bf16)(WHICH == 1 ? p * pacc[s][k2][v] : p);
                        }
            };
            half(std::integral_constant<int, 0>{});
            half(std::integral_constant<int, 1>{});
            tn_tile<D, NS>(t0 + (WHICH == 0 ? TILE : 2 * TILE), n16, q4, pf, acc);
            };
            tile_work(0);
            if (TPS > 1 && tb + 1 < nt) tile_work(1);
            stage ^= 1;
        }
    }
    const float scale = WHICH == 1 ? 1.0f / sqrtf((float)D) : 1.0f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        if (!valid[s]) continue;
#pragma unroll
        for (int e = 0; e < D / 16; ++e) {
            bf16x2 a, b;
            a[0] = (__bf16)(acc[s][e][0] * scale); a[1] = (__bf16)(acc[s][e][1] * scale);
            b[0] = (__bf16)(acc[s][e][2] * scale); b[1] = (__bf16)(acc[s][e][3] * scale);
            uint2 o;
            o.x = *reinterpret_cast<uint32_t *>(&a);
            o.y = *reinterpret_cast<uint32_t *>(&b);
            *reinterpret_cast<uint2 *>(dOut + krow[s] + 16 * e + 4 * q4) = o;
        }
    }
}

template <int D>
static hipError_t launch_bwd_d(const Geom &g, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                               const uint16_t *O, const float *lse, const uint16_t *dO, const uint32_t *sel_mask,
                               uint16_t *dQ, uint16_t *dK, uint16_t *dV, void *ws, hipStream_t st)
{
    const BwdWorkspace w = bwd_workspace(g, ws);
    hipError_t e = launch_kv_pack(g, K, V, w.packA, false, st);  // natural K as it is: exact score products
    if (e != hipSuccess) return e;
    e = launch_kv_pack(g, V, K, w.packB, false, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_pack_rows_kernel<D>), dim3(w.tpcr, g.N, g.Hkv), dim3(256), 0, st, g, Q, dO, O, lse, w.tpcr,
                       w.Qn, w.Qt, w.dOn, w.dOt, w.lse2, w.delta);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (sel_mask != nullptr) {
        hipLaunchKernelGGL(bwd_colmask_kernel, dim3(w.tpcr, g.N, g.Hkv), dim3(64), 0, st, g, sel_mask, w.tpcr, w.colmask);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const uint16_t *Kn = reinterpret_cast<const uint16_t *>(w.packA);
    const uint16_t *Vn = reinterpret_cast<const uint16_t *>(w.packB);
    const uint16_t *Kt = Vn + half_elems;
    const int32_t *csize = reinterpret_cast<const int32_t *>(Kt + half_elems);
    constexpr int TILE = 64 * D * 2;

    const int nblk = (g.Cmax * g.G + BWD_ROWS - 1) / BWD_ROWS;
    const dim3 grid_q(bwd_grid(g.Hkv, g.N * nblk));
    const int lds_q = 2 * 3 * TILE;
    const int nkb = (g.Cmax + BWD_ROWS - 1) / BWD_ROWS;
    const dim3 grid_k(bwd_grid(g.Hkv, g.N * nkb));
    const int lds_v = 2 * 2 * (2 * TILE + 512), lds_k = 2 * (3 * TILE + 512);
#define ADASPARK_BWD_LAUNCH(MASKED)                                                                                    \
    do {                                                                                                               \
        static LdsOptIn opted_q, opted_v, opted_k;                                                                     \
        e = opted_q.ensure(reinterpret_cast<const void *>(&attn_bwd_dq_kernel<D, MASKED>), lds_q);                     \
        if (e != hipSuccess) return e;                                                                                 \
        hipLaunchKernelGGL((attn_bwd_dq_kernel<D, MASKED>), grid_q, dim3(BWD_THREADS), lds_q, st, g, Q, dO, Kn, Vn,    \
                           Kt, csize, w.lse2, w.delta, w.tpcr, sel_mask, dQ);                                          \
        e = opted_v.ensure(reinterpret_cast<const void *>(&attn_bwd_dkv_kernel<D, 0, MASKED>), lds_v);                 \
        if (e != hipSuccess) return e;                                                                                 \
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, 0, MASKED>), grid_k, dim3(BWD_THREADS), lds_v, st, g, K, V, w.Qn,   \
                           w.Qt, w.dOn, w.dOt, w.lse2, w.delta, w.tpcr, csize, w.colmask, dV);                                 \
        e = opted_k.ensure(reinterpret_cast<const void *>(&attn_bwd_dkv_kernel<D, 1, MASKED>), lds_k);                 \
        if (e != hipSuccess) return e;                                                                                 \
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, 1, MASKED>), grid_k, dim3(BWD_THREADS), lds_k, st, g, K, V, w.Qn,   \
                           w.Qt, w.dOn, w.dOt, w.lse2, w.delta, w.tpcr, csize, w.colmask, dK);                                 \
    } while (0)
    if (sel_mask != nullptr)
        ADASPARK_BWD_LAUNCH(true);
    else
        ADASPARK_BWD_LAUNCH(false);
#undef ADASPARK_BWD_LAUNCH
    return hipGetLastError();
}

hipError_t launch_attn_bwd(const Geom &g, const uint16_t *Q, const uint16_t *K, const uint16_t *V, const uint16_t *O,
                           const float *lse, const uint16_t *dO, const uint32_t *sel_mask, uint16_t *dQ, uint16_t *dK,
                           uint16_t *dV, void *ws, hipStream_t st)
{
    if (g.D == 64) return launch_bwd_d<64>(g, Q, K, V, O, lse, dO, sel_mask, dQ, dK, dV, ws, st);
    return launch_bwd_d<128>(g, Q, K, V, O, lse, dO, sel_mask, dQ, dK, dV, ws, st);
}

}  // namespace adaspark
