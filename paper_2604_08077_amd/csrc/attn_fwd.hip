// Sparse (Eq. 3 + own-cube rule, Sec. 3.2) and dense causal attention: flash attention over the packed KV copy
// with per-cube row compaction.
//
// Selection is per (token, query head), so rows that share a query tile select independent cube subsets; a
// mask-based tile kernel would execute dense FLOPs.  Here a workgroup owns up to MMAX query rows of one
// (query cube i, KV head) -- all query heads of the GQA group, token-major -- and keeps their online-softmax
// state (fp32 O, m, l) in LDS (MI355X: 160 KB per CU).  It walks the key cubes j <= i that any of its rows
// attends.  For each cube
//   1. every wavefront ballots the selection bits of all rows and so knows the (sorted) list of rows that
//      attend j (dense mode, own cube: all rows); no extra barrier is needed,
//   2. the list is cut into 16-row slabs, dealt round-robin to the eight wavefronts (two per SIMD: while one
//      is in its softmax the other can feed the MFMA pipe),
//   3. per slab the Q operands are gathered (prefetched under the previous cube's last tile), the rows' state
//      moves from LDS into MFMA accumulators, flash attention runs over the cube's 64-key tiles with
//      mfma_f32_16x16x32_bf16 (S^T = K.Q^T, O^T += V^T.P^T: a lane owns one query row and a quarter of the
//      keys of a tile), and the state moves back.
// Executed MFMA work is the selected (row, cube) pairs rounded up to 16 rows per workgroup and cube.  In dense
// mode the row set never changes and the state stays in registers.
//
// K and V^T tiles come from the packed, pre-swizzled copy (kvtile.h) by direct-to-LDS loads into two LDS
// stages: the loads of tile t+1 are started right after the barrier that opens tile t and waited for at the
// barrier that closes it, so there is one barrier per 64-key tile.
#include <cstdlib>
#include <type_traits>

#include "kvtile.h"

namespace adaspark {

constexpr int FWD_MAX_THREADS = 512;  // largest workgroup of the two modes (register budget: 256 per lane)
constexpr int FWD_NS = 2;             // 16-row slabs a wavefront works on at a time

template <int D, bool SPARSE>
struct Fwd {
    // Sparse: one workgroup of eight wavefronts per CU (its LDS holds the rows' state).  Dense: workgroups of
    // four wavefronts, two per CU: they are not tied to each other's barriers and drift apart, which lets one
    // workgroup's softmax run under the other's MFMAs.
    static constexpr int WAVES = SPARSE ? 8 : 4;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int NS = FWD_NS;
    static constexpr int MMAX = SPARSE ? 168 : 16 * NS * WAVES;  // rows per workgroup (sparse: what LDS can hold)
    static constexpr int GROUPS = (MMAX + 63) / 64;              // 64-row ballot groups
    static constexpr int CHUNK = KEY_TILE * D * 2;               // bytes of a K tile (= bytes of a V^T tile)
    static constexpr int NBUF = 4;                               // LDS buffers: K and V^T of two tiles
    static constexpr int DMA = CHUNK / 1024 / WAVES;             // 1 KB direct-to-LDS loads per wavefront and tile
    static constexpr int OST = D + 4;  // floats per state row (padded: 16 rows start in 16 different bank groups)
    static constexpr int SMALL = (((MMAX + 1) * 4 + 15) / 16) * 16;
    static constexpr int OFF_KV = 0;
    static constexpr int OFF_ROWID = OFF_KV + NBUF * CHUNK;
    static constexpr int OFF_RANK = OFF_ROWID + SMALL;
    static constexpr int OFF_MISC = OFF_RANK + SMALL;  // 16 bytes of workgroup scalars
    static constexpr int OFF_UMASK = OFF_MISC + 16;
    static constexpr int OFF_LIST = OFF_UMASK + (ADASPARK_MAX_CUBES / 32) * 4;  // per wavefront: 64*GROUPS bytes
    static constexpr int OFF_CUBES = OFF_LIST + WAVES * 64 * GROUPS;            // attended cubes, u16 each
    static constexpr int OFF_M = OFF_CUBES + ADASPARK_MAX_CUBES * 2;
    static constexpr int OFF_L = OFF_M + SMALL;
    static constexpr int OFF_O = OFF_L + SMALL;
    static constexpr int BYTES = SPARSE ? OFF_O + (MMAX + 1) * OST * 4 : OFF_UMASK;
    static_assert(MMAX <= 16 * NS * WAVES, "every attending row needs a slab");
    static_assert(DMA >= 1, "a tile is at least 1 KB per wavefront");
    static_assert(BYTES <= 160 * 1024, "LDS of one CU");
};

// Tile barrier.  Waits for everything this wavefront has in flight -- its LDS traffic and its direct-to-LDS loads
// of the next tile, started a whole tile ago -- then the workgroup barrier.
__device__ __forceinline__ void tile_barrier()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One wavefront copies 1 KB from global memory straight into LDS: lane l moves the 16 bytes at src (its own
// address) to lds_addr + 16*l.  lds_addr is wave-uniform.  Completion is counted by vmcnt like any vector load.
__device__ __forceinline__ void dma_1k(uint32_t lds_addr, const void *src)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(src)
                 : "memory", "m0");
}

// The same with the source given as a wave-uniform base (scalar registers) plus a 32-bit per-lane byte offset:
// a stream of tiles then advances with two scalar adds and no vector arithmetic.
__device__ __forceinline__ void dma_1k_s(uint32_t lds_addr, const void *sbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff),
                 "s"(sbase)
                 : "memory", "m0");
}

// Plain hardware max.  fmaxf() would first canonicalise each operand (one extra instruction per MFMA result);
// the scores are never signalling NaNs, and -inf (masked keys) orders as it should.
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// A-operand of all ones: (ones).P^T has the column sums of P^T, i.e. every query row's sum of probabilities, in each
// of its 16 rows.
__device__ __forceinline__ bf16x8 ones_operand()
{
    const __bf16 o = (__bf16)1.0f;
    return bf16x8{o, o, o, o, o, o, o, o};
}

// max / sum over the four lanes {n, n+16, n+32, n+48} that share a query row
__device__ __forceinline__ float quad_max(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = vmax(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return vmax(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_sum(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// S^T = K.Q^T for one 64-key tile and slabs S0..S1-1 of a wavefront.  MFMA M-row m of key group kg carries
// tile key 32*(kg/2) + 8*(m/4) + 4*(kg%2) + m%4, so that a lane's registers of groups 2sl, 2sl+1 hold keys
// 32sl + 8*q4 + 0..7: the operand order of the P.V MFMA.  One K operand load serves all slabs of the range.
template <int D, int S0, int S1, int NS>
__device__ __forceinline__ void qk_tile(const unsigned char *kt, int n16, int q4, const bf16x8 (&qf)[NS][D / 32],
                                        f32x4 (&sacc)[NS][4])
{
#pragma unroll
    for (int s = S0; s < S1; ++s)
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) sacc[s][kg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < D / 32; ++c)
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
            const int krow = 32 * (kg >> 1) + 8 * (n16 >> 2) + 4 * (kg & 1) + (n16 & 3);
            const bf16x8 af = *reinterpret_cast<const bf16x8 *>(kt + k_tile_off<D>(krow, 4 * c + q4));
#pragma unroll
            for (int s = S0; s < S1; ++s)
                sacc[s][kg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, qf[s][c], sacc[s][kg], 0, 0, 0);
        }
}

// fp32 online softmax of the tile's scores, base-2 exponentials; P rounded to bf16 in P.V operand order.
// The row sums are not taken here: l_run is an MFMA accumulator that the P.V step feeds with (all-ones).P^T, the
// sum of the very weights P.V uses, so here it is only rescaled along with O.  The slabs of the range go through every stage side by side: their dependency chains (maximum, row sum, the
// lane exchanges) are independent, and a wavefront alone on its SIMD's vector unit needs that parallelism.
// With MASKED, a row whose rsel flag is off takes no part in the tile: its probabilities are 0 and its running
// state stays as it is (the subtracted maximum is +inf, the rescale factor 1).
template <int D, int S0, int S1, int NS, bool MASKED = false>
__device__ __forceinline__ void softmax_tile(f32x4 (&sacc)[NS][4], bf16x8 (&pf)[NS][2], f32x4 (&oacc)[NS][D / 16],
                                             float (&m_run)[NS], f32x4 (&l_run)[NS], const int (&lim)[NS], int key0,
                                             bool need_mask, float c2, int q4, const bool (&rsel)[NS])
{
    if (need_mask) {
        // few tiles come here; the empty statement keeps the index arithmetic from being hoisted out to all
        int kb = key0 + 8 * q4;
        asm volatile("" : "+v"(kb));
#pragma unroll
        for (int s = S0; s < S1; ++s)
#pragma unroll
            for (int kg = 0; kg < 4; ++kg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int kr = kb + 32 * (kg >> 1) + 4 * (kg & 1) + v;
                    if (kr > lim[s]) sacc[s][kg][v] = -INFINITY;
                }
    }
    float mx[NS], m_new[NS], m_sub[NS], alpha[NS];
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(sacc[s][0][0], sacc[s][0][1], sacc[s][0][2]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(mx[s], sacc[s][0][3], sacc[s][1][0]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(mx[s], sacc[s][1][1], sacc[s][1][2]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(mx[s], sacc[s][1][3], sacc[s][2][0]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(mx[s], sacc[s][2][1], sacc[s][2][2]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(mx[s], sacc[s][2][3], sacc[s][3][0]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax3(mx[s], sacc[s][3][1], sacc[s][3][2]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = vmax(mx[s], sacc[s][3][3]);
#pragma unroll
    for (int s = S0; s < S1; ++s) mx[s] = quad_max(mx[s]);
    bool moved = false;
#pragma unroll
    for (int s = S0; s < S1; ++s) {
        m_new[s] = vmax(m_run[s], mx[s] * c2);
        if (MASKED && !rsel[s]) m_new[s] = m_run[s];
        m_sub[s] = (MASKED && !rsel[s]) ? INFINITY : m_new[s];
        alpha[s] = __builtin_amdgcn_exp2f(m_run[s] - m_new[s]);
        moved = moved || (m_new[s] != m_run[s]);
    }
#pragma unroll
    for (int kg = 0; kg < 4; ++kg)
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int s = S0; s < S1; ++s)
                pf[s][kg >> 1][4 * (kg & 1) + v] =
                    (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[s][kg][v], c2, -m_sub[s]));
#pragma unroll
    for (int s = S0; s < S1; ++s) m_run[s] = m_new[s];
    // the running maximum rarely moves after the first tiles: rescale only when some row needs it
    if (__ballot(moved) != 0ull) {
#pragma unroll
        for (int s = S0; s < S1; ++s)
#pragma unroll
            for (int e = 0; e < D / 16; ++e) oacc[s][e] *= alpha[s];
#pragma unroll
        for (int s = S0; s < S1; ++s) l_run[s] *= alpha[s];
    }
}

// The MFMA phase of a wavefront in the counter-phase kernel: P.V of one tile, then S of the next, as one stream
// of operand loads and MFMAs.  A wavefront that is alone in its MFMA phase cannot hide LDS latency behind a
// neighbour, so the operands run PF loads ahead of their use through a ring of registers, and the order written
// here is the order executed (nothing is scheduled across a step).  Step r < RV: V^T operand (sl, e), O^T of every
// slab; step r >= RV: K operand (c, kg), S^T of every slab.
template <int D, int NS, int PF, bool DO_PV, bool DO_QK>
__device__ __forceinline__ void mfma_phase(const unsigned char *vt, const unsigned char *kt, int n16, int q4,
                                           const bf16x8 (&pf)[NS][2], f32x4 (&oacc)[NS][D / 16], f32x4 (&l_run)[NS],
                                           const bf16x8 (&qf)[NS][D / 32], f32x4 (&sacc)[NS][4])
{
    constexpr int DT = D / 16, KSTEPS = D / 32;
    constexpr int RV = DO_PV ? 2 * DT : 0, RK = DO_QK ? 4 * KSTEPS : 0, R = RV + RK;
#ifdef PP_NO_MFMA
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
        for (int k = 0; k < 4; ++k) asm volatile("" : "+v"(sacc[s][k]));
#pragma unroll
        for (int k = 0; k < 2; ++k) asm volatile("" ::"v"(pf[s][k]));
    }
    return;
#endif
    bf16x8 ring[PF];
    auto operand = [&](int r) __attribute__((always_inline)) -> bf16x8 {
#ifdef PP_NO_LDS
        bf16x8 z = qf[0][0];
        asm volatile("" : "+v"(z));
        return z;
#endif
        if (r < RV) {
            const int sl = r / DT, e = r % DT;
            return *reinterpret_cast<const bf16x8 *>(vt + vt_tile_off(16 * e + n16, 4 * sl + q4));
        }
        const int c = (r - RV) / 4, kg = (r - RV) % 4;
        const int krow = 32 * (kg >> 1) + 8 * (n16 >> 2) + 4 * (kg & 1) + (n16 & 3);
        return *reinterpret_cast<const bf16x8 *>(kt + k_tile_off<D>(krow, 4 * c + q4));
    };
#pragma unroll
    for (int r = 0; r < PF && r < R; ++r) ring[r] = operand(r);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bf16x8 af = ring[r % PF];
        if (r < RV) {
            const int sl = r / DT, e = r % DT;
            if (e == 0) {  // row sums: no operand load, they fill the wait for the first V^T operands
                const bf16x8 ones = ones_operand();
#pragma unroll
                for (int s = 0; s < NS; ++s)
                    l_run[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[s][sl], l_run[s], 0, 0, 0);
            }
#pragma unroll
            for (int s = 0; s < NS; ++s)
                oacc[s][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf[s][sl], oacc[s][e], 0, 0, 0);
        } else {
            const int c = (r - RV) / 4, kg = (r - RV) % 4;
#pragma unroll
            for (int s = 0; s < NS; ++s)
                sacc[s][kg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    af, qf[s][c], c == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : sacc[s][kg], 0, 0, 0);
        }
        if (r + PF < R) ring[r % PF] = operand(r + PF);
#ifndef PP_NOSB
        __builtin_amdgcn_sched_barrier(0);
#endif
    }
}

// O^T += V^T.P^T and l += sum(P) for one 64-key tile; one V^T operand load serves all slabs of the range.
template <int D, int S0, int S1, int NS>
__device__ __forceinline__ void pv_tile(const unsigned char *vt, int n16, int q4, const bf16x8 (&pf)[NS][2],
                                        f32x4 (&oacc)[NS][D / 16], f32x4 (&l_run)[NS])
{
    const bf16x8 ones = ones_operand();
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int s = S0; s < S1; ++s)
            l_run[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[s][sl], l_run[s], 0, 0, 0);
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int e = 0; e < D / 16; ++e) {
            const bf16x8 af = *reinterpret_cast<const bf16x8 *>(vt + vt_tile_off(16 * e + n16, 4 * sl + q4));
#pragma unroll
            for (int s = S0; s < S1; ++s)
                oacc[s][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf[s][sl], oacc[s][e], 0, 0, 0);
        }
}

struct TilePos {
    int k;   // position in the workgroup's list of attended cubes
    int j;   // the cube
    int t;   // 64-key tile inside the cube
    int nt;  // tiles of cube j this workgroup reads
};

// SPARSE: rows are compacted per cube (state in LDS).  MASKED (with SPARSE off): the dense walk over fixed rows
// with every row's selection bit applied as a mask -- dense FLOPs, but no state traffic and two workgroups per
// CU; the better choice when most cubes are selected.  mode_flag (may be null): the kernel runs only if
// *mode_flag == my_mode, so that both variants can be enqueued and a device-side density estimate picks one.
template <int D, bool SPARSE, bool MASKED>
__global__ __launch_bounds__(FWD_MAX_THREADS) void attn_fwd_kernel(
    Geom g, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Kp, const uint16_t *__restrict__ Vt,
    const int32_t *__restrict__ csize, const uint32_t *__restrict__ sel_mask, const int *__restrict__ mode_flag,
    int my_mode, uint16_t *__restrict__ O, float *__restrict__ lse)
{
    static_assert(!(SPARSE && MASKED), "masking is the dense walk's way of honouring the selection");
    if (mode_flag != nullptr && *mode_flag != my_mode) return;
    using C = Fwd<D, SPARSE>;
    constexpr int NS = C::NS, MMAX = C::MMAX, OST = C::OST, THREADS = C::THREADS;
    constexpr int WAVES = C::WAVES, GROUPS = C::GROUPS;
    constexpr int KSTEPS = D / 32;  // MFMA k-steps of S^T (32 head-dim elements each)
    constexpr int DT = D / 16;      // 16-wide tiles of O^T
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
    unsigned char *kvbuf = smem + C::OFF_KV;
    int *rowid = reinterpret_cast<int *>(smem + C::OFF_ROWID);
    int *rrank = reinterpret_cast<int *>(smem + C::OFF_RANK);
    int *misc = reinterpret_cast<int *>(smem + C::OFF_MISC);
    uint32_t *umask = reinterpret_cast<uint32_t *>(smem + C::OFF_UMASK);
    uint16_t *cubes = reinterpret_cast<uint16_t *>(smem + C::OFF_CUBES);
    float *mst = reinterpret_cast<float *>(smem + C::OFF_M);
    float *lst = reinterpret_cast<float *>(smem + C::OFF_L);
    float *ost = reinterpret_cast<float *>(smem + C::OFF_O);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    unsigned char *clist = smem + C::OFF_LIST + wave * 64 * GROUPS;  // this wavefront's list of attending rows

    // workgroup -> (query cube, KV head, row block).  The row blocks of one (cube, KV head) stream the same K/V
    // tiles, so they are placed on the same XCD (hardware deals consecutive workgroup ids round-robin to the
    // 8 XCDs, each with its own L2) and next to each other in time; groups go round-robin over the XCDs, late
    // cubes (most preceding cubes) first.
    const int nblk_max = (g.G * g.Cmax + MMAX - 1) / MMAX;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int grp = (seq / nblk_max) * 8 + xcd;
    const int blk = seq % nblk_max;
    if (grp >= g.N * g.Hkv) return;
    const int kv = grp % g.Hkv;
    const int i = g.N - 1 - grp / g.Hkv;
    const CubeBox qbox = cube_box(g, i);
    const int qsize = qbox.size();
    const int P = g.G * qsize;  // rows of this (cube, KV head): rho = rank * G + head-in-group
    const int nblk = (P + MMAX - 1) / MMAX;
    if (blk >= nblk) return;
    const int row0 = (int)((long long)blk * P / nblk), row1 = (int)((long long)(blk + 1) * P / nblk);
    const int Mrows = row1 - row0;
    const int max_rank = (row1 - 1) / g.G;
    const int own_tiles = min((qsize + KEY_TILE - 1) / KEY_TILE, max_rank / KEY_TILE + 1);

    for (int r = tid; r < Mrows; r += THREADS) {
        const int rho = row0 + r, rank = rho / g.G, hg = rho % g.G;
        const int rid = token_of(g, qbox, rank) * g.Hq + kv * g.G + hg;
        rowid[r] = rid;
        rrank[r] = rank;
        if (SPARSE) { mst[r] = -1e30f; lst[r] = 0.f; }
        if (r == 0) {  // scratch row: read and written by the padding columns of a partial slab
            rowid[MMAX] = rid;
            rrank[MMAX] = 0;
            if (SPARSE) { mst[MMAX] = -1e30f; lst[MMAX] = 0.f; }
        }
    }
    if (SPARSE) {
        for (int x = tid; x < (MMAX + 1) * OST / 4; x += THREADS)
            reinterpret_cast<f32x4 *>(ost)[x] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int w = tid; w < g.words; w += THREADS) umask[w] = 0;
    }
    if (tid == 0) misc[0] = 0;
    __syncthreads();

    // ---- the cubes this workgroup attends (union over its rows), in order; the own cube i is always last
    int ncubes = i + 1;
    if (SPARSE) {
        for (int r = tid; r < Mrows; r += THREADS) {
            const uint32_t *mr = sel_mask + (size_t)rowid[r] * g.words;
            for (int w = 0; w < g.words; ++w) {
                const uint32_t bits = mr[w];
                if (bits) atomicOr(&umask[w], bits);
            }
        }
        __syncthreads();
        // word w holds cubes 32w..32w+31; only cubes below i count
        auto below_i = [&](int w) -> uint32_t {
            const int lo = 32 * w;
            const uint32_t keep = i >= lo + 32 ? 0xffffffffu : (i > lo ? (1u << (i - lo)) - 1u : 0u);
            return umask[w] & keep;
        };
        for (int w = tid; w < g.words; w += THREADS) {
            int base = 0;
            for (int w2 = 0; w2 < w; ++w2) base += __popc(below_i(w2));
            uint32_t bits = below_i(w);
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                cubes[base++] = (uint16_t)(32 * w + b);
            }
        }
        int nsel = 0;
        for (int w = 0; w < g.words; ++w) nsel += __popc(below_i(w));
        if (tid == 0) cubes[nsel] = (uint16_t)i;
        ncubes = nsel + 1;
        __syncthreads();
    }
    auto cube_at = [&](int k) -> int {
        return SPARSE ? __builtin_amdgcn_readfirstlane((int)cubes[k]) : k;
    };
    auto tiles_of = [&](int j) -> int {
        if (j == i) return own_tiles;
        return g.ragged ? (csize[j] + KEY_TILE - 1) / KEY_TILE : g.TPC;
    };
    // length of the tile stream
    {
        int part = 0;
        for (int k = tid; k < ncubes; k += THREADS) part += tiles_of(SPARSE ? (int)cubes[k] : k);
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        if (lane == 0) atomicAdd(&misc[0], part);
        __syncthreads();
    }
    const int ntiles = __builtin_amdgcn_readfirstlane(misc[0]);

    auto first_tile = [&]() -> TilePos {
        TilePos p;
        p.k = 0;
        p.j = cube_at(0);
        p.t = 0;
        p.nt = tiles_of(p.j);
        return p;
    };
    auto advance = [&](TilePos &p) __attribute__((always_inline)) {
        if (p.t + 1 < p.nt) ++p.t;
        else if (p.k + 1 < ncubes) {
            ++p.k;
            p.j = cube_at(p.k);
            p.t = 0;
            p.nt = tiles_of(p.j);
        } else {
            p.k = ncubes;  // past the end
        }
    };
    // this wavefront's share of a tile: DMA pieces of 1 KB, lane l moves 16 bytes
    auto issue = [&](const uint16_t *base, const TilePos &p, int buf) __attribute__((always_inline)) {
        const unsigned char *src = reinterpret_cast<const unsigned char *>(
            base + ((((size_t)kv * g.N + p.j) * g.TPC) + p.t) * (size_t)(KEY_TILE * D));
#pragma unroll
        for (int u = 0; u < C::DMA; ++u) {
            const int piece = wave * C::DMA + u;
            const uint32_t dst = __builtin_amdgcn_readfirstlane(
                (uint32_t)(uintptr_t)(kvbuf + buf * C::CHUNK + piece * 1024));
            dma_1k(dst, src + piece * 1024 + lane * 16);
        }
    };

    // ---- slabs of this wavefront for cube j.  The rows that attend j, in row order, are cut into 16-row slabs;
    // slab k goes to wavefront k % WAVES as its slot k / WAVES.  lr[s]: workgroup row in column n16 of slot s
    // (MMAX: padding column); ns: slots in use; lo/hi: smallest/largest rank among the wavefront's rows (own
    // cube only).
    int mrid[GROUPS];  // global row id behind (group, lane); -1: no such row
#pragma unroll
    for (int gq = 0; gq < GROUPS; ++gq) {
        const int r = 64 * gq + lane;
        mrid[gq] = r < Mrows ? rowid[r] : -1;
    }
    int cw = -1;  // mask word index cached in wbits
    uint32_t wbits[GROUPS];
#pragma unroll
    for (int gq = 0; gq < GROUPS; ++gq) wbits[gq] = 0;
    auto slab_rows = [&](int j, int (&lr)[NS], int &ns, int &lo, int &hi) __attribute__((always_inline)) {
        int total;
        const bool all = !SPARSE || j == i;
        if (all) total = Mrows;
        else {
            if ((j >> 5) != cw) {
                cw = j >> 5;
#pragma unroll
                for (int gq = 0; gq < GROUPS; ++gq)
                    wbits[gq] = mrid[gq] >= 0 ? sel_mask[(size_t)mrid[gq] * g.words + cw] : 0u;
            }
            // every attending row writes its index at its position in the list: the number
            // of attending rows below it.  The list is private to the wavefront: no barrier.
            total = 0;
#pragma unroll
            for (int gq = 0; gq < GROUPS; ++gq) {
                const bool sel = (wbits[gq] >> (j & 31)) & 1u;
                const unsigned long long bal = __ballot(sel);
                const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
                if (sel) clist[total + below] = (unsigned char)(64 * gq + lane);
                total += __popcll(bal);
            }
        }
        const int nslab = (total + 15) >> 4;
        ns = nslab > wave ? (nslab - wave + WAVES - 1) / WAVES : 0;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int idx = 16 * (wave + WAVES * s) + n16;
            int r = MMAX;
            if (idx < total) r = all ? idx : (int)clist[idx];
            lr[s] = r;
        }
        // rows are sorted by rank: the first column of slot 0 and the last used column of the last slot bound them
        lo = hi = 0;
        if (all && ns > 0) {
            lo = rrank[16 * wave];
            hi = rrank[min(16 * (wave + WAVES * (ns - 1)) + 15, total - 1)];
        }
        // the same in every lane: say so, and the tests on them become scalar branches
        lo = __builtin_amdgcn_readfirstlane(lo);
        hi = __builtin_amdgcn_readfirstlane(hi);
    };
    // Q operands of one slab: lane (n16, q4) takes head-dim elements 32c + 8*q4 .. +7 of its column's row
    auto load_q = [&](int row, bf16x8 (&q)[KSTEPS]) __attribute__((always_inline)) {
        const uint16_t *qrow = Q + (size_t)rowid[row] * D + 8 * q4;
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) q[c] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * c);
    };
    // The compiler places the wait for a load in front of the first use of its result.  Naming the registers
    // here puts that wait here, once, instead of in front of every S^T of the main loop (where it would also
    // hold up the direct-to-LDS loads in flight).
    auto settle_q = [&](bf16x8 (&q)[KSTEPS]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) asm volatile("" : "+v"(q[c]));
    };

    const float c2 = 1.44269504088896340736f / sqrtf((float)D);

    TilePos sc = first_tile();  // staging cursor: the tile whose K and V^T are being brought in
    TilePos cc = sc;            // compute cursor
    issue(Kp, sc, 0);           // tile 0 -> stage 0 (K in buffer 0, V^T in buffer 1)
    issue(Vt, sc, 1);

    int lr[NS], ns, rank_lo, rank_hi;
    bf16x8 qf[NS][KSTEPS];
    slab_rows(cc.j, lr, ns, rank_lo, rank_hi);
#pragma unroll
    for (int s = 0; s < NS; ++s) load_q(lr[s], qf[s]);
#pragma unroll
    for (int s = 0; s < NS; ++s) settle_q(qf[s]);

    // online-softmax state of the slabs being worked on
    int lim[NS];
    float m_run[NS];
    f32x4 l_run[NS];  // every element holds the row's running sum
    f32x4 oacc[NS][DT];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        m_run[s] = -1e30f;
        l_run[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < DT; ++e) oacc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto set_limits = [&](int j) __attribute__((always_inline)) -> int {
        const bool own = (j == i);
        const int jsize = own ? qsize : (g.ragged ? csize[j] : g.Cmax);
#pragma unroll
        for (int s = 0; s < NS; ++s) lim[s] = own ? min(rrank[lr[s]], jsize - 1) : jsize - 1;
        return jsize;
    };
    auto state_in = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < ns) {
                m_run[s] = mst[lr[s]];
                const float l = lst[lr[s]];
                l_run[s] = f32x4{l, l, l, l};
#pragma unroll
                for (int e = 0; e < DT; ++e)
                    oacc[s][e] = *reinterpret_cast<const f32x4 *>(&ost[lr[s] * OST + 16 * e + 4 * q4]);
            }
    };
    auto state_out = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < ns) {
#pragma unroll
                for (int e = 0; e < DT; ++e)
                    *reinterpret_cast<f32x4 *>(&ost[lr[s] * OST + 16 * e + 4 * q4]) = oacc[s][e];
                if (q4 == 0) {
                    mst[lr[s]] = m_run[s];
                    lst[lr[s]] = l_run[s][0];
                }
            }
    };
    // MASKED: does this lane's row (per slab) attend cube j?  One mask word per row is cached in registers.
    bool rsel[NS];
    uint32_t mword[NS];
    int mword_idx = -1;
#pragma unroll
    for (int s = 0; s < NS; ++s) { rsel[s] = true; mword[s] = 0; }
    auto set_rsel = [&](int j) __attribute__((always_inline)) {
        if (!MASKED) return;
        if (j == i) {
#pragma unroll
            for (int s = 0; s < NS; ++s) rsel[s] = true;
            return;
        }
        if ((j >> 5) != mword_idx) {
            mword_idx = j >> 5;
#pragma unroll
            for (int s = 0; s < NS; ++s) mword[s] = sel_mask[(size_t)rowid[lr[s]] * g.words + mword_idx];
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) rsel[s] = (mword[s] >> (j & 31)) & 1u;
    };
    set_rsel(cc.j);
    int jsize = set_limits(cc.j);  // first cube: the state registers already hold the initial state
    bool new_slabs = false;        // the slabs changed at the last cube boundary: their state is still in LDS
    int lr_n[NS], ns_n = 0, lo_n = 0, hi_n = 0;
    bf16x8 qf_n[KSTEPS];
    f32x4 sacc[NS][4];
    bf16x8 pf[NS][2];

    // ---- one 64-key tile per barrier.  Tile t sits in stage t % 2 (buffers 2*stage, 2*stage + 1).
    for (int tau = 0; tau < ntiles; ++tau) {
        tile_barrier();  // tile tau has landed; everybody is done with tile tau-1
        const int st = tau & 1;
        if (SPARSE && new_slabs) {
            // cube boundary: the slabs (and with them rows) move between wavefronts.  Every wavefront wrote
            // its state back before the barrier.
            ns = ns_n;
            rank_lo = lo_n;
            rank_hi = hi_n;
#pragma unroll
            for (int s = 0; s < NS; ++s) lr[s] = lr_n[s];
            if (ns > 0) {
#pragma unroll
                for (int c = 0; c < KSTEPS; ++c) qf[0][c] = qf_n[c];
            }
            // a second slab is rare (own cube, unusually popular cube): its Q operands come late
#pragma unroll
            for (int s = 1; s < NS; ++s)
                if (s < ns) {
                    load_q(lr[s], qf[s]);
                    settle_q(qf[s]);
                }
            state_in();
            jsize = set_limits(cc.j);
            new_slabs = false;
        }
        if (tau + 1 < ntiles) {
            advance(sc);
            issue(Kp, sc, 2 * (st ^ 1));
            issue(Vt, sc, 2 * (st ^ 1) + 1);
        }
        const unsigned char *kt = kvbuf + (2 * st) * C::CHUNK, *vt = kt + C::CHUNK;
        const bool own = (cc.j == i);
        const int key0 = KEY_TILE * cc.t;
        int nsl = (ns > 0 && !(own && key0 > rank_hi)) ? ns : 0;  // wave-uniform
        if (MASKED) {
            bool any = false;
#pragma unroll
            for (int s = 0; s < NS; ++s) any = any || rsel[s];
            if (!__any(any)) nsl = 0;  // none of the wavefront's rows attends this cube
        }
        const bool need_mask = (key0 + KEY_TILE > jsize) || (own && key0 + KEY_TILE - 1 > rank_lo);
        const bool cube_ends = cc.t + 1 == cc.nt && cc.k + 1 < ncubes;
        if (SPARSE && cube_ends) {
            // last tile of the cube: work out the next cube's slabs and start fetching the Q operands of the
            // first one into registers of their own.  They are copied over after the next barrier, which has
            // waited for them anyway.
            slab_rows(cube_at(cc.k + 1), lr_n, ns_n, lo_n, hi_n);
            if (ns_n > 0) load_q(lr_n[0], qf_n);
        }
        if (SPARSE) {
            // slab counts vary from cube to cube: one guarded block per slab
            if (nsl >= 1) {
                qk_tile<D, 0, 1, NS>(kt, n16, q4, qf, sacc);
                softmax_tile<D, 0, 1, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4, rsel);
                pv_tile<D, 0, 1, NS>(vt, n16, q4, pf, oacc, l_run);
            }
            if (NS >= 2 && nsl >= 2) {
                qk_tile<D, 1, NS, NS>(kt, n16, q4, qf, sacc);
                softmax_tile<D, 1, NS, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4, rsel);
                pv_tile<D, 1, NS, NS>(vt, n16, q4, pf, oacc, l_run);
            }
        } else if (nsl || !MASKED) {
            // fixed row set: all slabs, padding columns of a partial slab compute on the scratch row
            qk_tile<D, 0, NS, NS>(kt, n16, q4, qf, sacc);
#ifdef PP_NO_SOFTMAX
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int kg = 0; kg < 4; ++kg)
#pragma unroll
                    for (int v = 0; v < 4; ++v) pf[s][kg >> 1][4 * (kg & 1) + v] = (__bf16)sacc[s][kg][v];
#else
            softmax_tile<D, 0, NS, NS, MASKED>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4, rsel);
#endif
            pv_tile<D, 0, NS, NS>(vt, n16, q4, pf, oacc, l_run);
        }
        advance(cc);
        if (cube_ends) {
            if (SPARSE) {
                state_out();
                new_slabs = true;
            } else {
                jsize = set_limits(cc.j);
                set_rsel(cc.j);
            }
        }
    }

    // ---- normalise and write out (no direct-to-LDS load may outlive the workgroup's LDS allocation)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (SPARSE) {
        if (!new_slabs) state_out();
        __syncthreads();
        for (int x = tid; x < Mrows * (D / 8); x += THREADS) {
            const int r = x / (D / 8), c = x % (D / 8);
            const float inv = 1.0f / lst[r];
            const float *src = &ost[r * OST + 8 * c];
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                w[e] = (uint32_t)float_to_bf16_bits(src[2 * e] * inv) |
                       ((uint32_t)float_to_bf16_bits(src[2 * e + 1] * inv) << 16);
            *reinterpret_cast<uint4 *>(O + (size_t)rowid[r] * D + 8 * c) = make_uint4(w[0], w[1], w[2], w[3]);
        }
        if (lse != nullptr)
            for (int r = tid; r < Mrows; r += THREADS)
                lse[rowid[r]] = (mst[r] + log2f(lst[r])) * 0.69314718055994530942f;
    } else {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (lr[s] == MMAX) continue;
            const int rid = rowid[lr[s]];
            const float inv = 1.0f / l_run[s][0];
            uint16_t *orow = O + (size_t)rid * D + 4 * q4;
#pragma unroll
            for (int e = 0; e < DT; ++e) {
                const uint32_t w0 = (uint32_t)float_to_bf16_bits(oacc[s][e][0] * inv) |
                                    ((uint32_t)float_to_bf16_bits(oacc[s][e][1] * inv) << 16);
                const uint32_t w1 = (uint32_t)float_to_bf16_bits(oacc[s][e][2] * inv) |
                                    ((uint32_t)float_to_bf16_bits(oacc[s][e][3] * inv) << 16);
                *reinterpret_cast<uint2 *>(orow + 16 * e) = make_uint2(w0, w1);
            }
            if (lse != nullptr && q4 == 0) lse[rid] = (m_run[s] + log2f(l_run[s][0])) * 0.69314718055994530942f;
        }
    }
}

// =====================================================================================================
// Fixed-row walk with two wavefront sets in counter-phase (dense attention, and sparse attention with the
// selection applied as a mask).
//
// On a SIMD an MFMA keeps the matrix pipe busy for ~16 cycles and leaves room for two or three vector
// instructions; a wavefront alone cannot use that room, because its softmax needs the finished scores.  So a
// workgroup holds eight wavefronts, two per SIMD, and the two of a SIMD are kept half a tile apart: while set X
// (wavefronts 0-3) runs the softmax of tile t, set Y (4-7) runs P.V of tile t-1 and S = Q.K^T of tile t; then X
// runs P.V(t) and S(t+1) while Y runs softmax(t).  Two workgroup barriers per tile hold the sets in that phase.
//
//   slot a(t):  X: softmax(t)          Y: P.V(t-1), S(t)
//   slot b(t):  X: P.V(t), S(t+1)      Y: softmax(t)
//
// K and V^T tiles go through three LDS stages each (tile t in stage t % 3).  After the barrier that opens slot
// b(t) nobody reads K(t) or V(t-1) any more, and the direct-to-LDS loads of K(t+3) and V(t+2) go into their
// stages; they are waited for two barriers later (the loads started one tile ago may stay in flight).
template <int D>
struct Pp {
    static constexpr int WAVES = 8;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int NS = FWD_NS;
    static constexpr int MMAX = 16 * NS * WAVES;  // 256 rows
    static constexpr int NST = 3;
    static constexpr int CHUNK = KEY_TILE * D * 2;
    static constexpr int DMA = CHUNK / 1024 / WAVES;
    static constexpr int SMALL = (((MMAX + 1) * 4 + 15) / 16) * 16;
    static constexpr int OFF_K = 0;
    static constexpr int OFF_V = OFF_K + NST * CHUNK;
    static constexpr int OFF_ROWID = OFF_V + NST * CHUNK;
    static constexpr int OFF_RANK = OFF_ROWID + SMALL;
    static constexpr int OFF_MISC = OFF_RANK + SMALL;
    static constexpr int BYTES = OFF_MISC + 16;
    static_assert(DMA >= 1, "a tile is at least 1 KB per wavefront");
    static_assert(BYTES <= 160 * 1024, "LDS of one CU");
};

#ifndef PP_PF
#define PP_PF 4
#endif

// Barrier that opens a slot a: only this wavefront's LDS traffic has to be done.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Barrier that opens a slot b: all direct-to-LDS loads but the newest `KEEP` of this wavefront have landed.
template <int KEEP>
__device__ __forceinline__ void dma_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(KEEP) : "memory");
}

template <int D, bool MASKED>
__global__ __launch_bounds__(FWD_MAX_THREADS) void attn_pp_kernel(
    Geom g, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Kp, const uint16_t *__restrict__ Vt,
    const int32_t *__restrict__ csize, const uint32_t *__restrict__ sel_mask, const int *__restrict__ mode_flag,
    int my_mode, uint16_t *__restrict__ O, float *__restrict__ lse)
{
    if (mode_flag != nullptr && *mode_flag != my_mode) return;
    using C = Pp<D>;
    constexpr int NS = C::NS, MMAX = C::MMAX, THREADS = C::THREADS, WAVES = C::WAVES, NST = C::NST;
    constexpr int KSTEPS = D / 32, DT = D / 16;
    constexpr int PF = PP_PF;  // operand loads in flight ahead of the MFMAs
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
    int *rowid = reinterpret_cast<int *>(smem + C::OFF_ROWID);
    int *rrank = reinterpret_cast<int *>(smem + C::OFF_RANK);
    int *misc = reinterpret_cast<int *>(smem + C::OFF_MISC);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    const bool set_y = __builtin_amdgcn_readfirstlane(wave >> 2) != 0;

    // workgroup -> (query cube, KV head, row block): as in attn_fwd_kernel
    const int nblk_max = (g.G * g.Cmax + MMAX - 1) / MMAX;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int grp = (seq / nblk_max) * 8 + xcd;
    const int blk = seq % nblk_max;
    if (grp >= g.N * g.Hkv) return;
    const int kv = grp % g.Hkv;
    const int i = g.N - 1 - grp / g.Hkv;
    const CubeBox qbox = cube_box(g, i);
    const int qsize = qbox.size();
    const int P = g.G * qsize;
    const int nblk = (P + MMAX - 1) / MMAX;
    if (blk >= nblk) return;
    const int row0 = (int)((long long)blk * P / nblk), row1 = (int)((long long)(blk + 1) * P / nblk);
    const int Mrows = row1 - row0;
    const int max_rank = (row1 - 1) / g.G;
    const int own_tiles = min((qsize + KEY_TILE - 1) / KEY_TILE, max_rank / KEY_TILE + 1);

    for (int r = tid; r < Mrows; r += THREADS) {
        const int rho = row0 + r, rank = rho / g.G, hg = rho % g.G;
        const int rid = token_of(g, qbox, rank) * g.Hq + kv * g.G + hg;
        rowid[r] = rid;
        rrank[r] = rank;
        if (r == 0) {  // scratch row behind the padding columns of a partial slab
            rowid[MMAX] = rid;
            rrank[MMAX] = 0;
        }
    }
    if (tid == 0) misc[0] = 0;
    __syncthreads();

    // the tile stream: cubes 0..i in order, the own cube i last and only up to the largest rank of the block
    const int ncubes = i + 1;
    auto tiles_of = [&](int j) -> int {
        if (j == i) return own_tiles;
        return g.ragged ? (csize[j] + KEY_TILE - 1) / KEY_TILE : g.TPC;
    };
    {
        int part = 0;
        for (int k = tid; k < ncubes; k += THREADS) part += tiles_of(k);
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        if (lane == 0) atomicAdd(&misc[0], part);
        __syncthreads();
    }
    const int ntiles = __builtin_amdgcn_readfirstlane(misc[0]);

    auto first_tile = [&]() -> TilePos {
        TilePos p;
        p.k = p.j = 0;
        p.t = 0;
        p.nt = tiles_of(0);
        return p;
    };
    auto advance = [&](TilePos &p) __attribute__((always_inline)) {
        if (p.t + 1 < p.nt) ++p.t;
        else if (p.j + 1 < ncubes) {
            p.k = ++p.j;
            p.t = 0;
            p.nt = tiles_of(p.j);
        }  // the last tile stays where it is: nothing is issued or computed past the end
    };
    // The K and V^T tiles are fetched as two streams: a wave-uniform pointer to the current tile and a countdown
    // to the end of its cube (cubes are padded to TPC tiles in memory; a ragged cube's padding tiles are skipped).
    struct Stream {
        const unsigned char *tile;
        int j, t, nt;
    };
    auto stream_begin = [&](const uint16_t *base) -> Stream {
        Stream q;
        q.tile = reinterpret_cast<const unsigned char *>(base + (size_t)kv * g.N * g.TPC * (KEY_TILE * D));
        q.j = 0;
        q.t = 0;
        q.nt = tiles_of(0);
        return q;
    };
    auto stream_next = [&](Stream &q) __attribute__((always_inline)) {
        if (q.t + 1 < q.nt) {
            ++q.t;
            q.tile += C::CHUNK;
        } else {
            q.tile += (size_t)(g.TPC - q.t) * C::CHUNK;
            q.j = min(q.j + 1, i);  // past the end nothing is issued; the index only has to stay valid
            q.t = 0;
            q.nt = tiles_of(q.j);
        }
    };
    const uint32_t lds_piece =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + (uint32_t)(wave * C::DMA * 1024));
    const uint32_t src_piece = (uint32_t)(wave * C::DMA * 1024 + lane * 16);
    auto issue = [&](const Stream &q, int off_bytes) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < C::DMA; ++u)
            dma_1k_s(lds_piece + (uint32_t)(off_bytes + u * 1024), q.tile, src_piece + (uint32_t)(u * 1024));
    };
    auto next_stage = [](int st) -> int { return st + 1 == NST ? 0 : st + 1; };

    // rows of this wavefront: slab k of the block belongs to wavefront k % WAVES as its slot k / WAVES
    int lr[NS];
    int ns = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int idx = 16 * (wave + WAVES * s) + n16;
        lr[s] = idx < Mrows ? idx : MMAX;
        if (16 * (wave + WAVES * s) < Mrows) ns = s + 1;
    }
    int rank_lo = 0;
    if (ns > 0) rank_lo = rrank[16 * wave];
    rank_lo = __builtin_amdgcn_readfirstlane(rank_lo);

    // prologue: K(0..2), V(0..1)
    Stream sk = stream_begin(Kp), sv = stream_begin(Vt);
    int tk = 0, tv = 0;  // index of the tile sk / sv points at
    for (; tk < NST && tk < ntiles; ++tk) {
        issue(sk, C::OFF_K + tk * C::CHUNK);
        stream_next(sk);
    }
    for (; tv < NST - 1 && tv < ntiles; ++tv) {
        issue(sv, C::OFF_V + tv * C::CHUNK);
        stream_next(sv);
    }

    bf16x8 qf[NS][KSTEPS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const uint16_t *qrow = Q + (size_t)rowid[lr[s]] * D + 8 * q4;
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) qf[s][c] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * c);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) asm volatile("" : "+v"(qf[s][c]));

    const float c2 = 1.44269504088896340736f / sqrtf((float)D);
    int lim[NS];
    float m_run[NS];
    f32x4 l_run[NS];  // every element holds the row's running sum
    f32x4 oacc[NS][DT];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        m_run[s] = -1e30f;
        l_run[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < DT; ++e) oacc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    bool rsel[NS];
    uint32_t mword[NS];
    int mword_idx = -1;
#pragma unroll
    for (int s = 0; s < NS; ++s) { rsel[s] = true; mword[s] = 0; }
    int jsize = 0;
    // per-cube constants of the softmax: key limits of every row, and (MASKED) whether the row attends the cube
    auto enter_cube = [&](int j) __attribute__((always_inline)) {
        const bool own = (j == i);
        jsize = own ? qsize : (g.ragged ? csize[j] : g.Cmax);
#pragma unroll
        for (int s = 0; s < NS; ++s) lim[s] = own ? min(rrank[lr[s]], jsize - 1) : jsize - 1;
        if (MASKED) {
            if (own) {
#pragma unroll
                for (int s = 0; s < NS; ++s) rsel[s] = true;
            } else {
                if ((j >> 5) != mword_idx) {
                    mword_idx = j >> 5;
#pragma unroll
                    for (int s = 0; s < NS; ++s) mword[s] = sel_mask[(size_t)rowid[lr[s]] * g.words + mword_idx];
                }
#pragma unroll
                for (int s = 0; s < NS; ++s) rsel[s] = (mword[s] >> (j & 31)) & 1u;
            }
        }
    };
    TilePos cc = first_tile();  // the tile whose softmax comes next
    enter_cube(cc.j);

    f32x4 sacc[NS][4];
    bf16x8 pf[NS][2];
    auto softmax_step = [&]() __attribute__((always_inline)) {
        const bool own = (cc.j == i);
        const int key0 = KEY_TILE * cc.t;
        const bool need_mask = (key0 + KEY_TILE > jsize) || (own && key0 + KEY_TILE - 1 > rank_lo);
#ifdef PP_NO_SOFTMAX
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int kg = 0; kg < 4; ++kg)
#pragma unroll
                for (int v = 0; v < 4; ++v) pf[s][kg >> 1][4 * (kg & 1) + v] = (__bf16)sacc[s][kg][v];
#else
        softmax_tile<D, 0, NS, NS, MASKED>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4, rsel);
#endif
        const int j0 = cc.j;
        advance(cc);
        if (cc.j != j0) enter_cube(cc.j);
    };

    tile_barrier();  // the prologue's tiles have landed
    int st = 0;      // stage of tile T
    // opens slot b(T): waits for the loads started one slot b ago but one, then refills the two stages that
    // fell free (K(T)'s with K(T+3), V(T-1)'s with V(T+2))
    auto open_slot_b = [&](int T) __attribute__((always_inline)) {
        if (T + 2 < ntiles) dma_barrier<2 * C::DMA>();
        else tile_barrier();
        const int st_prev = st == 0 ? NST - 1 : st - 1;
        if (tk < ntiles) {
            issue(sk, C::OFF_K + st * C::CHUNK);
            stream_next(sk);
            ++tk;
        }
        if (tv < ntiles) {
            issue(sv, C::OFF_V + st_prev * C::CHUNK);
            stream_next(sv);
            ++tv;
        }
    };
    // The first and the last tile are peeled off the loops: a loop body with a conditional MFMA phase would merge
    // two versions of every accumulator at its end, at the price of a register copy each.
    if (!set_y) {
        mfma_phase<D, NS, PF, false, true>(nullptr, smem + C::OFF_K, n16, q4, pf, oacc, l_run, qf, sacc);
        for (int T = 0; T + 1 < ntiles; ++T) {
            lds_barrier();  // slot a(T)
            softmax_step();
            open_slot_b(T);
            const unsigned char *vt = smem + C::OFF_V + st * C::CHUNK;
            st = next_stage(st);
            mfma_phase<D, NS, PF, true, true>(vt, smem + C::OFF_K + st * C::CHUNK, n16, q4, pf, oacc, l_run, qf, sacc);
        }
        lds_barrier();
        softmax_step();
        open_slot_b(ntiles - 1);
        mfma_phase<D, NS, PF, true, false>(smem + C::OFF_V + st * C::CHUNK, nullptr, n16, q4, pf, oacc, l_run, qf, sacc);
    } else {
        lds_barrier();  // slot a(0)
        mfma_phase<D, NS, PF, false, true>(nullptr, smem + C::OFF_K, n16, q4, pf, oacc, l_run, qf, sacc);
        open_slot_b(0);
        softmax_step();
        for (int T = 1; T < ntiles; ++T) {
            const unsigned char *vt = smem + C::OFF_V + st * C::CHUNK;  // V(T-1)
            st = next_stage(st);
            lds_barrier();  // slot a(T)
            mfma_phase<D, NS, PF, true, true>(vt, smem + C::OFF_K + st * C::CHUNK, n16, q4, pf, oacc, l_run, qf, sacc);
            open_slot_b(T);
            softmax_step();
        }
        mfma_phase<D, NS, PF, true, false>(smem + C::OFF_V + st * C::CHUNK, nullptr, n16, q4, pf, oacc, l_run, qf, sacc);
    }

    // ---- normalise and write out (no direct-to-LDS load may outlive the workgroup's LDS allocation)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        if (lr[s] == MMAX) continue;
        const int rid = rowid[lr[s]];
        const float inv = 1.0f / l_run[s][0];
        uint16_t *orow = O + (size_t)rid * D + 4 * q4;
#pragma unroll
        for (int e = 0; e < DT; ++e) {
            const uint32_t w0 = (uint32_t)float_to_bf16_bits(oacc[s][e][0] * inv) |
                                ((uint32_t)float_to_bf16_bits(oacc[s][e][1] * inv) << 16);
            const uint32_t w1 = (uint32_t)float_to_bf16_bits(oacc[s][e][2] * inv) |
                                ((uint32_t)float_to_bf16_bits(oacc[s][e][3] * inv) << 16);
            *reinterpret_cast<uint2 *>(orow + 16 * e) = make_uint2(w0, w1);
        }
        if (lse != nullptr && q4 == 0) lse[rid] = (m_run[s] + log2f(l_run[s][0])) * 0.69314718055994530942f;
    }
}

// ---- choice between the compacting and the masked kernel: the share of candidate cubes the rows select, from a
// sample of rows.  One workgroup; writes 1 (compact) or 2 (masked) to *flag.
constexpr int DENSITY_THREADS = 1024;
constexpr int DENSITY_MAX_ROWS = 16384;
constexpr int MASKED_ABOVE_PERCENT = 35;  // measured crossover of the two kernels on MI355X

__global__ __launch_bounds__(DENSITY_THREADS) void sel_density_kernel(Geom g, const uint32_t *__restrict__ sel_mask,
                                                                      int *__restrict__ flag)
{
    __shared__ unsigned long long acc[2];
    if (threadIdx.x == 0) acc[0] = acc[1] = 0ull;
    __syncthreads();
    const long long R = (long long)g.S * g.Hq;
    const long long stride = max(1ll, R / DENSITY_MAX_ROWS);
    unsigned long long sel = 0, cand = 0;
    for (long long r = threadIdx.x * stride; r < R; r += DENSITY_THREADS * stride) {
        cand += (unsigned long long)cube_of_token(g, (int)(r / g.Hq));
        const uint32_t *mr = sel_mask + (size_t)r * g.words;
        for (int w = 0; w < g.words; ++w) sel += __popc(mr[w]);
    }
    atomicAdd(&acc[0], sel);
    atomicAdd(&acc[1], cand);
    __syncthreads();
    if (threadIdx.x == 0) *flag = (acc[0] * 100ull > acc[1] * (unsigned long long)MASKED_ABOVE_PERCENT) ? 2 : 1;
}

template <int D, bool SPARSE, bool MASKED>
static hipError_t launch_fwd(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                             const int *mode_flag, int my_mode, uint16_t *O, float *lse, hipStream_t st)
{
    using C = Fwd<D, SPARSE>;
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const uint16_t *Vt = Kp + half_elems;
    const int32_t *csize = reinterpret_cast<const int32_t *>(Vt + half_elems);
    const int nblk_max = (g.G * g.Cmax + C::MMAX - 1) / C::MMAX;
    const dim3 grid((unsigned)((size_t)((g.N * g.Hkv + 7) / 8) * nblk_max * 8));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_fwd_kernel<D, SPARSE, MASKED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attn_fwd_kernel<D, SPARSE, MASKED>), grid, dim3(C::THREADS), C::BYTES, st, g, Q, Kp, Vt, csize,
                       sel_mask, mode_flag, my_mode, O, lse);
    return hipGetLastError();
}

template <int D, bool MASKED>
static hipError_t launch_pp(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                            const int *mode_flag, int my_mode, uint16_t *O, float *lse, hipStream_t st)
{
    using C = Pp<D>;
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const uint16_t *Vt = Kp + half_elems;
    const int32_t *csize = reinterpret_cast<const int32_t *>(Vt + half_elems);
    const int nblk_max = (g.G * g.Cmax + C::MMAX - 1) / C::MMAX;
    const dim3 grid((unsigned)((size_t)((g.N * g.Hkv + 7) / 8) * nblk_max * 8));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_pp_kernel<D, MASKED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attn_pp_kernel<D, MASKED>), grid, dim3(C::THREADS), C::BYTES, st, g, Q, Kp, Vt, csize, sel_mask,
                       mode_flag, my_mode, O, lse);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_attn_d(const Geom &g, const uint16_t *Q, void *packed, const uint32_t *sel_mask,
                                int sparse_kernel, uint16_t *O, float *lse, hipStream_t st)
{
    static const bool pp = getenv("ADASPARK_PP") == nullptr || atoi(getenv("ADASPARK_PP")) != 0;
    if (sel_mask == nullptr)
        return pp ? launch_pp<D, false>(g, Q, packed, nullptr, nullptr, 0, O, lse, st)
                  : launch_fwd<D, false, false>(g, Q, packed, nullptr, nullptr, 0, O, lse, st);
    if (sparse_kernel == ADASPARK_SPARSE_COMPACT)
        return launch_fwd<D, true, false>(g, Q, packed, sel_mask, nullptr, 0, O, lse, st);
    if (sparse_kernel == ADASPARK_SPARSE_MASKED)
        return pp ? launch_pp<D, true>(g, Q, packed, sel_mask, nullptr, 0, O, lse, st)
                  : launch_fwd<D, false, true>(g, Q, packed, sel_mask, nullptr, 0, O, lse, st);
    // automatic: estimate the density on the device, enqueue both kernels, the one not chosen returns at once
    int *flag = reinterpret_cast<int *>(reinterpret_cast<char *>(packed) + attn_workspace_bytes(g) - 16);
    hipLaunchKernelGGL(sel_density_kernel, dim3(1), dim3(DENSITY_THREADS), 0, st, g, sel_mask, flag);
    hipError_t e = launch_fwd<D, true, false>(g, Q, packed, sel_mask, flag, 1, O, lse, st);
    if (e != hipSuccess) return e;
    return pp ? launch_pp<D, true>(g, Q, packed, sel_mask, flag, 2, O, lse, st)
              : launch_fwd<D, false, true>(g, Q, packed, sel_mask, flag, 2, O, lse, st);
}

hipError_t launch_attn(const Geom &g, const uint16_t *Q, void *packed, const uint32_t *sel_mask, int sparse_kernel,
                       uint16_t *O, float *lse, hipStream_t st)
{
    if (g.D == 64) return launch_attn_d<64>(g, Q, packed, sel_mask, sparse_kernel, O, lse, st);
    return launch_attn_d<128>(g, Q, packed, sel_mask, sparse_kernel, O, lse, st);
}

}  // namespace adaspark
