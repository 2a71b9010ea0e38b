// Sparse (Eq. 3 + own-cube rule, Sec. 3.2) and dense causal attention: flash attention over the packed KV copy
// with per-cube row compaction.
//
// Selection is per (token, query head), so rows that share a query tile select independent cube subsets; a
// mask-based tile kernel would execute dense FLOPs.  Here a workgroup owns up to MMAX query rows of one
// (query cube i, KV head) -- all query heads of the GQA group, token-major -- and keeps their online-softmax
// state (fp32 O, m, l) in LDS (MI355X: 160 KB per CU).  It walks the key cubes j <= i that any of its rows
// attends.  For each cube
//   1. every wavefront ballots the selection bits of all rows and so knows the (sorted) list of rows that
//      attend j (dense mode, own cube: all rows); no LDS list and no extra barrier are needed,
//   2. the list is cut into 16-row slabs, dealt round-robin to the eight wavefronts (two per SIMD, so one
//      wavefront's softmax can overlap the other's MFMA),
//   3. per slab the Q operands are gathered (prefetched under the previous cube's last tile), the rows' state
//      moves from LDS into MFMA accumulators, flash attention runs over the cube's 64-key tiles with
//      mfma_f32_16x16x32_bf16 (S^T = K.Q^T, O^T += V^T.P^T: a lane owns one query row and a quarter of the
//      keys of a tile), and the state moves back.
// Executed MFMA work is the selected (row, cube) pairs rounded up to 16 rows per workgroup and cube.  In dense
// mode the row set never changes and the state stays in registers.
//
// K and V^T tiles come from the packed, pre-swizzled copy (kvtile.h).  The tile stream K0 V0 K1 V1 ... rotates
// through three LDS buffers; a tile is fetched into registers two phases before it is needed and written to
// the buffer that was read two phases ago, so one barrier per phase (two per key tile) is enough and no wave
// ever waits on a load it has just issued.
#include <type_traits>

#include "kvtile.h"

namespace adaspark {

constexpr int FWD_WAVES = 8;  // two wavefronts per SIMD
constexpr int FWD_THREADS = 64 * FWD_WAVES;
constexpr int FWD_NS = 2;     // 16-row slabs a wavefront works on at a time

template <int D, bool SPARSE>
struct Fwd {
    static constexpr int WAVES = FWD_WAVES;
    static constexpr int THREADS = FWD_THREADS;
    static constexpr int NS = FWD_NS;
    static constexpr int MMAX = SPARSE ? 192 : 16 * NS * WAVES;  // rows per workgroup (sparse: what LDS can hold)
    static constexpr int GROUPS = (MMAX + 63) / 64;              // 64-row ballot groups
    static constexpr int CHUNK = KEY_TILE * D * 2;               // bytes of a K tile (= bytes of a V^T tile)
    static constexpr int CPT = CHUNK / 16 / THREADS;             // 16-byte pieces of a tile per thread
    static constexpr int OST = D + 4;  // floats per state row (padded: 16 rows start in 16 different bank groups)
    static constexpr int SMALL = (((MMAX + 1) * 4 + 15) / 16) * 16;
    static constexpr int OFF_KV = 0;
    static constexpr int OFF_ROWID = OFF_KV + 3 * CHUNK;
    static constexpr int OFF_RANK = OFF_ROWID + SMALL;
    static constexpr int OFF_UMASK = OFF_RANK + SMALL;
    static constexpr int OFF_M = OFF_UMASK + (ADASPARK_MAX_CUBES / 32) * 4;
    static constexpr int OFF_L = OFF_M + SMALL;
    static constexpr int OFF_O = OFF_L + SMALL;
    static constexpr int BYTES = SPARSE ? OFF_O + (MMAX + 1) * OST * 4 : OFF_M;
    static_assert(MMAX <= 16 * NS * WAVES, "every attending row needs a slab");
    static_assert(CPT >= 1, "tile smaller than one 16-byte piece per thread");
};

// waits for this wavefront's LDS traffic, then the workgroup barrier; global loads in flight stay in flight
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// max / sum over the four lanes {n, n+16, n+32, n+48} that share a query row
__device__ __forceinline__ float quad_max(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_sum(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Position of the k-th (0-based) set bit of m; k < popcount(m).
__device__ __forceinline__ int kth_set_bit(unsigned long long m, int k)
{
    int pos = 0;
#pragma unroll
    for (int w = 32; w > 0; w >>= 1) {
        const unsigned long long low = m & ((1ull << w) - 1ull);
        const int c = __popcll(low);
        if (k >= c) { k -= c; m >>= w; pos += w; }
        else m = low;
    }
    return pos;
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
template <int D, int S0, int S1, int NS>
__device__ __forceinline__ void softmax_tile(f32x4 (&sacc)[NS][4], bf16x8 (&pf)[NS][2], f32x4 (&oacc)[NS][D / 16],
                                             float (&m_run)[NS], float (&l_run)[NS], const int (&lim)[NS], int key0,
                                             bool need_mask, float c2, int q4)
{
#pragma unroll
    for (int s = S0; s < S1; ++s) {
        if (need_mask) {
#pragma unroll
            for (int kg = 0; kg < 4; ++kg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int kr = key0 + 32 * (kg >> 1) + 8 * q4 + 4 * (kg & 1) + v;
                    if (kr > lim[s]) sacc[s][kg][v] = -INFINITY;
                }
        }
        float mx = fmaxf(fmaxf(sacc[s][0][0], sacc[s][0][1]), fmaxf(sacc[s][0][2], sacc[s][0][3]));
#pragma unroll
        for (int kg = 1; kg < 4; ++kg)
            mx = fmaxf(fmaxf(mx, fmaxf(sacc[s][kg][0], sacc[s][kg][1])), fmaxf(sacc[s][kg][2], sacc[s][kg][3]));
        mx = quad_max(mx);
        const float m_new = fmaxf(m_run[s], mx * c2);
        const float alpha = __builtin_amdgcn_exp2f(m_run[s] - m_new);
        float rs = 0.f;
#pragma unroll
        for (int kg = 0; kg < 4; ++kg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[s][kg][v], c2, -m_new));
                rs += p;
                pf[s][kg >> 1][4 * (kg & 1) + v] = (__bf16)p;
            }
        rs = quad_sum(rs);
        l_run[s] = l_run[s] * alpha + rs;
        // the running maximum rarely moves after the first tiles: rescale only when some row needs it
        if (__ballot(m_new != m_run[s]) != 0ull) {
#pragma unroll
            for (int e = 0; e < D / 16; ++e) oacc[s][e] *= alpha;
        }
        m_run[s] = m_new;
    }
}

// O^T += V^T.P^T for one 64-key tile; one V^T operand load serves all slabs of the range.
template <int D, int S0, int S1, int NS>
__device__ __forceinline__ void pv_tile(const unsigned char *vt, int n16, int q4, const bf16x8 (&pf)[NS][2],
                                        f32x4 (&oacc)[NS][D / 16])
{
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
    int j;   // key cube (> i: past the end)
    int t;   // 64-key tile inside the cube
    int nt;  // tiles of cube j this workgroup reads
};

template <int D, bool SPARSE>
__global__ __launch_bounds__(FWD_THREADS) void attn_fwd_kernel(
    Geom g, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Kp, const uint16_t *__restrict__ Vt,
    const uint32_t *__restrict__ sel_mask, uint16_t *__restrict__ O, float *__restrict__ lse)
{
    using C = Fwd<D, SPARSE>;
    constexpr int NS = C::NS, MMAX = C::MMAX, OST = C::OST, CPT = C::CPT, THREADS = C::THREADS;
    constexpr int WAVES = C::WAVES, GROUPS = C::GROUPS;
    constexpr int KSTEPS = D / 32;  // MFMA k-steps of S^T (32 head-dim elements each)
    constexpr int DT = D / 16;      // 16-wide tiles of O^T
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
    unsigned char *kvbuf = smem + C::OFF_KV;
    int *rowid = reinterpret_cast<int *>(smem + C::OFF_ROWID);
    int *rrank = reinterpret_cast<int *>(smem + C::OFF_RANK);
    uint32_t *umask = reinterpret_cast<uint32_t *>(smem + C::OFF_UMASK);
    float *mst = reinterpret_cast<float *>(smem + C::OFF_M);
    float *lst = reinterpret_cast<float *>(smem + C::OFF_L);
    float *ost = reinterpret_cast<float *>(smem + C::OFF_O);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;

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
        for (int x = tid; x < (MMAX + 1) * OST; x += THREADS) ost[x] = 0.f;
        for (int w = tid; w < g.words; w += THREADS) umask[w] = 0;
    }
    __syncthreads();
    // every wavefront tracks the selection bits of all rows: lane l speaks for rows l, l+64, ...
    int mrid[GROUPS];  // global row id behind (group, lane); -1: no such row
#pragma unroll
    for (int gq = 0; gq < GROUPS; ++gq) {
        const int r = 64 * gq + lane;
        mrid[gq] = r < Mrows ? rowid[r] : -1;
    }
    if (SPARSE) {
        for (int r = tid; r < Mrows; r += THREADS) {
            const uint32_t *mr = sel_mask + (size_t)rowid[r] * g.words;
            for (int w = 0; w < g.words; ++w) {
                const uint32_t bits = mr[w];
                if (bits) atomicOr(&umask[w], bits);
            }
        }
        __syncthreads();
    }

    // ---- the tile stream of this workgroup
    auto tiles_of = [&](int j) -> int {
        if (j == i) return min((qsize + KEY_TILE - 1) / KEY_TILE, max_rank / KEY_TILE + 1);
        return (cube_box(g, j).size() + KEY_TILE - 1) / KEY_TILE;
    };
    // next key cube after j that some row of this workgroup attends (the own cube i always is); i+1: none
    auto next_cube = [&](int j) -> int {
        if (!SPARSE) return j + 1;
        int c = j + 1;
        while (c < i) {
            const uint32_t w = umask[c >> 5] >> (c & 31);
            if (w) return min(c + __ffs(w) - 1, i);
            c = (c | 31) + 1;
        }
        return j < i ? i : i + 1;
    };
    auto advance = [&](const TilePos &p) -> TilePos {
        TilePos n;
        if (p.t + 1 < p.nt) { n.j = p.j; n.t = p.t + 1; n.nt = p.nt; }
        else {
            n.j = next_cube(p.j);
            n.t = 0;
            n.nt = n.j <= i ? tiles_of(n.j) : 0;
        }
        return n;
    };
    auto tile_ptr = [&](const uint16_t *base, const TilePos &p) -> const u32x4 * {
        return reinterpret_cast<const u32x4 *>(base + ((((size_t)kv * g.N + p.j) * g.TPC) + p.t) * (size_t)(KEY_TILE * D));
    };
    auto fetch = [&](u32x4 (&r)[CPT], const u32x4 *src) {
#pragma unroll
        for (int u = 0; u < CPT; ++u) r[u] = src[tid + THREADS * u];
    };
    auto stash = [&](const u32x4 (&r)[CPT], int buf) {
        u32x4 *dst = reinterpret_cast<u32x4 *>(kvbuf + buf * C::CHUNK);
#pragma unroll
        for (int u = 0; u < CPT; ++u) dst[tid + THREADS * u] = r[u];
    };

    // ---- slabs of this wavefront for cube j.  The rows that attend j, in row order, are cut into 16-row slabs;
    // slab k goes to wavefront k % WAVES as its slot k / WAVES.  lr[s]: workgroup row in column n16 of slot s
    // (MMAX: padding column); ns: slots in use; lo/hi: smallest/largest rank among the wavefront's rows.
    int cw = -1;  // mask word index cached in wbits
    uint32_t wbits[GROUPS];
#pragma unroll
    for (int gq = 0; gq < GROUPS; ++gq) wbits[gq] = 0;
    auto slab_rows = [&](int j, int (&lr)[NS], int &ns, int &lo, int &hi) {
        int total;
        unsigned long long bal[GROUPS];
        const bool all = !SPARSE || j == i;
        if (all) total = Mrows;
        else {
            if ((j >> 5) != cw) {
                cw = j >> 5;
#pragma unroll
                for (int gq = 0; gq < GROUPS; ++gq)
                    wbits[gq] = mrid[gq] >= 0 ? sel_mask[(size_t)mrid[gq] * g.words + cw] : 0u;
            }
            total = 0;
#pragma unroll
            for (int gq = 0; gq < GROUPS; ++gq) {
                bal[gq] = __ballot((wbits[gq] >> (j & 31)) & 1u);
                total += __popcll(bal[gq]);
            }
        }
        const int nslab = (total + 15) >> 4;
        ns = nslab > wave ? (nslab - wave + WAVES - 1) / WAVES : 0;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            int idx = 16 * (wave + WAVES * s) + n16;
            int r = MMAX;
            if (idx < total) {
                if (all) r = idx;
                else {
                    int base = 0;
#pragma unroll
                    for (int gq = 0; gq < GROUPS; ++gq) {
                        const int c = __popcll(bal[gq]);
                        if (r == MMAX) {
                            if (idx < c) r = base + kth_set_bit(bal[gq], idx);
                            else { idx -= c; base += 64; }
                        }
                    }
                }
            }
            lr[s] = r;
        }
        // rows are sorted by rank: the first column of slot 0 and the last used column of the last slot bound them
        lo = hi = 0;
        if (all && ns > 0) {
            lo = rrank[16 * wave];
            hi = rrank[min(16 * (wave + WAVES * (ns - 1)) + 15, total - 1)];
        }
    };
    auto load_q = [&](const int (&lr)[NS], int ns, bf16x8 (&qf)[NS][KSTEPS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < ns) {
                const uint16_t *qrow = Q + (size_t)rowid[lr[s]] * D + 8 * q4;
#pragma unroll
                for (int c = 0; c < KSTEPS; ++c) qf[s][c] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * c);
            }
    };

    const float c2 = 1.44269504088896340736f / sqrtf((float)D);

    TilePos cur, nxt;
    cur.j = SPARSE ? next_cube(-1) : 0;
    cur.t = 0;
    cur.nt = tiles_of(cur.j);
    nxt = advance(cur);

    u32x4 gk[CPT], gv[CPT];
    fetch(gk, tile_ptr(Kp, cur));
    fetch(gv, tile_ptr(Vt, cur));

    int lr[NS], ns, rank_lo, rank_hi;
    bf16x8 qf[NS][KSTEPS];
    slab_rows(cur.j, lr, ns, rank_lo, rank_hi);
    load_q(lr, ns, qf);

    // online-softmax state of the slabs being worked on
    int lim[NS];
    float m_run[NS], l_run[NS];
    f32x4 oacc[NS][DT];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        m_run[s] = -1e30f;
        l_run[s] = 0.f;
#pragma unroll
        for (int e = 0; e < DT; ++e) oacc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto set_limits = [&](int j) {
        const bool own = (j == i);
        const int jsize = own ? qsize : cube_box(g, j).size();
#pragma unroll
        for (int s = 0; s < NS; ++s) lim[s] = own ? min(rrank[lr[s]], jsize - 1) : jsize - 1;
    };
    auto state_in = [&]() {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < ns) {
                m_run[s] = mst[lr[s]];
                l_run[s] = lst[lr[s]];
#pragma unroll
                for (int e = 0; e < DT; ++e)
                    oacc[s][e] = *reinterpret_cast<const f32x4 *>(&ost[lr[s] * OST + 16 * e + 4 * q4]);
            }
    };
    auto state_out = [&]() {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < ns) {
#pragma unroll
                for (int e = 0; e < DT; ++e)
                    *reinterpret_cast<f32x4 *>(&ost[lr[s] * OST + 16 * e + 4 * q4]) = oacc[s][e];
                if (q4 == 0) {
                    mst[lr[s]] = m_run[s];
                    lst[lr[s]] = l_run[s];
                }
            }
    };
    set_limits(cur.j);  // first cube: the state registers already hold the initial state

    stash(gk, 0);
    if (nxt.j <= i) fetch(gk, tile_ptr(Kp, nxt));
    int bk = 0;             // LDS buffer of K(cur); V(cur) -> bk+1, K(nxt) -> bk+2 (mod 3)
    bool new_slabs = false;  // the slabs changed at the last cube boundary: their state is still in LDS

    while (true) {
        const bool own = (cur.j == i);
        const bool has_next = nxt.j <= i;
        const bool cube_ends = has_next && nxt.j != cur.j;
        const int jsize = own ? qsize : cube_box(g, cur.j).size();
        const int key0 = KEY_TILE * cur.t;
        const bool active = ns > 0 && !(own && key0 > rank_hi);
        const bool need_mask = (key0 + KEY_TILE > jsize) || (own && key0 + KEY_TILE - 1 > rank_lo);
        const int bv = bk == 2 ? 0 : bk + 1, bn = bv == 2 ? 0 : bv + 1;

        // the next cube's slabs are worked out under this cube's last tile
        int lr_n[NS], ns_n = 0, lo_n = 0, hi_n = 0;
        if (SPARSE && cube_ends) slab_rows(nxt.j, lr_n, ns_n, lo_n, hi_n);

        f32x4 sacc[NS][4];
        bf16x8 pf[NS][2];
        const int nsl = active ? ns : 0;  // wave-uniform
        lds_barrier();  // K(cur) is in buffer bk; at a cube boundary every row's state is back in LDS
        if (SPARSE && new_slabs) state_in();
        {
            const unsigned char *kt = kvbuf + bk * C::CHUNK;
            if (SPARSE) {
                // slab counts vary from cube to cube: one guarded block per slab
                if (nsl >= 1) qk_tile<D, 0, 1, NS>(kt, n16, q4, qf, sacc);
                if (NS >= 2 && nsl >= 2) qk_tile<D, 1, NS, NS>(kt, n16, q4, qf, sacc);
            } else if (nsl) {
                // fixed row set: all slabs, padding columns of a partial slab compute on the scratch row
                qk_tile<D, 0, NS, NS>(kt, n16, q4, qf, sacc);
            }
        }
        // this cube's Q operands have had their last use: the next cube's arrive under the softmax and P.V
        if (SPARSE && cube_ends) load_q(lr_n, ns_n, qf);
        stash(gv, bv);  // V(cur)
        if (has_next) fetch(gv, tile_ptr(Vt, nxt));
        if (SPARSE) {
            if (nsl >= 1) softmax_tile<D, 0, 1, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4);
            if (NS >= 2 && nsl >= 2)
                softmax_tile<D, 1, NS, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4);
        } else if (nsl) {
            softmax_tile<D, 0, NS, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4);
        }
        lds_barrier();  // V(cur) is in buffer bv
        {
            const unsigned char *vt = kvbuf + bv * C::CHUNK;
            if (SPARSE) {
                if (nsl >= 1) pv_tile<D, 0, 1, NS>(vt, n16, q4, pf, oacc);
                if (NS >= 2 && nsl >= 2) pv_tile<D, 1, NS, NS>(vt, n16, q4, pf, oacc);
            } else if (nsl) {
                pv_tile<D, 0, NS, NS>(vt, n16, q4, pf, oacc);
            }
        }
        new_slabs = false;
        if (!has_next) break;
        stash(gk, bn);  // K(nxt)
        const TilePos nn = advance(nxt);
        if (nn.j <= i) fetch(gk, tile_ptr(Kp, nn));

        if (cube_ends) {
            if (SPARSE) {
                // slabs move between wavefronts from cube to cube: state back to LDS now, the new slabs'
                // state out of LDS after the next barrier
                state_out();
                ns = ns_n;
                rank_lo = lo_n;
                rank_hi = hi_n;
#pragma unroll
                for (int s = 0; s < NS; ++s) lr[s] = lr_n[s];
                new_slabs = true;
            }
            set_limits(nxt.j);
        }
        cur = nxt;
        nxt = nn;
        bk = bn;
    }

    // ---- normalise and write out
    if (SPARSE) {
        state_out();
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
            const float inv = 1.0f / l_run[s];
            uint16_t *orow = O + (size_t)rid * D + 4 * q4;
#pragma unroll
            for (int e = 0; e < DT; ++e) {
                const uint32_t w0 = (uint32_t)float_to_bf16_bits(oacc[s][e][0] * inv) |
                                    ((uint32_t)float_to_bf16_bits(oacc[s][e][1] * inv) << 16);
                const uint32_t w1 = (uint32_t)float_to_bf16_bits(oacc[s][e][2] * inv) |
                                    ((uint32_t)float_to_bf16_bits(oacc[s][e][3] * inv) << 16);
                *reinterpret_cast<uint2 *>(orow + 16 * e) = make_uint2(w0, w1);
            }
            if (lse != nullptr && q4 == 0) lse[rid] = (m_run[s] + log2f(l_run[s])) * 0.69314718055994530942f;
        }
    }
}

template <int D, bool SPARSE>
static hipError_t launch_fwd(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                             uint16_t *O, float *lse, hipStream_t st)
{
    using C = Fwd<D, SPARSE>;
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const uint16_t *Vt = Kp + (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const int nblk_max = (g.G * g.Cmax + C::MMAX - 1) / C::MMAX;
    const dim3 grid((unsigned)((size_t)((g.N * g.Hkv + 7) / 8) * nblk_max * 8));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_fwd_kernel<D, SPARSE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attn_fwd_kernel<D, SPARSE>), grid, dim3(C::THREADS), C::BYTES, st, g, Q, Kp, Vt, sel_mask, O,
                       lse);
    return hipGetLastError();
}

hipError_t launch_attn(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask, uint16_t *O,
                       float *lse, hipStream_t st)
{
    if (sel_mask != nullptr) {
        if (g.D == 64) return launch_fwd<64, true>(g, Q, packed, sel_mask, O, lse, st);
        return launch_fwd<128, true>(g, Q, packed, sel_mask, O, lse, st);
    }
    if (g.D == 64) return launch_fwd<64, false>(g, Q, packed, nullptr, O, lse, st);
    return launch_fwd<128, false>(g, Q, packed, nullptr, O, lse, st);
}

}  // namespace adaspark
