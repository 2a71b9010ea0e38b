// Sparse attention (Eq. 3 + own-cube rule, Sec. 3.2) with per-cube row compaction: executed MFMA work follows the
// selection.
//
// Selection is per (token, query head), so rows that share a query tile select independent cube subsets.  A
// workgroup owns up to MMAX query rows of one (query cube i, KV head) -- all query heads of the GQA group,
// token-major -- and keeps their online-softmax state (fp32 O, m, l) in LDS (MI355X: 160 KB per CU).  It walks
// the key cubes j <= i that any of its rows attends.  For each cube
//   1. every wavefront ballots the selection bits of all rows and so knows the (sorted) list of rows that
//      attend j (own cube: all rows); no extra barrier is needed,
//   2. the list is cut into 16-row slabs, dealt round-robin to the eight wavefronts,
//   3. per slab the Q operands are gathered (a whole cube ahead), the rows' state moves from LDS into MFMA
//      accumulators, flash attention runs over the cube's 64-key tiles, and the state moves back.
// Executed MFMA work is the selected (row, cube) pairs rounded up to 16 rows per workgroup and cube; every cube
// that some row of the workgroup attends is streamed, one workgroup barrier per 64-key tile.  That fixed cost
// per tile makes this kernel the better one only when few cubes are selected (or whole workgroups agree on
// what they skip); otherwise the masked walk (attn_walk.hip) wins.
//
// K and V^T tiles go through two LDS stages: the loads of tile t+1 are started right after the barrier that
// opens tile t and waited for at the barrier that closes it.
#include "attn_tile.h"

namespace adaspark {

template <int D>
struct Compact {
    static constexpr int WAVES = 8;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int NS = FWD_NS;
    static constexpr int MMAX = 168;                 // rows per workgroup: what LDS can hold
    static constexpr int GROUPS = (MMAX + 63) / 64;  // 64-row ballot groups
    static constexpr int CHUNK = KEY_TILE * D * 2;   // bytes of a K tile (= bytes of a V^T tile)
    static constexpr int NBUF = 4;                   // LDS buffers: K and V^T of two tiles
    static constexpr int DMA = CHUNK / 1024 / WAVES; // 1 KB direct-to-LDS loads per wavefront and tile
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
    static constexpr int BYTES = OFF_O + (MMAX + 1) * OST * 4;
    static_assert(MMAX <= 16 * NS * WAVES, "every attending row needs a slab");
    static_assert(DMA >= 1, "a tile is at least 1 KB per wavefront");
    static_assert(BYTES <= 160 * 1024, "LDS of one CU");
};

// flags (may be null): the kernel-choice flags (geom.h).  A workgroup runs only if flags[FLAG_MODE] == my_mode and
// (kv_modes) its KV head has not been handed to the key-stationary kernel, so that all sparse kernels can be
// enqueued and the choice is made on the device.
template <int D>
__global__ __launch_bounds__(FWD_MAX_THREADS) void attn_compact_kernel(
    Geom g, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Kp, const uint16_t *__restrict__ Vt,
    const int32_t *__restrict__ csize, const uint32_t *__restrict__ sel_mask, const int *__restrict__ mode_flag,
    int my_mode, int kv_modes, uint16_t *__restrict__ O, float *__restrict__ lse)
{
    if (mode_flag != nullptr && mode_flag[FLAG_MODE] != my_mode) return;
    using C = Compact<D>;
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
    // A KV head normally stays on the same XCDs (grp % 8 = xcd: its K/V tiles are the ones that XCD's L2 holds).
    // When some heads are handed to the key-stationary kernel, the head is rotated with the cube instead, so that
    // the heads that remain still spread over all XCDs.
    const int rot = (kv_modes && mode_flag[FLAG_ACTIVE]) ? grp / g.Hkv : 0;
    const int kv = (grp % g.Hkv + rot) % g.Hkv;
    if (kv_modes && mode_flag[FLAG_KV + kv] == 3) return;
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
        mst[r] = -1e30f;
        lst[r] = 0.f;
        if (r == 0) {  // scratch row: read and written by the padding columns of a partial slab
            rowid[MMAX] = rid;
            rrank[MMAX] = 0;
            mst[MMAX] = -1e30f;
            lst[MMAX] = 0.f;
        }
    }
    for (int x = tid; x < (MMAX + 1) * OST / 4; x += THREADS)
        reinterpret_cast<f32x4 *>(ost)[x] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int w = tid; w < g.words; w += THREADS) umask[w] = 0;
    if (tid == 0) misc[0] = 0;
    __syncthreads();

    // ---- the cubes this workgroup attends (union over its rows), in order; the own cube i is always last
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
    const int ncubes = nsel + 1;
    __syncthreads();

    auto cube_at = [&](int k) -> int {
        return __builtin_amdgcn_readfirstlane((int)cubes[k]);
    };
    auto tiles_of = [&](int j) -> int {
        if (j == i) return own_tiles;
        return g.ragged ? (csize[j] + KEY_TILE - 1) / KEY_TILE : g.TPC;
    };
    // length of the tile stream
    {
        int part = 0;
        for (int k = tid; k < ncubes; k += THREADS) part += tiles_of((int)cubes[k]);
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
    const uint32_t lds_piece =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)kvbuf + (uint32_t)(wave * C::DMA * 1024));
    const uint32_t src_piece = (uint32_t)(wave * C::DMA * 1024 + lane * 16);
    auto issue = [&](const uint16_t *base, const TilePos &p, int buf) __attribute__((always_inline)) {
        // wave-uniform tile address (scalar registers) + per-lane byte offset
        const unsigned char *tile = reinterpret_cast<const unsigned char *>(
            base + ((((size_t)kv * g.N + p.j) * g.TPC) + p.t) * (size_t)(KEY_TILE * D));
#pragma unroll
        for (int u = 0; u < C::DMA; ++u)
            dma_1k_s(lds_piece + (uint32_t)(buf * C::CHUNK + u * 1024), tile, src_piece + (uint32_t)(u * 1024));
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
        const bool all = j == i;
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
    // Settled, the operands are turned into the score products' fp16 (attn_tile.h; this kernel applies the softmax
    // scale to the scores afterwards, so the conversion is exact within fp16's range).
    auto settle_q = [&](bf16x8 (&q)[KSTEPS]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) asm volatile("" : "+v"(q[c]));
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) q[c] = score_operand(q[c], 1.0f);
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
    bool attends[NS];  // the softmax takes a per-row flag; compacted rows all attend
#pragma unroll
    for (int s = 0; s < NS; ++s) attends[s] = true;
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
        if (new_slabs) {
            // cube boundary: the slabs (and with them rows) move between wavefronts.  Every wavefront wrote
            // its state back before the barrier.
            ns = ns_n;
            rank_lo = lo_n;
            rank_hi = hi_n;
#pragma unroll
            for (int s = 0; s < NS; ++s) lr[s] = lr_n[s];
            if (ns > 0) {
#pragma unroll
                for (int c = 0; c < KSTEPS; ++c) qf[0][c] = score_operand(qf_n[c], 1.0f);
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
        const int nsl = (ns > 0 && !(own && key0 > rank_hi)) ? ns : 0;  // wave-uniform
        const bool need_mask = (key0 + KEY_TILE > jsize) || (own && key0 + KEY_TILE - 1 > rank_lo);
        const bool cube_ends = cc.t + 1 == cc.nt && cc.k + 1 < ncubes;
        if (cc.t == 0 && cc.k + 1 < ncubes) {
            // first tile of a cube: work out the next cube's slabs and start fetching the Q operands of the
            // first one into registers of their own, a whole cube ahead of their use (they are gathered from
            // global memory).  They are copied over after the barrier that opens the next cube.
            slab_rows(cube_at(cc.k + 1), lr_n, ns_n, lo_n, hi_n);
            if (ns_n > 0) load_q(lr_n[0], qf_n);
        }
        // slab counts vary from cube to cube: one guarded block per slab
        if (nsl >= 1) {
            qk_tile<D, 0, 1, NS>(kt, n16, q4, qf, sacc);
            softmax_tile<D, 0, 1, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4, attends);
            pv_tile<D, 0, 1, NS>(vt, n16, q4, pf, oacc, l_run);
        }
        if (NS >= 2 && nsl >= 2) {
            qk_tile<D, 1, NS, NS>(kt, n16, q4, qf, sacc);
            softmax_tile<D, 1, NS, NS>(sacc, pf, oacc, m_run, l_run, lim, key0, need_mask, c2, q4, attends);
            pv_tile<D, 1, NS, NS>(vt, n16, q4, pf, oacc, l_run);
        }
        advance(cc);
        if (cube_ends) {
            state_out();
            new_slabs = true;
        }
    }

    // ---- normalise and write out (no direct-to-LDS load may outlive the workgroup's LDS allocation)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
}

template <int D>
static hipError_t launch_compact_d(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                                   const int *mode_flag, int my_mode, int kv_modes, uint16_t *O, float *lse, hipStream_t st)
{
    using C = Compact<D>;
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const uint16_t *Vt = Kp + half_elems;
    const int32_t *csize = reinterpret_cast<const int32_t *>(Vt + half_elems);
    const int nblk_max = (g.G * g.Cmax + C::MMAX - 1) / C::MMAX;
    const dim3 grid((unsigned)((size_t)((g.N * g.Hkv + 7) / 8) * nblk_max * 8));
    static LdsOptIn opted;
    const hipError_t e = opted.ensure(reinterpret_cast<const void *>(&attn_compact_kernel<D>), C::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attn_compact_kernel<D>), grid, dim3(C::THREADS), C::BYTES, st, g, Q, Kp, Vt, csize, sel_mask,
                       mode_flag, my_mode, kv_modes, O, lse);
    return hipGetLastError();
}

hipError_t launch_attn_compact(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                               const int *mode_flag, int my_mode, int kv_modes, uint16_t *O, float *lse, hipStream_t st)
{
    if (g.D == 64) return launch_compact_d<64>(g, Q, packed, sel_mask, mode_flag, my_mode, kv_modes, O, lse, st);
    return launch_compact_d<128>(g, Q, packed, sel_mask, mode_flag, my_mode, kv_modes, O, lse, st);
}

}  // namespace adaspark
