// Dense causal attention, and sparse attention (Eq. 3 + own-cube rule, Sec. 3.2) with the selection applied as a
// mask: every row walks every preceding cube.  Also the entry that chooses between this kernel and the
// compacting one (attn_compact.hip).
//
// Fixed-row walk with two wavefront sets in counter-phase.
//
// On a SIMD an MFMA keeps the matrix pipe busy for ~16 cycles, and vector instructions of another wavefront can
// issue underneath it; a wavefront alone cannot use that room, because its softmax needs its finished scores.  So
// a workgroup holds eight wavefronts, two per SIMD, and the two of a SIMD take the two halves of a tile's work in
// opposite order.  Per tile t every wavefront runs one MFMA phase -- P.V of tile t-1, then S = Q.K^T of tile t --
// and one softmax; set X (wavefronts 0-3) runs the MFMA phase first and the softmax of tile t after it, set Y (4-7)
// first runs the softmax of tile t-1 (one tile late) and then the MFMA phase:
//
//   slot t:   X: [P.V(t-1), S(t)]  softmax(t)
//             Y: softmax(t-1)      [P.V(t-1), S(t)]
//
// so that one wavefront's softmax runs under the other's MFMAs, with one workgroup barrier per tile.
//
// K and V^T tiles go through three LDS stages each (tile t in stage t % 3).  Slot t reads K(t) and V(t-1); after
// the barrier that opens it nobody reads K(t-1) or V(t-2) any more, and the direct-to-LDS loads of K(t+2) and
// V(t+1) go into their stages; they are waited for two barriers later (the loads started one tile ago may stay in
// flight).
#include "attn_tile.h"

namespace adaspark {

template <int D>
struct Walk {
    static constexpr int WAVES = 8;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int NS = FWD_NS;
    static constexpr int MMAX = 16 * NS * WAVES;  // 256 rows per workgroup
    static constexpr int NST = 3;  // LDS stages of K and of V^T
    static constexpr int PF = 4;   // operand loads in flight ahead of the MFMAs
    static constexpr int CHUNK = KEY_TILE * D * 2;
    static constexpr int DMA = CHUNK / 1024 / WAVES;
    static constexpr int SMALL = (((MMAX + 1) * 4 + 15) / 16) * 16;
    static constexpr int OFF_K = 0;
    static constexpr int OFF_V = OFF_K + NST * CHUNK;
    static constexpr int OFF_ROWID = OFF_V + NST * CHUNK;
    static constexpr int OFF_RANK = OFF_ROWID + SMALL;
    static constexpr int OFF_MISC = OFF_RANK + SMALL;
    // the cubes some row of the workgroup attends (sparse entry): union of the rows' mask words, then the list of
    // its set bits in cube order
    static constexpr int LIST_MAX = ADASPARK_MAX_CUBES;
    static constexpr int OFF_UNION = OFF_MISC + 16;
    static constexpr int OFF_LIST = OFF_UNION + LIST_MAX / 8;
    static constexpr int BYTES = OFF_LIST + LIST_MAX * 2;
    static_assert(DMA >= 1, "a tile is at least 1 KB per wavefront");
    static_assert(BYTES <= 160 * 1024, "LDS of one CU");
};


// Barrier that opens a slot: all direct-to-LDS loads but the newest KEEP of this wavefront have landed.  Nothing
// waits for LDS reads here: the operand reads of a slot are consumed by its MFMAs before the wavefront gets here.
template <int KEEP>
__device__ __forceinline__ void dma_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(KEEP) : "memory");
}

template <int D, bool MASKED>
__global__ __launch_bounds__(FWD_MAX_THREADS) void attn_walk_kernel(
    Geom g, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Kp, const uint16_t *__restrict__ Vt,
    const int32_t *__restrict__ csize, const uint32_t *__restrict__ sel_mask, const int *__restrict__ mode_flag,
    int my_mode, int kv_modes, uint16_t *__restrict__ O, float *__restrict__ lse)
{
    if (mode_flag != nullptr && mode_flag[FLAG_MODE] != my_mode) return;
    using C = Walk<D>;
    constexpr int NS = C::NS, MMAX = C::MMAX, THREADS = C::THREADS, WAVES = C::WAVES, NST = C::NST;
    constexpr int KSTEPS = D / 32, DT = D / 16;
    constexpr int PF = C::PF;
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
    int *rowid = reinterpret_cast<int *>(smem + C::OFF_ROWID);
    int *rrank = reinterpret_cast<int *>(smem + C::OFF_RANK);
    int *misc = reinterpret_cast<int *>(smem + C::OFF_MISC);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    const bool set_y = __builtin_amdgcn_readfirstlane(wave >> 2) != 0;

    // workgroup -> (query cube, KV head, row block), the blocks of one (cube, head) on the same XCD
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
    if (kv_modes && mode_flag[FLAG_KV + kv] == 3) return;  // the key-stationary kernel has this head's rows
    const int i = g.N - 1 - grp / g.Hkv;
    const CubeBox qbox = cube_box(g, i);
    const int qsize = qbox.size();
    const int P = g.G * qsize;
    const int nblk = (P + MMAX - 1) / MMAX;
    if (blk >= nblk) return;
    const int row0 = (int)((long long)blk * P / nblk), row1 = (int)((long long)(blk + 1) * P / nblk);
    const int Mrows = row1 - row0;
    // Rows of a (cube, KV head) are numbered head by head (row = head-in-group * tokens + rank): a workgroup's rows
    // are neighbouring tokens of one query head (of two, where a head has fewer rows than the workgroup), the rows
    // most likely to select the same cubes.
    const int max_rank = (row0 / qsize == (row1 - 1) / qsize) ? (row1 - 1) % qsize : qsize - 1;
    // (non-causal mode: the whole own cube, and the walk goes on over the cubes after it)
    const int own_tiles = g.causal ? min((qsize + KEY_TILE - 1) / KEY_TILE, max_rank / KEY_TILE + 1)
                                   : (qsize + KEY_TILE - 1) / KEY_TILE;

    for (int r = tid; r < Mrows; r += THREADS) {
        const int rho = row0 + r, hg = rho / qsize, rank = rho - hg * qsize;
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
    const int ncubes = g.causal ? i + 1 : g.N;
    auto tiles_of = [&](int j) -> int {
        if (j == i) return own_tiles;
        return g.ragged ? (csize[j] + KEY_TILE - 1) / KEY_TILE : g.TPC;
    };
    // Sparse entry: a cube that no row of the workgroup selected is left out of the stream altogether.  Rows that
    // select independently of each other leave no such cube; rows of neighbouring tokens with similar queries do.
    constexpr bool listed = MASKED;  // (the entry points admit at most LIST_MAX cubes)
    const uint16_t *clist = reinterpret_cast<const uint16_t *>(smem + C::OFF_LIST);
    int nlist = ncubes;
    if (listed) {
        uint32_t *uni = reinterpret_cast<uint32_t *>(smem + C::OFF_UNION);
        uint16_t *wlist = reinterpret_cast<uint16_t *>(smem + C::OFF_LIST);
        const int wlim = (ncubes + 31) >> 5;  // mask words that hold cubes of the stream
        for (int w = tid; w < wlim; w += THREADS) uni[w] = 0u;
        __syncthreads();
        for (int x = tid; x < Mrows * wlim; x += THREADS) {
            const int r = x / wlim, w = x - r * wlim;
            const uint32_t m = sel_mask[(size_t)rowid[r] * g.words + w];
            if (m) atomicOr(&uni[w], m);
        }
        __syncthreads();
        if (wave == 0) {  // set bits in cube order; the own cube is always there
            int n = 0;
            for (int c0 = 0; c0 < ncubes; c0 += 64) {
                const int c = c0 + lane;
                const bool in = c < ncubes && (c == i || ((uni[c >> 5] >> (c & 31)) & 1u));
                const unsigned long long b = __ballot(in);
                if (in) wlist[n + __popcll(b & ((1ull << lane) - 1ull))] = (uint16_t)c;
                n += __popcll(b);
            }
            if (lane == 0) misc[1] = n;
        }
        __syncthreads();
        nlist = __builtin_amdgcn_readfirstlane(misc[1]);
    }
    auto cube_at = [&](int k) -> int { return listed ? (int)__builtin_amdgcn_readfirstlane((int)clist[k]) : k; };
    // The list entry after position k, fetched when position k is entered and used a whole cube later: the LDS
    // read is long over by then (read and used at the same cube boundary, its latency showed in every stream).
    auto peek_after = [&](int k) -> int {
        const int kk = min(k + 1, nlist - 1);  // past the end the entry only has to be a valid cube
        return listed ? (int)clist[kk] : kk;
    };
    {
        int part = 0;
        for (int k = tid; k < nlist; k += THREADS) part += tiles_of(listed ? (int)clist[k] : k);
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
    int cc_next = peek_after(0);  // for the position that `advance` moves (there is one: the softmax's)
    auto advance = [&](TilePos &p) __attribute__((always_inline)) {
        if (p.t + 1 < p.nt) ++p.t;
        else if (p.k + 1 < nlist) {
            p.j = __builtin_amdgcn_readfirstlane(cc_next);
            cc_next = peek_after(++p.k);
            p.t = 0;
            p.nt = tiles_of(p.j);
        }  // the last tile stays where it is: nothing is issued or computed past the end
    };
    // The K and V^T tiles are fetched in the same order, V^T one tile behind K: one stream walks the list of cubes
    // (cubes are padded to TPC tiles in memory; a ragged cube's padding tiles are skipped) and yields the byte
    // offset of its current tile from the KV head's first tile, which is the same in the K and the V^T half of the
    // packed copy; the V^T load of a slot takes the offset the K load of the slot before it used.  (Two independent
    // streams cost twice the scalar registers and instructions, and this kernel has none to spare: what does not
    // fit is kept in lanes of a vector register and read back with vector instructions.)
    struct Stream {
        uint32_t off;  // of the current tile
        int k, t, nt;  // position in the list of cubes, tile in the cube, tiles of the cube
        int next;      // the cube at position k + 1 (per lane, as read from the list)
    };
    const unsigned char *khead = reinterpret_cast<const unsigned char *>(Kp + (size_t)kv * g.N * g.TPC * (KEY_TILE * D));
    const unsigned char *vhead = reinterpret_cast<const unsigned char *>(Vt + (size_t)kv * g.N * g.TPC * (KEY_TILE * D));
    auto stream_begin = [&]() -> Stream {
        Stream q;
        q.k = 0;
        const int j = cube_at(0);
        q.off = (uint32_t)j * (uint32_t)(g.TPC * C::CHUNK);
        q.t = 0;
        q.nt = tiles_of(j);
        q.next = peek_after(0);
        return q;
    };
    auto stream_next = [&](Stream &q) __attribute__((always_inline)) {
        if (q.t + 1 < q.nt) {
            ++q.t;
            q.off += C::CHUNK;
        } else {
            q.k = min(q.k + 1, nlist - 1);  // past the end nothing is issued; the index only has to stay valid
            const int j = __builtin_amdgcn_readfirstlane(q.next);
            q.next = peek_after(q.k);
            q.off = (uint32_t)j * (uint32_t)(g.TPC * C::CHUNK);
            q.t = 0;
            q.nt = tiles_of(j);
        }
    };
    const uint32_t lds_piece =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + (uint32_t)(wave * C::DMA * 1024));
    const uint32_t src_piece = (uint32_t)(wave * C::DMA * 1024 + lane * 16);
    auto issue = [&](const unsigned char *head, uint32_t off, int off_bytes) __attribute__((always_inline)) {
        const void *tile = uniform_ptr(head + off);
#pragma unroll
        for (int u = 0; u < C::DMA; ++u)
            dma_1k_s(lds_piece + (uint32_t)(off_bytes + u * 1024), tile, src_piece + (uint32_t)(u * 1024));
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
    int rank_lo = 0x7fffffff;  // lowest rank among the wavefront's rows
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (lr[s] != MMAX) rank_lo = min(rank_lo, rrank[lr[s]]);
    for (int off = 32; off > 0; off >>= 1) rank_lo = min(rank_lo, __shfl_xor(rank_lo, off, 64));
    rank_lo = __builtin_amdgcn_readfirstlane(rank_lo == 0x7fffffff ? 0 : rank_lo);

    // prologue: K(0), K(1), V(0)
    Stream sk = stream_begin();
    uint32_t klast = sk.off;  // offset of the K tile issued last
    issue(khead, sk.off, C::OFF_K);  // (ntiles >= 1: the own cube has a tile)
    issue(vhead, sk.off, C::OFF_V);
    stream_next(sk);
    if (ntiles > 1) {
        klast = sk.off;
        issue(khead, sk.off, C::OFF_K + C::CHUNK);
        stream_next(sk);
    }

    const float c2 = 1.44269504088896340736f / sqrtf((float)D);  // softmax scale in base 2, folded into Q
    bf16x8 qf[NS][KSTEPS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const uint16_t *qrow = Q + (size_t)rowid[lr[s]] * D + 8 * q4;
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) qf[s][c] = score_operand(*reinterpret_cast<const bf16x8 *>(qrow + 32 * c), c2);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int c = 0; c < KSTEPS; ++c) asm volatile("" : "+v"(qf[s][c]));

    int lim[NS];
    float m_run[NS];
    bool fresh[NS];
    f32x4 l_run[NS];  // every element holds the row's running sum
    f32x4 oacc[NS][DT];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        m_run[s] = 0.f;   // reference point of the exponentials; set by the row's first tile (fresh)
        fresh[s] = true;
        l_run[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < DT; ++e) oacc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    bool rsel[NS];
    // The rows' mask words: the one in use, and the next one, fetched when the walk enters a word so that it has
    // long arrived when the walk gets there 32 cubes later (read and used at the same cube boundary, every
    // wavefront stood still for a memory latency once per 32 cubes).
    uint32_t mword[NS], mword_ahead[NS];
    int mword_idx = -1;
#pragma unroll
    for (int s = 0; s < NS; ++s) { rsel[s] = true; mword[s] = 0; mword_ahead[s] = 0; }
    if (MASKED) {
#pragma unroll
        for (int s = 0; s < NS; ++s) mword_ahead[s] = sel_mask[(size_t)rowid[lr[s]] * g.words];
    }
    int jsize = 0;
    // per-cube constants of the softmax: key limits of every row, and (MASKED) whether the row attends the cube
    auto enter_cube = [&](int j) __attribute__((always_inline)) {
        const bool own = (j == i);
        jsize = own ? qsize : (g.ragged ? csize[j] : g.Cmax);
#pragma unroll
        for (int s = 0; s < NS; ++s) lim[s] = (own && g.causal) ? min(rrank[lr[s]], jsize - 1) : jsize - 1;
        if (MASKED) {
            if (own) {
#pragma unroll
                for (int s = 0; s < NS; ++s) rsel[s] = true;
            } else {
                if ((j >> 5) != mword_idx) {
                    const bool ahead = (j >> 5) == mword_idx + 1;  // (the walk ascends; words can be skipped)
                    mword_idx = j >> 5;
                    const int nxt = min(mword_idx + 1, g.words - 1);
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        const uint32_t *mr = sel_mask + (size_t)rowid[lr[s]] * g.words;
                        mword[s] = ahead ? mword_ahead[s] : mr[mword_idx];
                        mword_ahead[s] = mr[nxt];
                    }
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
    bool settled = false;  // wave-uniform: no row of the wavefront is fresh any more (softmax_tile_fast may be tried)
    auto softmax_step = [&]() __attribute__((always_inline)) {
        const bool own = (cc.j == i);
        const int key0 = KEY_TILE * cc.t;
        const bool need_mask = (key0 + KEY_TILE > jsize) || (own && g.causal && key0 + KEY_TILE - 1 > rank_lo);
        if (need_mask || !softmax_tile_fast<NS>(sacc, pf, settled)) {
            softmax_tile_folded<D, NS>(sacc, pf, oacc, m_run, l_run, fresh, lim, key0, need_mask, q4);
            bool open = false;
#pragma unroll
            for (int s = 0; s < NS; ++s) open = open || fresh[s];
            settled = __ballot(open) == 0ull;  // every row of the wavefront has a reference point by now
        }
        const int j0 = cc.j;
        advance(cc);
        if (cc.j != j0) enter_cube(cc.j);
    };

    // what the scores of the next tile start from: minus the reference point of the row's exponentials, or -inf
    // for a row that did not select the tile's cube (its probabilities are then 0 and its state stays as it is)
    f32x4 sinit[NS];
    auto set_sinit = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const float x = (MASKED && !rsel[s]) ? -INFINITY : -m_run[s];
            sinit[s] = f32x4{x, x, x, x};
        }
    };
    static_assert(NST == 3, "the stage arithmetic below is for three stages");
    int kst = 0;  // stage of K(t); V(t-1) sits in stage (kst + 2) % 3
    bf16x8 ring[PF];
    // Opens slot t.  The loads started after the previous barrier, K(t+1) and V(t), may stay in flight; everything
    // older has landed: K(t) and V(t-1).  Then K(t+2) and V(t+1) are started into the stages that fell free.
    auto open_slot = [&](int t) __attribute__((always_inline)) {
        if (t > 0 && t + 1 < ntiles) dma_barrier<2 * C::DMA>();
        else dma_barrier<0>();
        const int st_v = kst == 0 ? 2 : kst - 1;  // (kst + 2) % 3: stage of V(t-1), and of K(t+2)
        const int st_n = kst == 2 ? 0 : kst + 1;  // (kst + 1) % 3: stage of V(t+1)
        if (t + 1 < ntiles)  // V^T(t+1): the tile K(t+1), whose offset the K load of the slot before this one used
            issue(vhead, klast, C::OFF_V + st_n * C::CHUNK);
        if (t + 2 < ntiles) {
            klast = sk.off;
            issue(khead, sk.off, C::OFF_K + st_v * C::CHUNK);
            stream_next(sk);
        }
    };
    auto k_tile = [&]() -> const unsigned char * { return smem + C::OFF_K + kst * C::CHUNK; };
    auto v_tile = [&]() -> const unsigned char * { return smem + C::OFF_V + (kst == 0 ? 2 : kst - 1) * C::CHUNK; };
    // The first and the last slot are peeled off the loops: a loop body with a conditional MFMA phase would merge
    // two versions of every accumulator at its end, at the price of a register copy each.
    open_slot(0);
    phase_prefetch<D, PF, false, true>(nullptr, k_tile(), n16, q4, ring);
    set_sinit();
    mfma_phase_from<D, NS, PF, false, true>(nullptr, k_tile(), n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);
    if (!set_y) {
        softmax_step();
        for (int t = 1; t < ntiles; ++t) {
            kst = next_stage(kst);
            open_slot(t);
            phase_prefetch<D, PF, true, true>(v_tile(), k_tile(), n16, q4, ring);
            set_sinit();
            mfma_phase_from<D, NS, PF, true, true>(v_tile(), k_tile(), n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);
            softmax_step();
        }
        kst = next_stage(kst);
        open_slot(ntiles);
        phase_prefetch<D, PF, true, false>(v_tile(), nullptr, n16, q4, ring);
        mfma_phase_from<D, NS, PF, true, false>(v_tile(), nullptr, n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);
    } else {
        for (int t = 1; t < ntiles; ++t) {
            kst = next_stage(kst);
            open_slot(t);
            softmax_step();  // of tile t-1
            phase_prefetch<D, PF, true, true>(v_tile(), k_tile(), n16, q4, ring);
            set_sinit();
            mfma_phase_from<D, NS, PF, true, true>(v_tile(), k_tile(), n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);
        }
        kst = next_stage(kst);
        open_slot(ntiles);
        softmax_step();
        phase_prefetch<D, PF, true, false>(v_tile(), nullptr, n16, q4, ring);
        mfma_phase_from<D, NS, PF, true, false>(v_tile(), nullptr, n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);
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

// ---- the share of candidate cubes the rows select, per KV head, from a sample of rows.  One workgroup; writes
// flags[FLAG_MODE] = 1 (compaction) or 2 (masked walk) from the overall share, flags[FLAG_ESTIMATE] = the smallest
// share of a KV head in permille, and (kv_modes) clears the per-head part.
constexpr int DENSITY_THREADS = 1024;
constexpr int DENSITY_MAX_ROWS = 2048;  // two sampled rows per thread: an estimate is all that is needed
constexpr int DENSITY_GROUPS = 16;          // sampled (cube, query head) pairs for the union estimate
constexpr int DENSITY_UNION_WORDS = ADASPARK_MAX_CUBES / 32;
// Measured on MI355X with rows that select independently of each other: the compacting kernel wins only below
// about 1.5 % selected cubes.
constexpr int MASKED_ABOVE_PERMILLE = 15;

__global__ __launch_bounds__(DENSITY_THREADS) void sel_density_kernel(Geom g, const uint32_t *__restrict__ sel_mask,
                                                                      int *__restrict__ flags, int kv_modes)
{
    __shared__ unsigned long long acc[2][PAIRS_MAX_KV_HEADS];  // selected, candidates; heads beyond the array fold
    for (int x = threadIdx.x; x < 2 * PAIRS_MAX_KV_HEADS; x += DENSITY_THREADS) (&acc[0][0])[x] = 0ull;
    __syncthreads();
    // sample k: token (k * tstride) mod S, query head k mod Hq -- every head gets its share of the samples
    const int samples = (int)min((long long)DENSITY_MAX_ROWS, (long long)g.S * g.Hq);
    const int tstride = max(1, g.S / samples) | 1;
    for (int k = threadIdx.x; k < samples; k += DENSITY_THREADS) {
        const int n = (int)(((long long)k * tstride) % g.S), a = k % g.Hq;
        const int i = cube_of_token(g, n);
        const uint32_t *mr = sel_mask + ((size_t)n * g.Hq + a) * g.words;
        unsigned long long sel = 0;
        for (int w = 0; 32 * w < i; ++w) sel += __popc(mr[w]);
        const int kv = (a / g.G) % PAIRS_MAX_KV_HEADS;
        atomicAdd(&acc[0][kv], sel);
        atomicAdd(&acc[1][kv], (unsigned long long)i);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long sel = 0, cand = 0, least = 1000ull;
        for (int kv = 0; kv < min(g.Hkv, PAIRS_MAX_KV_HEADS); ++kv) {
            sel += acc[0][kv];
            cand += acc[1][kv];
            if (acc[1][kv] > 0ull) least = min(least, acc[0][kv] * 1000ull / acc[1][kv]);
        }
        flags[FLAG_MODE] = (sel * 1000ull > cand * (unsigned long long)MASKED_ABOVE_PERMILLE) ? 2 : 1;
        flags[FLAG_ESTIMATE] = (int)least;
        flags[FLAG_ACTIVE] = 0;
    }
    // What the masked walk cannot leave out: the share of candidate cubes in the union of the selections of one
    // query head's tokens in a cube (a workgroup's rows), over DENSITY_GROUPS sampled (cube, head) pairs, one per
    // wavefront, all at once.
    {
        static_assert(DENSITY_THREADS / 64 == DENSITY_GROUPS, "one sampled (cube, head) pair per wavefront");
        __shared__ uint32_t uni[DENSITY_GROUPS][DENSITY_UNION_WORDS];
        __shared__ unsigned long long ucount[2];  // cubes in the unions, candidate cubes
        if (threadIdx.x < 2) ucount[threadIdx.x] = 0ull;
        const int k = threadIdx.x >> 6, t = threadIdx.x & 63;
        const bool measured = g.causal != 0;
        const int i = g.N - 1 - (int)((long long)k * g.N / DENSITY_GROUPS);  // late cubes weigh most, as in the walk
        const int a = (k * 5 + 1) % g.Hq;
        const int wlim = (i + 31) >> 5;
        if (measured)
            for (int w = t; w < wlim; w += 64) uni[k][w] = 0u;
        __syncthreads();
        if (measured) {
            const CubeBox box = cube_box(g, i);
            const int size = box.size();
            // every second token of the cube: each row read is a cache line of its own, and one CU fetches them all
            for (int r0 = 0; r0 < size; r0 += 512)
                for (int w0 = 0; w0 < wlim; w0 += 8) {  // 4 tokens x 8 words in flight per lane, then combined
                    uint32_t m[4][8];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int r = r0 + 2 * (64 * q + t);
                        const uint32_t *mr =
                            sel_mask + ((size_t)token_of(g, box, min(r, size - 1)) * g.Hq + a) * g.words;
#pragma unroll
                        for (int u = 0; u < 8; ++u) m[q][u] = (r < size && w0 + u < wlim) ? mr[w0 + u] : 0u;
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        uint32_t x = m[0][u] | m[1][u] | m[2][u] | m[3][u];
                        for (int off = 32; off > 0; off >>= 1) x |= __shfl_xor(x, off, 64);
                        if (t == 0 && x) uni[k][w0 + u] |= x;  // the wavefront owns this row of `uni`
                    }
                }
        }
        __syncthreads();
        if (measured) {
            unsigned long long n = 0;
            for (int w = t; w < wlim; w += 64)
                n += __popc(uni[k][w] & (w == (i >> 5) ? (1u << (i & 31)) - 1u : ~0u));
            if (n) atomicAdd(&ucount[0], n);
            if (t == 0) atomicAdd(&ucount[1], (unsigned long long)i);
        }
        __syncthreads();
        if (threadIdx.x == 0)
            flags[FLAG_UNION] = ucount[1] > 0ull ? max(1, (int)(ucount[0] * 1000ull / ucount[1])) : 1000;
    }
    if (kv_modes) {
        unsigned long long *kv_sel =
            reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(flags) + FLAG_BLOCK_BYTES);
        for (int kv = threadIdx.x; kv < g.Hkv; kv += DENSITY_THREADS) {
            flags[FLAG_KV + kv] = 0;
            kv_sel[kv] = 0ull;
        }
    }
}

template <int D, bool MASKED>
static hipError_t launch_walk(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                              const int *mode_flag, int my_mode, int kv_modes, uint16_t *O, float *lse, hipStream_t st)
{
    using C = Walk<D>;
    if (g.N > C::LIST_MAX) return hipErrorInvalidValue;  // the kernel's cube list is that long (the entry points check)
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const uint16_t *Vt = Kp + half_elems;
    const int32_t *csize = reinterpret_cast<const int32_t *>(Vt + half_elems);
    const int nblk_max = (g.G * g.Cmax + C::MMAX - 1) / C::MMAX;
    const dim3 grid((unsigned)((size_t)((g.N * g.Hkv + 7) / 8) * nblk_max * 8));
    static LdsOptIn opted;  // one per kernel instantiation
    const hipError_t e = opted.ensure(reinterpret_cast<const void *>(&attn_walk_kernel<D, MASKED>), C::BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attn_walk_kernel<D, MASKED>), grid, dim3(C::THREADS), C::BYTES, st, g, Q, Kp, Vt, csize,
                       sel_mask, mode_flag, my_mode, kv_modes, O, lse);
    return hipGetLastError();
}

// Below this many candidate (row, cube) pairs the automatic choice is the masked walk outright (see launch_attn_d).
constexpr unsigned long long AUTO_MIN_CANDIDATE_PAIRS = 2ull << 20;

// Measured on MI355X (65,536 tokens, 28/4 heads, head_dim 128, rows selecting independently): the key-stationary
// kernel is the faster one below this share of selected candidate cubes (break-even at 44 %).
constexpr int PAIRS_BELOW_PERMILLE = 400;

template <int D>
static hipError_t launch_attn_d(const Geom &g, const uint16_t *Q, void *packed, const uint32_t *sel_mask,
                                int sparse_kernel, void *scratch, size_t scratch_bytes, uint16_t *O, float *lse,
                                hipStream_t st)
{
    if (sel_mask == nullptr) return launch_walk<D, false>(g, Q, packed, nullptr, nullptr, 0, 0, O, lse, st);
    if (sparse_kernel == ADASPARK_SPARSE_COMPACT && g.causal)
        return launch_attn_compact(g, Q, packed, sel_mask, nullptr, 0, 0, O, lse, st);
    if (sparse_kernel == ADASPARK_SPARSE_MASKED || !g.causal)  // non-causal mode: the masked walk is the one kernel
        return launch_walk<D, true>(g, Q, packed, sel_mask, nullptr, 0, 0, O, lse, st);
    // Small problems (8,192 rows of 64 cubes, say) are bound by the latency from one dependent kernel to the next:
    // the dozen kernels that measure the selection and prepare the other paths would cost more than any choice
    // among them can win back.  The masked walk is the one kernel then.
    if (sparse_kernel == ADASPARK_SPARSE_AUTO && candidate_pairs(g) < AUTO_MIN_CANDIDATE_PAIRS)
        return launch_walk<D, true>(g, Q, packed, sel_mask, nullptr, 0, 0, O, lse, st);
    // Automatic (or the key-stationary kernel asked for): the choice is made on the device, every candidate kernel
    // is enqueued, and the workgroups of those not chosen return at once.  First the selected share from a sample
    // of rows: that decides between the two row-stationary kernels, and whether the exact count for the
    // key-stationary one is worth taking at all; with room for its tables the choice is then made per KV head.
    int *flags = pairs_flags(g, scratch, scratch_bytes);
    const int kv_modes = flags != nullptr;
    if (!kv_modes) {
        if (sparse_kernel == ADASPARK_SPARSE_PAIRS) return hipErrorInvalidValue;  // the entry point checks this first
        flags = reinterpret_cast<int *>(reinterpret_cast<char *>(packed) + attn_workspace_bytes(g) - 16);
    }
    hipLaunchKernelGGL(sel_density_kernel, dim3(1), dim3(DENSITY_THREADS), 0, st, g, sel_mask, flags, kv_modes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (kv_modes) {
        e = launch_attn_pairs(g, Q, packed, sel_mask, scratch, scratch_bytes, sparse_kernel == ADASPARK_SPARSE_PAIRS,
                              PAIRS_BELOW_PERMILLE, O, lse, st);
        if (e != hipSuccess) return e;
    }
    e = launch_attn_compact(g, Q, packed, sel_mask, flags, 1, kv_modes, O, lse, st);
    if (e != hipSuccess) return e;
    return launch_walk<D, true>(g, Q, packed, sel_mask, flags, 2, kv_modes, O, lse, st);
}

hipError_t launch_attn(const Geom &g, const uint16_t *Q, void *packed, const uint32_t *sel_mask, int sparse_kernel,
                       void *scratch, size_t scratch_bytes, uint16_t *O, float *lse, hipStream_t st)
{
    if (g.D == 64) return launch_attn_d<64>(g, Q, packed, sel_mask, sparse_kernel, scratch, scratch_bytes, O, lse, st);
    return launch_attn_d<128>(g, Q, packed, sel_mask, sparse_kernel, scratch, scratch_bytes, O, lse, st);
}

}  // namespace adaspark
