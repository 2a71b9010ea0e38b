// Sparse attention (Eq. 3 + own-cube rule, Sec. 3.2), key-stationary: the work follows the selected
// (query row, key cube) pairs instead of the rows.
//
// The two row-stationary kernels (attn_walk.hip, attn_compact.hip) stream every key cube past every block of
// rows, so with rows that select independently they cost what dense attention costs however little is selected.
// Here the selection is first transposed into one work list per (KV head, key cube): the rows that selected the
// cube.  A workgroup keeps ONE key cube's K and V^T tiles in LDS and its wavefronts run a chunk of that list
// through the tiles, 32 rows at a time, with no workgroup barrier after the load.  What a row gets from one cube
// is a partial result -- unnormalised O, running maximum m, sum l -- written to a record in caller-provided
// scratch memory.  A record holds m, l and s = max |O| in fp32 and O / s in fp16: the merged output is a weighted
// mean of the records' O / l, so a record's rounding error enters it with at most 2^-11 of that record's largest
// element, an eighth of the rounding of the bf16 output itself, at half the memory traffic of fp32 records.  The causal part of every row's own cube is one more record, written by a second launch of the
// same kernel over the rows of each cube.  A last kernel merges each row's records (they are contiguous: a row's
// records are numbered in cube order after an exclusive scan of the per-row counts, the own cube last) into the
// output.
//
// Cost: MFMA work in proportion to the selected pairs, plus 2 * D + 16 bytes written and read per pair and 8
// bytes of work list.  The entry (attn_walk.hip: launch_attn) decides on the device, from the exact pair count and
// per KV head (heads can differ widely in how much they select), whether this path or a row-stationary kernel
// takes the head's rows.
#include <algorithm>

#include "attn_tile.h"

namespace adaspark {

constexpr int PAIRS_MAX_TPC = 4;          // a key cube of up to 256 tokens stays in LDS
constexpr int PAIRS_MAX_SEGMENTS = 8192;  // (KV head, cube) work lists: two LDS histograms of that many counters
constexpr int PAIRS_CHUNK = 3584;         // work-list entries per workgroup (staged in LDS: 28 KB); 14 steps per wavefront
constexpr int PAIRS_HIST_ROWS = 256;      // rows per workgroup in the two transposition passes

template <int D>
struct Pairs {
    static constexpr int WAVES = 8;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int NS = FWD_NS;
    static constexpr int ROWS = 16 * NS;  // rows a wavefront takes per step
    static constexpr int PF = 4;
    static constexpr int CHUNK = KEY_TILE * D * 2;
    static constexpr int PIECES = CHUNK / 1024;  // 1 KB direct-to-LDS copies per tile
    // K and V^T tiles alternate in LDS (K0 V0 K1 V1 ...): both tiles of a step's operand loads then lie within 64 KB
    // of one base register, the reach of the LDS instructions' immediate offset
    static constexpr int OFF_K = 0;
    static constexpr int OFF_V = CHUNK;
    static constexpr int TILE_STRIDE = 2 * CHUNK;
    static constexpr int OFF_ROWS = 2 * PAIRS_MAX_TPC * CHUNK;  // (row id, record) of the workgroup's rows
    static constexpr int BYTES = OFF_ROWS + PAIRS_CHUNK * 8;
    static_assert(BYTES <= 160 * 1024, "LDS of one CU");
    static_assert(PAIRS_CHUNK % (2 * WAVES * ROWS) == 0, "an even number of steps per wavefront");
};

bool pairs_supported(const Geom &g)
{
    return g.TPC <= PAIRS_MAX_TPC && g.Hkv * g.N <= PAIRS_MAX_SEGMENTS && g.Hkv <= PAIRS_MAX_KV_HEADS;
}

// Scratch memory of the pair path, carved from `bytes` bytes at `base` (256-byte aligned):
//   flags      i32 [4 + Hkv]  the kernel-choice flags (geom.h)
//   kv_sel     u64 [Hkv]      selected (row, cube) pairs per KV head
//   qs         fp16 [R][D]    Q times the softmax scale in base 2 (rows of the heads this path takes): the operand of
//                             the score MFMAs, see softmax_tile_folded
//   cnt        i32 [R]        records per row = selected cubes + 1 (the own cube); 0 for rows of heads left to a
//                             row-stationary kernel
//   pair_ptr   i64 [R + 1]    exclusive scan of cnt: a row's records, in cube order, the own cube last
//   tile_sum                  scratch of that scan
//   seg_count  u32 [Hkv * N]  rows that selected cube j, per KV head
//   seg_start  u32 [Hkv * N + 1]
//   seg_cursor u32 [Hkv * N]
//   seg_chunk  u32 [Hkv * N + 1]  exclusive scan of the lists' chunk counts (a chunk: PAIRS_CHUNK entries)
//   entries    u32 [cap][2]   the work lists: (row id, record index), list (kv, j) at seg_start[kv * N + j]
//   ml         f32 [cap][4]   of every record: running maximum m (base-2, scaled), sum l, s = max |O|, unused
//   rec        f16 [cap][D]   O / s, unnormalised partial outputs scaled to [-1, 1]; element (e, q4, v) of the
//                             MFMA output layout (head-dim 16 e + 4 q4 + v) sits at ((e / 2) * 4 + q4) * 8 + (e % 2) * 4 + v
struct PairsScratch {
    int *flags;
    unsigned long long *kv_sel;
    uint16_t *qs;
    int32_t *cnt;
    int64_t *pair_ptr;
    long long *tile_sum;
    uint32_t *seg_count, *seg_start, *seg_cursor, *seg_chunk;
    uint32_t *entries;
    float *ml;
    uint16_t *rec;
    long long cap;  // records that fit; <= 0: not even the tables do
};

static size_t up256(size_t x) { return (x + 255) / 256 * 256; }

static size_t pairs_table_bytes(const Geom &g)
{
    const size_t R = (size_t)g.S * g.Hq, segs = (size_t)g.Hkv * g.N;
    return FLAG_BLOCK_BYTES + 512 + up256(R * (size_t)g.D * 2) + up256(R * 4) + up256((R + 1) * 8) + up256(scan_tile_sum_bytes((long long)R)) +
           4 * up256((segs + 1) * 4);
}

static size_t pairs_record_bytes(const Geom &g, size_t records)
{
    return up256(records * 8) + up256(records * 16) + up256(records * (size_t)g.D * 2);
}

size_t pairs_scratch_bytes(const Geom &g, long long max_selected)
{
    const size_t records = (size_t)max_selected + (size_t)g.S * g.Hq;
    return pairs_table_bytes(g) + pairs_record_bytes(g, records);
}

static PairsScratch pairs_layout(const Geom &g, void *base, size_t bytes)
{
    PairsScratch s{};
    const size_t R = (size_t)g.S * g.Hq, segs = (size_t)g.Hkv * g.N;
    const size_t tables = pairs_table_bytes(g);
    if (base == nullptr || bytes < tables + pairs_record_bytes(g, 1)) {
        s.cap = 0;
        return s;
    }
    static_assert((FLAG_KV + PAIRS_MAX_KV_HEADS) * 4 <= FLAG_BLOCK_BYTES && PAIRS_MAX_KV_HEADS * 8 <= 512,
                  "flag block, head totals");
    char *p = reinterpret_cast<char *>(base);
    s.flags = reinterpret_cast<int *>(p);
    p += FLAG_BLOCK_BYTES;
    s.kv_sel = reinterpret_cast<unsigned long long *>(p);  // right behind the flag block (geom.h)
    p += 512;
    s.qs = reinterpret_cast<uint16_t *>(p);
    p += up256(R * (size_t)g.D * 2);
    s.cnt = reinterpret_cast<int32_t *>(p);
    p += up256(R * 4);
    s.pair_ptr = reinterpret_cast<int64_t *>(p);
    p += up256((R + 1) * 8);
    s.tile_sum = reinterpret_cast<long long *>(p);
    p += up256(scan_tile_sum_bytes((long long)R));
    s.seg_count = reinterpret_cast<uint32_t *>(p);
    p += up256((segs + 1) * 4);
    s.seg_start = reinterpret_cast<uint32_t *>(p);
    p += up256((segs + 1) * 4);
    s.seg_cursor = reinterpret_cast<uint32_t *>(p);
    p += up256((segs + 1) * 4);
    s.seg_chunk = reinterpret_cast<uint32_t *>(p);
    p += up256((segs + 1) * 4);
    const size_t left = bytes - tables;
    size_t cap = left / (24 + (size_t)g.D * 2);
    while (cap > 0 && pairs_record_bytes(g, cap) > left) --cap;  // every array starts on a 256-byte boundary
    if (cap > 0xfffffff0ull) cap = 0xfffffff0ull;                // record indices are 32-bit
    s.entries = reinterpret_cast<uint32_t *>(p);
    p += up256(cap * 8);
    s.ml = reinterpret_cast<float *>(p);
    p += up256(cap * 16);
    s.rec = reinterpret_cast<uint16_t *>(p);
    s.cap = (long long)cap;
    return s;
}

// Bits of a row's mask word w that count: cubes before the row's own cube i (a well-formed mask has no others;
// stray ones are ignored here as the row-stationary kernels ignore them).
__device__ __forceinline__ uint32_t valid_bits(uint32_t word, int w, int i)
{
    const int hi = i - 32 * w;
    if (hi <= 0) return 0u;
    return hi >= 32 ? word : (word & ((1u << hi) - 1u));
}

// The counting kernels are skipped when the sampled estimate of the selected share (flag[1], permille) says that
// this path will not be chosen anyway: well above the threshold, and not forced.
// The break-even share was measured against a masked walk that computes every candidate cube; it computes only the
// share flag[FLAG_UNION] of them (cubes no row of a workgroup selected are left out), and the break-even moves with it.
__device__ __forceinline__ int pairs_threshold(const int *flag, int pairs_below_permille)
{
    // (a tenth of the candidates on top: the walk's fixed costs do not shrink with the union)
    return (int)((long long)pairs_below_permille * min(1000, flag[FLAG_UNION] + 100) / 1000);
}

__device__ __forceinline__ bool pairs_gate_closed(const int *flag, int force, int pairs_below_permille)
{
    const int below = pairs_threshold(flag, pairs_below_permille);
    return !force && flag[FLAG_ESTIMATE] > below + below / 4;
}

__global__ __launch_bounds__(256) void pair_count_kernel(Geom g, long long R, const uint32_t *__restrict__ sel_mask,
                                                         int32_t *__restrict__ cnt, uint32_t *__restrict__ seg_count,
                                                         uint32_t *__restrict__ seg_cursor, int segs,
                                                         unsigned long long *__restrict__ kv_sel,
                                                         const int *__restrict__ flag, int force, int pairs_below_permille)
{
    if (pairs_gate_closed(flag, force, pairs_below_permille)) return;
    __shared__ unsigned int part[PAIRS_MAX_KV_HEADS];
    if (threadIdx.x < PAIRS_MAX_KV_HEADS) part[threadIdx.x] = 0u;
    __syncthreads();
    const long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < segs) {  // cleared here for the passes that follow
        seg_count[r] = 0u;
        seg_cursor[r] = 0u;
    }
    if (r < R) {
        const uint32_t *mr = sel_mask + (size_t)r * g.words;
        const int i = cube_of_token(g, (int)(r / g.Hq));
        int c = 0;
        for (int w = 0; 32 * w < i; ++w) c += __popc(valid_bits(mr[w], w, i));
        cnt[r] = c + 1;  // and the own cube
        atomicAdd(&part[(int)(r % g.Hq) / g.G], (unsigned int)c);
    }
    __syncthreads();
    if (threadIdx.x < g.Hkv && part[threadIdx.x]) atomicAdd(&kv_sel[threadIdx.x], (unsigned long long)part[threadIdx.x]);
}

// Per KV head: the key-stationary kernel takes the head's rows (flags[FLAG_KV + kv] = 3) if its share of selected
// candidate cubes is below the threshold (or force); if the records of the heads so chosen do not fit, none is
// taken.  Then cnt is cleared for the rows of the other heads (run as a second kernel: pair_keep_kernel).
__global__ __launch_bounds__(PAIRS_MAX_KV_HEADS) void pairs_mode_kernel(Geom g, long long cap,
                                                                        unsigned long long candidates_per_head,
                                                                        const unsigned long long *__restrict__ kv_sel,
                                                                        int force, int pairs_below_permille,
                                                                        int *__restrict__ flags)
{
    if (pairs_gate_closed(flags, force, pairs_below_permille)) return;
    __shared__ unsigned long long need[PAIRS_MAX_KV_HEADS];
    const int kv = threadIdx.x;
    bool take = false;
    if (kv < g.Hkv) {
        take = force || kv_sel[kv] * 1000ull < candidates_per_head * (unsigned long long)pairs_threshold(flags, pairs_below_permille);
        need[kv] = take ? kv_sel[kv] + (unsigned long long)g.S * g.G : 0ull;
    }
    __syncthreads();
    unsigned long long total = 0;
    for (int k = 0; k < g.Hkv; ++k) total += need[k];
    const bool fits = total <= (unsigned long long)cap;
    if (kv < g.Hkv) flags[FLAG_KV + kv] = (take && fits) ? 3 : 0;
    if (kv == 0) flags[FLAG_ACTIVE] = (fits && total > 0ull) ? 1 : 0;
}

__global__ void pair_keep_kernel(Geom g, long long R, const int *__restrict__ flags, int32_t *__restrict__ cnt)
{
    if (!flags[FLAG_ACTIVE]) return;
    const long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < R && flags[FLAG_KV + (int)(r % g.Hq) / g.G] != 3) cnt[r] = 0;
}

// qs = fp16(Q * log2(e)/sqrt(D)) for the rows of the heads this path takes (the score operand: attn_tile.h); 8 elements
// per thread.
__global__ void pairs_scale_q_kernel(Geom g, long long chunks, float c2, const int *__restrict__ flags,
                                     const uint16_t *__restrict__ Q, uint16_t *__restrict__ qs)
{
    if (!flags[FLAG_ACTIVE]) return;
    // grid-stride: the grid is bounded, so that a launch that has nothing to do costs little
    for (long long x = (long long)blockIdx.x * blockDim.x + threadIdx.x; x < chunks; x += (long long)gridDim.x * blockDim.x) {
        const long long row = x / (g.D / 8);
        if (flags[FLAG_KV + (int)(row % g.Hq) / g.G] != 3) continue;
        const bf16x8 q = *reinterpret_cast<const bf16x8 *>(Q + x * 8);
        *reinterpret_cast<bf16x8 *>(qs + x * 8) = score_operand(q, c2);
    }
}

// Transposition of the selection, two passes over the set bits of PAIRS_HIST_ROWS rows per workgroup.
// FILL = false: seg_count[kv * N + j] += rows of this block that selected cube j.
// FILL = true: the same count reserves a range of list (kv, j) with one global atomic, and every (row, cube) pair
// is written into it as (row id, record index).
template <bool FILL>
__global__ __launch_bounds__(PAIRS_HIST_ROWS) void pair_transpose_kernel(
    Geom g, long long R, const uint32_t *__restrict__ sel_mask, const int64_t *__restrict__ pair_ptr,
    const int *__restrict__ mode_flag, uint32_t *__restrict__ seg_count, const uint32_t *__restrict__ seg_start, uint32_t *__restrict__ seg_cursor, uint32_t *__restrict__ entries)
{
    if (!mode_flag[FLAG_ACTIVE]) return;
    extern __shared__ uint32_t hist[];  // [segs] counts, then (FILL) [segs] positions handed out
    const int segs = g.Hkv * g.N;
    uint32_t *taken = hist + segs;
    for (int x = threadIdx.x; x < (FILL ? 2 : 1) * segs; x += PAIRS_HIST_ROWS) hist[x] = 0u;
    __syncthreads();
    const long long r = (long long)blockIdx.x * PAIRS_HIST_ROWS + threadIdx.x;
    int i = 0, kvN = 0;
    const uint32_t *mr = nullptr;
    bool mine = false;  // rows of heads left to a row-stationary kernel take no part
    if (r < R) {
        const int kv = (int)((r % g.Hq) / g.G);
        mine = mode_flag[FLAG_KV + kv] == 3;
        i = mine ? cube_of_token(g, (int)(r / g.Hq)) : 0;
        kvN = kv * g.N;
        mr = sel_mask + (size_t)r * g.words;
        for (int w = 0; 32 * w < i; ++w) {
            uint32_t bits = valid_bits(mr[w], w, i);
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                atomicAdd(&hist[kvN + 32 * w + b], 1u);
            }
        }
    }
    __syncthreads();
    if (!FILL) {
        for (int x = threadIdx.x; x < segs; x += PAIRS_HIST_ROWS)
            if (hist[x]) atomicAdd(&seg_count[x], hist[x]);
        return;
    }
    // reserve this block's range in every list it adds to; hist[x] becomes the range's first position
    for (int x = threadIdx.x; x < segs; x += PAIRS_HIST_ROWS)
        if (hist[x]) hist[x] = seg_start[x] + atomicAdd(&seg_cursor[x], hist[x]);
    __syncthreads();
    if (r < R && mine) {
        uint32_t slot = (uint32_t)pair_ptr[r];  // records of a row are numbered in cube order
        for (int w = 0; 32 * w < i; ++w) {
            uint32_t bits = valid_bits(mr[w], w, i);
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                const int x = kvN + 32 * w + b;
                const uint32_t pos = hist[x] + atomicAdd(&taken[x], 1u);
                *reinterpret_cast<uint2 *>(entries + 2 * (size_t)pos) = make_uint2((uint32_t)r, slot);
                ++slot;
            }
        }
    }
}

// One workgroup: seg_start = exclusive scan of seg_count, seg_chunk = exclusive scan of the lists' chunk counts.
constexpr int PLAN_THREADS = 1024;
__global__ __launch_bounds__(PLAN_THREADS) void pairs_plan_kernel(int segs, const uint32_t *__restrict__ seg_count,
                                                                  uint32_t *__restrict__ seg_start,
                                                                  uint32_t *__restrict__ seg_chunk,
                                                                  const int *__restrict__ flags)
{
    if (!flags[FLAG_ACTIVE]) return;
    __shared__ uint32_t part[PLAN_THREADS], cpart[PLAN_THREADS];
    const int t = threadIdx.x;
    const int per = (segs + PLAN_THREADS - 1) / PLAN_THREADS;
    uint32_t s = 0, cs = 0;
    for (int k = 0; k < per; ++k)
        if (t * per + k < segs) {
            s += seg_count[t * per + k];
            cs += (seg_count[t * per + k] + PAIRS_CHUNK - 1) / PAIRS_CHUNK;
        }
    part[t] = s;
    cpart[t] = cs;
    __syncthreads();
    for (int off = 1; off < PLAN_THREADS; off <<= 1) {
        const uint32_t v = t >= off ? part[t - off] : 0u, cv = t >= off ? cpart[t - off] : 0u;
        __syncthreads();
        part[t] += v;
        cpart[t] += cv;
        __syncthreads();
    }
    uint32_t run = part[t] - s, crun = cpart[t] - cs;
    for (int k = 0; k < per; ++k)
        if (t * per + k < segs) {
            seg_start[t * per + k] = run;
            seg_chunk[t * per + k] = crun;
            run += seg_count[t * per + k];
            crun += (seg_count[t * per + k] + PAIRS_CHUNK - 1) / PAIRS_CHUNK;
        }
    if (t == PLAN_THREADS - 1) {
        seg_start[segs] = part[t];
        seg_chunk[segs] = cpart[t];
    }
}

// OWN = false: workgroup b runs chunk b of all lists' chunks: entries [c * PAIRS_CHUNK, ...) of the work list (kv, j)
//              with seg_chunk[kv * N + j] <= b < seg_chunk[kv * N + j + 1], c = b - seg_chunk[kv * N + j].
// OWN = true:  workgroup (kv, j, c) runs rows [c * PAIRS_CHUNK, ...) of cube j itself against it, causally (key rank
//              <= query rank); own_chunks workgroups per cube.
template <int D, bool OWN>
__global__ __launch_bounds__(FWD_MAX_THREADS) void attn_pairs_kernel(
    Geom g, int own_chunks, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Kp,
    const uint16_t *__restrict__ Vt, const int32_t *__restrict__ csize, const int64_t *__restrict__ pair_ptr, const uint32_t *__restrict__ seg_count,
    const uint32_t *__restrict__ seg_start, const uint32_t *__restrict__ seg_chunk,
    const uint32_t *__restrict__ entries, const int *__restrict__ mode_flag, uint16_t *__restrict__ rec,
    float *__restrict__ ml)
{
    if (!mode_flag[FLAG_ACTIVE]) return;
    using C = Pairs<D>;
    constexpr int NS = C::NS, WAVES = C::WAVES, PF = C::PF;
    constexpr int KSTEPS = D / 32, DT = D / 16;
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n16 = lane & 15, q4 = lane >> 4;

    uint2 *rows = reinterpret_cast<uint2 *>(smem + C::OFF_ROWS);
    int seg = (int)(blockIdx.x / own_chunks), c = (int)(blockIdx.x % own_chunks);
    if (!OWN) {
        // the list this chunk belongs to: the last seg with seg_chunk[seg] <= blockIdx.x (scalar binary search)
        const int segs = g.Hkv * g.N;
        const uint32_t b = blockIdx.x;
        if (b >= seg_chunk[segs]) return;
        int lo = 0, hi = segs - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (seg_chunk[mid] <= b) lo = mid;
            else hi = mid - 1;
        }
        seg = lo;
        c = (int)(b - seg_chunk[seg]);
    }
    const int j = seg % g.N, kv = seg / g.N;
    if (OWN && mode_flag[FLAG_KV + kv] != 3) return;  // (the lists of such a head are empty)
    const int jsize = __builtin_amdgcn_readfirstlane(g.ragged ? csize[j] : g.Cmax);
    const CubeBox jbox = cube_box(g, j);  // (OWN) the rows
    // this workgroup's rows: positions [first, first + nrows) of the work list, or all rows of cube j
    uint32_t first = 0;
    int nrows;
    if (OWN) {
        first = (uint32_t)c * PAIRS_CHUNK;
        nrows = min(g.G * jsize - (int)first, PAIRS_CHUNK);
        if (nrows <= 0) return;
    } else {
        const uint32_t count = seg_count[seg];
        first = seg_start[seg] + (uint32_t)c * PAIRS_CHUNK;
        nrows = (int)min(count - (uint32_t)c * PAIRS_CHUNK, (uint32_t)PAIRS_CHUNK);
    }
    nrows = __builtin_amdgcn_readfirstlane(nrows);
    const int nsteps = (nrows + C::ROWS - 1) / C::ROWS;
    const int nt = (jsize + KEY_TILE - 1) / KEY_TILE;  // 1 .. PAIRS_MAX_TPC

    // ---- the key cube's tiles: global -> LDS, all wavefronts
    {
        const size_t cube_off = ((size_t)kv * g.N + j) * g.TPC * C::CHUNK;
        const unsigned char *kbase = reinterpret_cast<const unsigned char *>(Kp) + cube_off;
        const unsigned char *vbase = reinterpret_cast<const unsigned char *>(Vt) + cube_off;
        const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
        const int per = nt * C::PIECES;  // 1 KB pieces of K, and of V^T
        for (int p = wave; p < 2 * per; p += WAVES) {
            const bool isv = p >= per;
            const int q = isv ? p - per : p;  // = tile * PIECES + piece: the tiles of a cube are contiguous in memory
            // wave-uniform by construction; said again so that they are kept in scalar registers
            const uint32_t dst = __builtin_amdgcn_readfirstlane(
                lds0 + (uint32_t)((isv ? C::OFF_V : C::OFF_K) + (q / C::PIECES) * C::TILE_STRIDE + (q % C::PIECES) * 1024));
            const unsigned char *src = reinterpret_cast<const unsigned char *>(isv ? vbase : kbase) + (size_t)q * 1024;
            dma_1k_s(dst, uniform_ptr(src), (uint32_t)(lane * 16));
        }
    }

    // ---- the workgroup's rows as (row id, record) in LDS: a piece of the work list, or (OWN) rows of cube j in
    // (rank, head) order with the own cube's record, which is the row's last
    for (int x = tid; x < nrows; x += C::THREADS) {
        if (OWN) {
            const int idx = (int)first + x;
            const uint32_t rid = (uint32_t)(token_of(g, jbox, idx / g.G) * g.Hq + kv * g.G + idx % g.G);
            rows[x] = make_uint2(rid, (uint32_t)(pair_ptr[rid + 1] - 1));
        } else {
            rows[x] = *reinterpret_cast<const uint2 *>(entries + 2 * (size_t)(first + x));
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tiles (direct-to-LDS loads) and the rows
    __syncthreads();

    // ---- the Q operands run a step ahead of the MFMAs
    struct RowIds {
        uint32_t rid[NS], slot[NS];
        int lim[NS];  // last key (rank in cube j) the row attends
    };
    auto ids_of = [&](int step, RowIds &r) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int idx = min(step * C::ROWS + 16 * s + n16, nrows - 1);  // padding rows repeat the last one
            const uint2 e = rows[idx];
            r.rid[s] = e.x;
            r.slot[s] = e.y;
            r.lim[s] = OWN ? ((int)first + idx) / g.G : jsize - 1;
        }
    };
    auto q_of = [&](const RowIds &r, bf16x8 (&q)[NS][KSTEPS]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const uint16_t *qrow = Q + (size_t)r.rid[s] * D + 8 * q4;
#pragma unroll
            for (int k = 0; k < KSTEPS; ++k) q[s][k] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * k);
        }
    };
    // A step: 32 rows (ids: their row ids and records, q: their Q operands) through the cube's tiles; then the
    // buffers are refilled for step `refill`, two of this wavefront's steps ahead, and the records are written.
    // The loop below alternates between two sets of buffers, so that what is loaded here is read only after the
    // other set's step: no register copies, and the wait for these loads (which, the counter being in order, is
    // also a wait for the older stores) finds everything long done.
    auto run_step = [&](RowIds &ids, bf16x8 (&qf)[NS][KSTEPS], int step, int refill) __attribute__((always_inline)) {
        // (the scores start from minus the reference point of the exponentials: softmax_tile_folded)
        float m_run[NS];
        bool fresh[NS];
        f32x4 l_run[NS], sinit[NS];
        f32x4 oacc[NS][DT];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            m_run[s] = 0.f;
            fresh[s] = true;
            l_run[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < DT; ++e) oacc[s][e] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        f32x4 sacc[NS][4];
        bf16x8 pf[NS][2];
        bf16x8 ring[PF];
        // (OWN) rows come in rank order: no row of the step attends keys past the rank of its last row
        int nts = nt;
        if (OWN) nts = min(nt, ((int)first + min(step * C::ROWS + C::ROWS, nrows) - 1) / g.G / KEY_TILE + 1);
        auto k_tile = [&](int t) -> const unsigned char * { return smem + C::OFF_K + t * C::TILE_STRIDE; };
        auto v_tile = [&](int t) -> const unsigned char * { return smem + C::OFF_V + t * C::TILE_STRIDE; };
        auto softmax_step = [&](int t) __attribute__((always_inline)) {
            const int key0 = KEY_TILE * t;
            const bool need_mask = OWN || (key0 + KEY_TILE > jsize);
            // (after a step's first tile every row has its reference point: fresh is false for all)
            if (need_mask || !softmax_tile_fast<NS>(sacc, pf, t > 0))
                softmax_tile_folded<D, NS>(sacc, pf, oacc, m_run, l_run, fresh, ids.lim, key0, need_mask, q4);
#pragma unroll
            for (int s = 0; s < NS; ++s) sinit[s] = f32x4{-m_run[s], -m_run[s], -m_run[s], -m_run[s]};
        };
#pragma unroll
        for (int s = 0; s < NS; ++s) sinit[s] = f32x4{0.f, 0.f, 0.f, 0.f};
        phase_prefetch<D, PF, false, true>(nullptr, k_tile(0), n16, q4, ring);
        mfma_phase_from<D, NS, PF, false, true>(nullptr, k_tile(0), n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);
        softmax_step(0);
        for (int t = 1; t < nts; ++t) {
            phase_prefetch<D, PF, true, true>(v_tile(t - 1), k_tile(t), n16, q4, ring);
            mfma_phase_from<D, NS, PF, true, true>(v_tile(t - 1), k_tile(t), n16, q4, ring, pf, oacc, l_run, qf, sinit,
                                                   sacc);
            softmax_step(t);
        }
        phase_prefetch<D, PF, true, false>(v_tile(nts - 1), nullptr, n16, q4, ring);
        mfma_phase_from<D, NS, PF, true, false>(v_tile(nts - 1), nullptr, n16, q4, ring, pf, oacc, l_run, qf, sinit, sacc);

        uint32_t slot[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) slot[s] = ids.slot[s];
        ids_of(refill, ids);
        q_of(ids, qf);
        // The records: m, l, s = max |O| and O / s in fp16 (round toward zero).  A lane holds 4 consecutive head-dim
        // elements per block of 16; two blocks make one 16-byte store.  Straight-line code, so that the stores are
        // counted exactly and the wait for the operands loaded above does not become a wait for them: a padding
        // row repeats the step's last row and writes the same record with the same values again.
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            float amax = 0.f;
#pragma unroll
            for (int e = 0; e < DT; ++e)
#pragma unroll
                for (int v = 0; v < 4; ++v) amax = vmax(amax, fabsf(oacc[s][e][v]));
            amax = vmax(quad_max(amax), 1e-30f);
            const float inv = 1.0f / amax;
            uint16_t *orec = rec + (size_t)slot[s] * D + 8 * q4;
#pragma unroll
            for (int e = 0; e < DT; e += 2) {
                typedef __fp16 h2 __attribute__((ext_vector_type(2)));
                union { h2 h[4]; u32x4 u; } pk;
                pk.h[0] = __builtin_amdgcn_cvt_pkrtz(oacc[s][e][0] * inv, oacc[s][e][1] * inv);
                pk.h[1] = __builtin_amdgcn_cvt_pkrtz(oacc[s][e][2] * inv, oacc[s][e][3] * inv);
                pk.h[2] = __builtin_amdgcn_cvt_pkrtz(oacc[s][e + 1][0] * inv, oacc[s][e + 1][1] * inv);
                pk.h[3] = __builtin_amdgcn_cvt_pkrtz(oacc[s][e + 1][2] * inv, oacc[s][e + 1][3] * inv);
                // written once, read once by the merge kernel: streaming stores
                __builtin_nontemporal_store(pk.u, reinterpret_cast<u32x4 *>(orec + 16 * e));
            }
            // the four lanes of a row write one of the four scalars each
            ml[(size_t)slot[s] * 4 + q4] = q4 == 0 ? m_run[s] : q4 == 1 ? l_run[s][0] : q4 == 2 ? amax : 0.f;
        }
    };

    // This wavefront's steps are wave, wave + WAVES, ...; even ones use buffer set A, odd ones set B.  Past the end
    // a step index is clamped to the last step: that step is then done again -- by this wavefront, and possibly by
    // other wavefronts of the workgroup at the same time -- and every such repetition writes the same records.
    // The duplicates are benign because they are bit-identical: a step's result depends only on its rows' Q, the
    // cube's tiles and a fixed instruction sequence (no atomics, no data-dependent order), so concurrent writers
    // store the same bytes to the same addresses.  Everything in the loop stays unconditional (a guarded store
    // would make the compiler merge its wait counts with the operand loads').  The tests that force this kernel
    // run geometries whose step counts are not multiples of the wavefront count, so the repeated step is covered.
    if (wave >= nsteps) return;
    const int last = nsteps - 1;
    RowIds ids_a{}, ids_b{};
    bf16x8 q_a[NS][KSTEPS], q_b[NS][KSTEPS];
    ids_of(wave, ids_a);
    q_of(ids_a, q_a);
    ids_of(min(wave + WAVES, last), ids_b);
    q_of(ids_b, q_b);
    // vmcnt(0), as a builtin so that the compiler's own wait-count bookkeeping knows nothing is pending at the
    // loop's entry (through inline assembly it would not, and would wait at the loop's top, on every trip, for the
    // record stores of the trip before)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    for (int step = wave; step < nsteps; step += 2 * WAVES) {
        run_step(ids_a, q_a, step, min(step + 2 * WAVES, last));
        run_step(ids_b, q_b, min(step + WAVES, last), min(step + 3 * WAVES, last));
    }
}

// D / 4 lanes per row: O = sum_k 2^(m_k - M) s_k h_k / sum_k 2^(m_k - M) l_k over the row's records (h = O / s in
// fp16), in one pass with a running maximum.  A lane owns four adjacent head-dim elements: the four fp16 values at
// byte 8 * lane of a record.
template <int D>
__global__ __launch_bounds__(256) void pairs_merge_kernel(long long R, const int64_t *__restrict__ pair_ptr,
                                                          const uint16_t *__restrict__ rec, const float *__restrict__ ml,
                                                          const int *__restrict__ mode_flag, int Hq, int G,
                                                          uint16_t *__restrict__ O, float *__restrict__ lse)
{
    if (!mode_flag[FLAG_ACTIVE]) return;
    constexpr int LPR = D / 4;  // lanes per row
    typedef __fp16 h4 __attribute__((ext_vector_type(4)));
    const int l = threadIdx.x % LPR;
    // grid-stride over the rows: the grid is bounded, so that a launch that has nothing to do costs little
    for (long long row = (long long)blockIdx.x * (256 / LPR) + threadIdx.x / LPR; row < R;
         row += (long long)gridDim.x * (256 / LPR)) {
    if (mode_flag[FLAG_KV + (int)(row % Hq) / G] != 3) continue;  // another kernel writes that row
    const long long p0 = pair_ptr[row];
    const int n = (int)(pair_ptr[row + 1] - p0);
    const float *mlr = ml + (size_t)p0 * 4;
    const uint16_t *recr = rec + (size_t)p0 * D + 4 * l;
    float M = -INFINITY, L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int U = 8;  // records in flight per lane
    for (int k0 = 0; k0 < n; k0 += U) {
        f32x4 x[U];
        h4 h[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = min(k0 + u, n - 1);  // past the end: the last record again, with weight 0 below
            x[u] = *reinterpret_cast<const f32x4 *>(mlr + (size_t)k * 4);  // m, l, s
            h[u] = *reinterpret_cast<const h4 *>(recr + (size_t)k * D);
        }
        float mx = M;
#pragma unroll
        for (int u = 0; u < U; ++u) mx = fmaxf(mx, x[u][0]);
        const float scale = __builtin_amdgcn_exp2f(M - mx);  // 0 on the first trip (M = -inf)
        M = mx;
        L *= scale;
        acc *= scale;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float w = (k0 + u < n) ? __builtin_amdgcn_exp2f(x[u][0] - M) : 0.f;
            L = fmaf(w, x[u][1], L);
            const float ws = w * x[u][2];
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] = fmaf(ws, (float)h[u][v], acc[v]);
        }
    }
    const float inv = 1.0f / L;
    // position 4 l of a record is element (e, q4, v = 0) with e = 2 * (l / 8) + l % 2, q4 = (l % 8) / 2
    const int d = 16 * (2 * (l / 8) + l % 2) + 4 * ((l % 8) / 2);
    const uint32_t w0 = (uint32_t)float_to_bf16_bits(acc[0] * inv) | ((uint32_t)float_to_bf16_bits(acc[1] * inv) << 16);
    const uint32_t w1 = (uint32_t)float_to_bf16_bits(acc[2] * inv) | ((uint32_t)float_to_bf16_bits(acc[3] * inv) << 16);
    *reinterpret_cast<uint2 *>(O + (size_t)row * D + d) = make_uint2(w0, w1);
    if (lse != nullptr && l == 0) lse[row] = (M + log2f(L)) * 0.69314718055994530942f;
    }
}

// Number of candidate (row, cube) pairs: every row of cube i has i preceding cubes.
unsigned long long candidate_pairs(const Geom &g)
{
    unsigned long long c = 0;
    for (int i = 0; i < g.N; ++i) c += (unsigned long long)i * (unsigned long long)cube_box(g, i).size();
    return c * (unsigned long long)g.Hq;
}

template <int D>
static hipError_t launch_pairs_d(const Geom &g, const uint16_t *Q, const void *packed, const PairsScratch &sc,
                                 const int *flag, uint16_t *O, float *lse, hipStream_t st)
{
    using C = Pairs<D>;
    const uint16_t *Kp = reinterpret_cast<const uint16_t *>(packed);
    const size_t half_elems = (size_t)g.Hkv * g.N * g.TPC * KEY_TILE * D;
    const uint16_t *Vt = Kp + half_elems;
    const int32_t *csize = reinterpret_cast<const int32_t *>(Vt + half_elems);
    const long long R = (long long)g.S * g.Hq;
    static LdsOptIn opted_lists, opted_own;  // one per kernel instantiation
    hipError_t e = opted_lists.ensure(reinterpret_cast<const void *>(&attn_pairs_kernel<D, false>), C::BYTES);
    if (e != hipSuccess) return e;
    e = opted_own.ensure(reinterpret_cast<const void *>(&attn_pairs_kernel<D, true>), C::BYTES);
    if (e != hipSuccess) return e;
    // Chunks of all lists together: at most one partly filled chunk per list, and no more entries than records fit
    // (or than there are candidate pairs).  Workgroups past the actual number of chunks return at once.
    const long long segs = (long long)g.Hkv * g.N;
    const long long most = (long long)std::min<unsigned long long>((unsigned long long)sc.cap, candidate_pairs(g));
    const long long chunks = most / PAIRS_CHUNK + segs;
    const int own_chunks = (g.G * g.Cmax + PAIRS_CHUNK - 1) / PAIRS_CHUNK;
    const long long q_chunks = R * (D / 8);
    hipLaunchKernelGGL(pairs_scale_q_kernel, dim3((unsigned)std::min<long long>((q_chunks + 255) / 256, 256 * 32)), dim3(256), 0, st, g, q_chunks,
                       1.44269504088896340736f / sqrtf((float)D), flag, Q, sc.qs);
    hipLaunchKernelGGL((attn_pairs_kernel<D, false>), dim3((unsigned)chunks), dim3(C::THREADS), C::BYTES, st, g, 1, sc.qs, Kp, Vt,
                       csize, sc.pair_ptr, sc.seg_count, sc.seg_start, sc.seg_chunk, sc.entries, flag, sc.rec, sc.ml);
    hipLaunchKernelGGL((attn_pairs_kernel<D, true>), dim3((unsigned)(segs * own_chunks)), dim3(C::THREADS), C::BYTES, st, g,
                       own_chunks, sc.qs, Kp, Vt, csize, sc.pair_ptr, sc.seg_count, sc.seg_start, sc.seg_chunk, sc.entries, flag, sc.rec, sc.ml);
    const int rows_per_block = 256 / (D / 4);
    const long long merge_blocks = std::min<long long>((R + rows_per_block - 1) / rows_per_block, 256 * 64);
    hipLaunchKernelGGL((pairs_merge_kernel<D>), dim3((unsigned)merge_blocks), dim3(256), 0, st, R, sc.pair_ptr, sc.rec,
                       sc.ml, flag, g.Hq, g.G, O, lse);
    return hipGetLastError();
}

int *pairs_flags(const Geom &g, void *scratch, size_t scratch_bytes)
{
    if (!pairs_supported(g)) return nullptr;
    const PairsScratch sc = pairs_layout(g, scratch, scratch_bytes);
    return sc.cap > 0 ? sc.flags : nullptr;
}

// Counts the pairs per KV head, hands heads to this path (flags), numbers their records, and enqueues this path's
// kernels (they return at once for heads, or altogether, when nothing was handed over).
hipError_t launch_attn_pairs(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask, void *scratch,
                             size_t scratch_bytes, int force, int pairs_below_permille, uint16_t *O, float *lse,
                             hipStream_t st)
{
    const PairsScratch sc = pairs_layout(g, scratch, scratch_bytes);
    if (!pairs_supported(g) || sc.cap <= 0) return hipErrorInvalidValue;
    int *flag = sc.flags;
    const long long R = (long long)g.S * g.Hq;
    const int segs = g.Hkv * g.N;
    const long long count_threads = R > segs ? R : segs;
    const unsigned row_blocks = (unsigned)((R + 255) / 256);
    const unsigned hist_blocks = (unsigned)((R + PAIRS_HIST_ROWS - 1) / PAIRS_HIST_ROWS);
    hipLaunchKernelGGL(pair_count_kernel, dim3((unsigned)((count_threads + 255) / 256)), dim3(256), 0, st, g, R, sel_mask,
                       sc.cnt, sc.seg_count, sc.seg_cursor, segs, sc.kv_sel, flag, force, pairs_below_permille);
    hipLaunchKernelGGL(pairs_mode_kernel, dim3(1), dim3(PAIRS_MAX_KV_HEADS), 0, st, g, sc.cap,
                       candidate_pairs(g) / (unsigned long long)g.Hkv, sc.kv_sel, force, pairs_below_permille, flag);
    hipLaunchKernelGGL(pair_keep_kernel, dim3(row_blocks), dim3(256), 0, st, g, R, flag, sc.cnt);
    launch_exclusive_scan(sc.cnt, R, sc.tile_sum, sc.pair_ptr, st);
    hipLaunchKernelGGL((pair_transpose_kernel<false>), dim3(hist_blocks), dim3(PAIRS_HIST_ROWS), (size_t)segs * 4, st, g,
                       R, sel_mask, sc.pair_ptr, flag, sc.seg_count, sc.seg_start, sc.seg_cursor, sc.entries);
    hipLaunchKernelGGL(pairs_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, st, segs, sc.seg_count, sc.seg_start,
                       sc.seg_chunk, flag);
    hipLaunchKernelGGL((pair_transpose_kernel<true>), dim3(hist_blocks), dim3(PAIRS_HIST_ROWS), (size_t)segs * 8, st, g,
                       R, sel_mask, sc.pair_ptr, flag, sc.seg_count, sc.seg_start, sc.seg_cursor, sc.entries);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return g.D == 64 ? launch_pairs_d<64>(g, Q, packed, sc, flag, O, lse, st)
                     : launch_pairs_d<128>(g, Q, packed, sc, flag, O, lse, st);
}

}  // namespace adaspark
