// Relevance scoring + Top-p cube selection (Eqs. 1-2), and the compact cube-index list built from the selection
// bitmask.
//
// The logits of 16 query rows against 16 cubes are one 16x16 tile of K-bar.Q^T.  The fp32 mean keys are split
// into three bf16 terms (hi + mid + lo reproduces the fp32 value to 2^-25), so three bf16 MFMAs accumulate the
// fp32-accurate dot product; Q is bf16 already.  A wavefront holds the logits of its 16-row slabs in MFMA
// accumulators: lane (n16, q4) owns row n16 and cubes 16*cg + 4*q4 + v.  Then, per row:
//   1. softmax numerators e_j = exp2(logit_j*log2(e)/sqrt(D) - max) and their sum Z,
//   2. Top-p without sorting: the kept set is {e_j > tau} plus, in cube order, as many cubes with e_j == tau as
//      are needed, where tau is the largest value with mass{e_j >= tau} >= p*Z.  tau is found bit by bit on the
//      fp32 pattern (positive floats order like unsigned integers).  This equals "sort descending, ties by lower
//      index, keep while the mass before an element is < p",
//   3. the kept flags become mask words.
// A lane works on its own 4*MAXG values and a row's four lanes combine with two lane-swap steps: no
// wavefront-wide reductions, no sort.  All rows of a workgroup belong to one query cube, so they share the number
// of candidate cubes.  Query cubes with up to 256 candidates are handled by cube_select_mfma_kernel (a wavefront
// holds all candidates of its rows), later ones by cube_select_wide_kernel (four or eight wavefronts share the
// rows and split the candidates).
#include <algorithm>

#include "geom.h"

namespace adaspark {

constexpr int SELM_THREADS = 256;
constexpr int SELM_SLABS = 2;                                      // 16-row slabs per wavefront
constexpr int SELM_ROWS = (SELM_THREADS / 64) * SELM_SLABS * 16;  // rows per workgroup
constexpr int SELM_MAX_CUBES = 256;
constexpr int SELM_SWITCH_BIT = 21;  // Top-p threshold search: bits down to this one on all candidates, the rest on a short list
constexpr int SELM_SHORT = 16;       // entries of a lane's short list

typedef __bf16 sel_bf16x8 __attribute__((ext_vector_type(8)));
typedef float sel_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int sel_u32x4 __attribute__((ext_vector_type(4)));

// kbar [N][Hkv][D] fp32 -> ksplit [Hkv][NG][D/32][3][64 lanes][8] bf16: the A operands of
// mfma_f32_16x16x32_bf16 for cube group cg (cubes 16cg..16cg+15), k-step c, term (hi, mid, lo): lane (n16, q4)
// holds cube 16cg + n16, head-dim elements 32c + 8*q4 .. +7.  Cubes beyond N are zero.
__global__ void kbar_split_kernel(Geom g, int NG, const float *__restrict__ kbar, uint16_t *__restrict__ ksplit,
                                  int32_t *__restrict__ status)
{
    // the call's status word starts out as "ok"; the compact list's kernel, which runs later, may change it
    if (blockIdx.x == 0 && threadIdx.x == 0) *status = (int32_t)ADASPARK_OK;
    const int KS = g.D / 32;
    const size_t total = (size_t)g.Hkv * NG * KS * 64;
    for (size_t x = blockIdx.x * (size_t)blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(x % 64);
        const int c = (int)((x / 64) % KS);
        const int cg = (int)((x / (64 * KS)) % NG);
        const int kv = (int)(x / ((size_t)64 * KS * NG));
        const int cube = 16 * cg + (lane & 15), d0 = 32 * c + 8 * (lane >> 4);
        uint16_t t[3][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = cube < g.N ? kbar[((size_t)cube * g.Hkv + kv) * g.D + d0 + e] : 0.f;
            const uint16_t hi = float_to_bf16_bits(v);
            const float r1 = v - bf16_bits_to_float(hi);  // exact
            const uint16_t mid = float_to_bf16_bits(r1);
            const float r2 = r1 - bf16_bits_to_float(mid);  // exact
            t[0][e] = hi;
            t[1][e] = mid;
            t[2][e] = float_to_bf16_bits(r2);
        }
        uint16_t *dst = ksplit + ((((size_t)kv * NG + cg) * KS + c) * 3 * 64 + lane) * 8;
#pragma unroll
        for (int term = 0; term < 3; ++term) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (uint32_t)t[term][2 * e] | ((uint32_t)t[term][2 * e + 1] << 16);
            *reinterpret_cast<uint4 *>(dst + (size_t)term * 64 * 8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// Order-preserving map of a float onto unsigned integers (larger float <=> larger key); never 0 for a number.
__device__ __forceinline__ uint32_t sel_order_key(float x)
{
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Bits of mask word w (cubes 32w .. 32w+31) that fall into the cube range [lo, hi).
__device__ __forceinline__ uint32_t sel_range_bits(int w, int lo, int hi)
{
    const int a = max(lo - 32 * w, 0), b = min(hi - 32 * w, 32);
    if (b <= a) return 0u;
    const uint32_t upto_b = b >= 32 ? 0xffffffffu : ((1u << b) - 1u);
    return upto_b & ~((1u << a) - 1u);
}

// Bits of word w that a row of cube i always has: the text cubes before its own (leading ones are cubes
// [0, Np), trailing ones follow the video cubes), which are attended whatever the rule selects.
__device__ __forceinline__ uint32_t sel_forced_bits(const Geom &g, int w, int i)
{
    if (g.causal) return sel_range_bits(w, 0, min(i, g.Np)) | sel_range_bits(w, g.Np + g.Nv, i);
    // non-causal: every text cube but the own one
    const uint32_t own = (i >> 5) == w ? 1u << (i & 31) : 0u;
    return (sel_range_bits(w, 0, g.Np) | sel_range_bits(w, g.Np + g.Nv, g.N)) & ~own;
}

// The candidates of a row of cube i (Eqs. 1-2): video cubes [Np, cend) -- those before the own cube, or, in
// non-causal mode, all of them but the own one (`skip`, -1 if none) -- and the text cubes it always attends.
struct SelRange {
    int cend, skip, ncand, nforced;
};
__device__ __forceinline__ SelRange sel_range(const Geom &g, int i)
{
    SelRange r;
    const int vend = g.Np + g.Nv;
    if (g.causal) {
        r.cend = min(i, vend);
        r.skip = -1;
        r.ncand = max(r.cend - g.Np, 0);
        r.nforced = i - r.ncand;
    } else {
        const bool own_video = i >= g.Np && i < vend;
        r.cend = vend;
        r.skip = own_video ? i : -1;
        r.ncand = g.Nv - (own_video ? 1 : 0);
        r.nforced = g.N - g.Nv - (own_video ? 0 : 1);
    }
    return r;
}
// bits of word w for "every candidate kept" (all = true) or "none"
__device__ __forceinline__ uint32_t sel_all_candidates(const Geom &g, int w, const SelRange &r, bool all)
{
    if (!all) return 0u;
    const uint32_t own = (r.skip >= 0 && (r.skip >> 5) == w) ? 1u << (r.skip & 31) : 0u;
    return sel_range_bits(w, g.Np, r.cend) & ~own;
}

// OR / sum / max over the four lanes {n, n+16, n+32, n+48} that share a query row
__device__ __forceinline__ uint32_t selm_quad_or(uint32_t x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    const uint32_t y = a[0] | a[1];
    const auto b = __builtin_amdgcn_permlane32_swap(y, y, false, false);
    return b[0] | b[1];
}
__device__ __forceinline__ uint32_t selm_quad_umax(uint32_t x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    const uint32_t y = max(a[0], a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(y, y, false, false);
    return max(b[0], b[1]);
}
__device__ __forceinline__ float selm_quad_sum(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
__device__ __forceinline__ float selm_quad_max(float x)
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// TOPK: fixed Top-K selection (the ablation baseline of "Effect of Top-P Adaptive Selection") instead of Top-p: the
// top_k most relevant preceding cubes, ties by lower index.  The values ranked are then the logits themselves
// (as order-preserving integer keys: no softmax, nothing can underflow) and the "mass" is a count.
template <int D, int MAXG, bool TOPK>
__global__ __launch_bounds__(SELM_THREADS, 2) void cube_select_mfma_kernel(
    Geom g, int NG, int i_end, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ ksplit, float top_p,
    int top_k, uint32_t *__restrict__ sel_mask, int32_t *__restrict__ sel_count)
{
    constexpr int KS = D / 32;
    // the threshold search's short lists (see below): SELM_SHORT entries and a dump slot per lane
    __shared__ uint32_t shortlist[SELM_THREADS / 64][SELM_SHORT + 1][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    // workgroup -> (query cube, KV head, block of rows); late cubes (most candidates) first
    const int nblk_max = (g.G * g.Cmax + SELM_ROWS - 1) / SELM_ROWS;
    const int blk = blockIdx.x % nblk_max;
    const int kv = (blockIdx.x / nblk_max) % g.Hkv;
    const int i = i_end - 1 - blockIdx.x / (nblk_max * g.Hkv);  // this launch covers query cubes [.., i_end)
    const CubeBox qbox = cube_box(g, i);
    const int P = g.G * qbox.size();  // rows of this (cube, KV head): rho = rank * G + head-in-group
    if (blk * SELM_ROWS >= P) return;
    // Candidates are the video cubes before the own cube: cubes [Np, cend).  A query after the video scores every
    // video cube; the text cubes before a row's own are always attended: those bits are set whatever the rule
    // selects.
    const SelRange cr = sel_range(g, i);
    const int cend = cr.cend, ncand = cr.ncand, nforced = cr.nforced;

    int rowg[SELM_SLABS];  // global row id of this lane's column, -1: past the end
    int rowq[SELM_SLABS];  // row whose Q is loaded (a valid one also for padding columns)
#pragma unroll
    for (int s = 0; s < SELM_SLABS; ++s) {
        const int rho = blk * SELM_ROWS + (wave * SELM_SLABS + s) * 16 + n16;
        const int rc = min(rho, P - 1);
        const int rid = token_of(g, qbox, rc / g.G) * g.Hq + kv * g.G + rc % g.G;
        rowg[s] = rho < P ? rid : -1;
        rowq[s] = rid;
    }

    if (ncand == 0 || (TOPK ? (top_k <= 0 || top_k >= ncand) : (top_p <= 0.f || top_p >= 1.f))) {
        // p >= 1 (or k >= number of candidates): every candidate; p = 0 (k = 0): none
        const int keep = (TOPK ? top_k >= ncand : top_p >= 1.f) ? ncand : 0;
#pragma unroll
        for (int s = 0; s < SELM_SLABS; ++s) {
            if (rowg[s] < 0) continue;
            for (int w = q4; w < g.words; w += 4)
                sel_mask[(size_t)rowg[s] * g.words + w] = sel_all_candidates(g, w, cr, keep != 0) | sel_forced_bits(g, w, i);
            if (q4 == 0) sel_count[rowg[s]] = keep + nforced;
        }
        return;
    }

    sel_bf16x8 qf[SELM_SLABS][KS];
#pragma unroll
    for (int s = 0; s < SELM_SLABS; ++s)
#pragma unroll
        for (int c = 0; c < KS; ++c)
            qf[s][c] = *reinterpret_cast<const sel_bf16x8 *>(Q + (size_t)rowq[s] * D + 32 * c + 8 * q4);

    // ---- logits: acc[s][cg][v] = q(row n16 of slab s) . kbar(cube 16cg + 4q4 + v)
    const int ng = (cend + 15) >> 4;  // cube groups up to the last candidate (the same for every row here)
    sel_f32x4 acc[SELM_SLABS][MAXG];
#pragma unroll
    for (int s = 0; s < SELM_SLABS; ++s)
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg) acc[s][cg] = sel_f32x4{0.f, 0.f, 0.f, 0.f};
    // The mean-key operands go from global memory (they stay in L2: a few MB per call) straight into registers,
    // half a cube group ahead of the MFMAs that use them: no staging through LDS, no barriers.
    constexpr int OPS = KS * 3, HALF = OPS / 2, KSH = KS / 2;
    static_assert(KS % 2 == 0, "a cube group's operands are fetched in two halves");
    const sel_bf16x8 *src = reinterpret_cast<const sel_bf16x8 *>(ksplit) + (size_t)kv * NG * (OPS * 64) + lane;
    sel_bf16x8 buf0[HALF], buf1[HALF];
#pragma unroll
    for (int o = 0; o < HALF; ++o) buf0[o] = src[o * 64];  // ng >= 1 here
#pragma unroll
    for (int cg = 0; cg < MAXG; ++cg) {
        if (cg < ng) {  // uniform for the workgroup
#pragma unroll
            for (int o = 0; o < HALF; ++o) buf1[o] = src[((size_t)cg * OPS + HALF + o) * 64];
#pragma unroll
            for (int o = 0; o < HALF; ++o)
#pragma unroll
                for (int s = 0; s < SELM_SLABS; ++s)
                    acc[s][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf0[o], qf[s][o / 3], acc[s][cg], 0, 0, 0);
            if (cg + 1 < ng) {
#pragma unroll
                for (int o = 0; o < HALF; ++o) buf0[o] = src[((size_t)(cg + 1) * OPS + o) * 64];
            }
#pragma unroll
            for (int o = 0; o < HALF; ++o)
#pragma unroll
                for (int s = 0; s < SELM_SLABS; ++s)
                    acc[s][cg] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf1[o], qf[s][KSH + o / 3], acc[s][cg], 0, 0, 0);
        }
    }

    const float scale = 1.44269504088896340736f / sqrtf((float)D);
    const int ng4 = (ng + 3) >> 2;  // groups are processed four at a time below
#pragma unroll
    for (int s = 0; s < SELM_SLABS; ++s) {
        // ---- softmax numerators e = exp2(logit*log2(e)/sqrt(D) - max), 0 for non-candidates; kept in acc
        // (a cube group whose 16 cubes are all candidates -- most are -- needs no test per value: the group-level
        // conditions are the same in every lane and become scalar branches)
        float mx = -INFINITY;
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg) {
            const bool whole = 16 * cg >= g.Np && 16 * cg + 16 <= cend && (cr.skip >> 4) != cg;
            if (whole) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = acc[s][cg][v] * scale;
                    acc[s][cg][v] = x;
                    mx = fmaxf(mx, x);
                }
            } else if (16 * cg < cend) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int cube = 16 * cg + 4 * q4 + v;
                    const bool valid = cube >= g.Np && cube < cend && cube != cr.skip;
                    const float x = valid ? acc[s][cg][v] * scale : -INFINITY;
                    acc[s][cg][v] = x;
                    mx = fmaxf(mx, x);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[s][cg][v] = -INFINITY;
            }
        }
        mx = selm_quad_max(mx);
        float target;
        if (TOPK) {
            // rank the logits themselves: acc holds their order keys (0 for non-candidates)
#pragma unroll
            for (int cg = 0; cg < MAXG; ++cg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = acc[s][cg][v];
                    acc[s][cg][v] = __uint_as_float((x == -INFINITY) ? 0u : sel_order_key(x));
                }
            target = (float)top_k;
        } else {
            float part = 0.f;
#pragma unroll
            for (int cg = 0; cg < MAXG; ++cg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // (non-candidates hold -inf and the maximum is finite -- there is a candidate: exp2 gives 0)
                    const float e = __builtin_amdgcn_exp2f(acc[s][cg][v] - mx);
                    acc[s][cg][v] = e;
                    part += e;
                }
            target = top_p * selm_quad_sum(part);
        }

        // ---- largest tau (as a bit pattern) with mass{e >= tau} >= target: positive floats order like
        // unsigned integers, so tau is found bit by bit; every row (four lanes) runs its own search
        auto mass_at = [&](uint32_t cand) __attribute__((always_inline)) -> float {
            float sum = 0.f;
#pragma unroll
            for (int k4 = 0; k4 < (MAXG + 3) / 4; ++k4)
                if (k4 < ng4) {
#pragma unroll
                    for (int cg = 4 * k4; cg < 4 * k4 + 4 && cg < MAXG; ++cg)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const float e = acc[s][cg][v];
                            sum += (__float_as_uint(e) >= cand) ? (TOPK ? 1.f : e) : 0.f;
                        }
                }
            return selm_quad_sum(sum);
        };
        uint32_t tau = 0;
        int b_first = 31;
        if (!TOPK) {
            // The numerators lie in (0, 1]: bit 30 is never set.  And in all but very flat rows the threshold is
            // above 2^-7 (pattern 0x3C000000: bits 29..26 set): if every row of the slab has its mass there, those
            // four bits are settled in one step -- each of them would have been accepted in turn.
            constexpr uint32_t guess = 0x3C000000u;
            b_first = 29;
            if (__all(mass_at(guess) >= target)) {
                tau = guess;
                b_first = 25;
            }
        }
        bool single = false;  // the search ended early: every row has exactly one element equal to tau
        // After bit b is settled, tau (the smallest kept element) lies in the bucket [tau, tau + 2^b), and of
        // everything else only one number matters: `above`, the mass of the elements beyond the bucket.  On
        // independent rows of a hundred-odd candidates the bucket is down to a twelfth of the row after bit
        // SELM_SWITCH_BIT; the elements in it are then copied out (through LDS: a lane appends its own to a short
        // list of its own) and the remaining bits are settled on those few instead of on all 4 * MAXG registers.
        float above = 0.f;
        int b_next = b_first;
        if (!TOPK) {
            for (; b_next >= SELM_SWITCH_BIT; --b_next) {
                const uint32_t cand = tau | (1u << b_next);
                const float m = mass_at(cand);
                if (m >= target) tau = cand;
                else above = m;
            }
            // ---- the bucket's elements, per lane, into shortlist[..][lane]; slot SELM_SHORT is a dump for the rest
            uint32_t *mine = &shortlist[wave][0][lane];
#pragma unroll
            for (int k = 0; k < SELM_SHORT; ++k) mine[k * 64] = 0u;
            constexpr uint32_t width = 1u << SELM_SWITCH_BIT;
            int cnt = 0;
#pragma unroll
            for (int k4 = 0; k4 < (MAXG + 3) / 4; ++k4)
                if (k4 < ng4) {
#pragma unroll
                    for (int cg = 4 * k4; cg < 4 * k4 + 4 && cg < MAXG; ++cg)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                            const bool inb = bits - tau < width;
                            mine[(inb ? min(cnt, SELM_SHORT) : SELM_SHORT) * 64] = bits;
                            cnt += inb ? 1 : 0;
                        }
                }
            if (!__any(cnt > SELM_SHORT)) {  // (else: the plain search below goes on from where this one stands)
                // the longest list of the wavefront, rounded up to four, bounds the loops over list entries
                const int kmax = __any(cnt > 12) ? 16 : __any(cnt > 8) ? 12 : __any(cnt > 4) ? 8 : 4;
                uint32_t c[SELM_SHORT];
#pragma unroll
                for (int k = 0; k < SELM_SHORT; ++k) c[k] = k < kmax ? mine[k * 64] : 0u;
                for (; b_next >= 0; --b_next) {
                    // the upper half of the bucket: [cand, cand + 2^b)
                    const uint32_t cand = tau | (1u << b_next), half = 1u << b_next;
                    float sum = 0.f;
#pragma unroll
                    for (int k4 = 0; k4 < SELM_SHORT / 4; ++k4)
                        if (4 * k4 < kmax) {
#pragma unroll
                            for (int k = 4 * k4; k < 4 * k4 + 4; ++k)
                                sum += (c[k] - cand < half) ? __uint_as_float(c[k]) : 0.f;
                        }
                    const float m = above + selm_quad_sum(sum);
                    if (m >= target) tau = cand;
                    else above = m;
                    if ((b_next & 1) == 0) {  // one element left in every row's bucket: it is tau
                        int left = 0;
                        uint32_t it = 0u;
#pragma unroll
                        for (int k4 = 0; k4 < SELM_SHORT / 4; ++k4)
                            if (4 * k4 < kmax) {
#pragma unroll
                                for (int k = 4 * k4; k < 4 * k4 + 4; ++k) {
                                    const bool inb = c[k] - tau < half;
                                    left += inb ? 1 : 0;
                                    it = inb ? c[k] : it;
                                }
                            }
                        if (__all((int)selm_quad_sum((float)left) == 1)) {  // small counts: exact in fp32
                            tau = selm_quad_umax(it);
                            single = true;
                            break;
                        }
                    }
                }
                b_next = -1;
            }
        }
        for (int b = b_next; b >= 0; --b) {
            const uint32_t cand = tau | (1u << b);
            if (mass_at(cand) >= target) tau = cand;
            // tau is the value of one of the row's elements, the smallest kept one, and it lies in
            // [tau, tau + 2^b).  Once that bucket holds a single element for every row of the slab the remaining
            // bits are known; looked at every fourth step once the exponent bits are settled.
            if (b <= 22 && (b & 3) == 2) {
                const uint32_t width = 1u << b;
                int cnt = 0;
#pragma unroll
                for (int k4 = 0; k4 < (MAXG + 3) / 4; ++k4)
                    if (k4 < ng4) {
#pragma unroll
                        for (int cg = 4 * k4; cg < 4 * k4 + 4 && cg < MAXG; ++cg)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                cnt += (__float_as_uint(acc[s][cg][v]) - tau < width) ? 1 : 0;
                    }
                if (__all((int)selm_quad_sum((float)cnt) == 1)) {  // small counts: exact in fp32
                    uint32_t it = 0u;  // the one element of the bucket
#pragma unroll
                    for (int k4 = 0; k4 < (MAXG + 3) / 4; ++k4)
                        if (k4 < ng4) {
#pragma unroll
                            for (int cg = 4 * k4; cg < 4 * k4 + 4 && cg < MAXG; ++cg)
#pragma unroll
                                for (int v = 0; v < 4; ++v) {
                                    const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                                    it = (bits - tau < width) ? bits : it;
                                }
                        }
                    tau = selm_quad_umax(it);
                    single = true;
                    break;
                }
            }
        }

        // ---- kept flags.  An element equal to tau is kept while the mass before it (in cube order among the
        // tied ones) is below the target; with a single such element that is always the case.
        uint32_t nib[MAXG];  // bit v of nib[cg]: cube 16cg + 4q4 + v is kept
        if (!TOPK && single) {
            // kept <=> pattern >= tau <=> (tau - 1) - pattern is negative as a signed number (both are below
            // 2^31): its sign bits are shifted into the nibble, no compare masks in scalar registers
            const uint32_t tm1 = tau - 1u;
#pragma unroll
            for (int cg = 0; cg < MAXG; ++cg) {
                uint32_t bitsk = 0u;
#pragma unroll
                for (int v = 3; v >= 0; --v)
                    bitsk = __builtin_amdgcn_alignbit(bitsk, tm1 - __float_as_uint(acc[s][cg][v]), 31);
                nib[cg] = bitsk;
            }
        } else {
        const float tauf = TOPK ? 1.f : __uint_as_float(tau);  // weight of an element equal to tau
        float sgt = 0.f;
        int neq = 0;
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                sgt += bits > tau ? (TOPK ? 1.f : acc[s][cg][v]) : 0.f;
                neq += (bits == tau && tau != 0) ? 1 : 0;
            }
        const float mass_gt = selm_quad_sum(sgt);
        const int neq_row = (int)selm_quad_sum((float)neq);  // small counts: exact in fp32
        if (__any(neq_row > 1)) {
            int running = 0;  // tied elements of this row in earlier cube groups
#pragma unroll
            for (int cg = 0; cg < MAXG; ++cg) {
                int own = 0;
                bool eq[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    eq[v] = __float_as_uint(acc[s][cg][v]) == tau && tau != 0;
                    own += eq[v] ? 1 : 0;
                }
                // counts of the row's four lanes: c0..c3 -> exclusive prefix for this lane, and the total
                const auto a = __builtin_amdgcn_permlane16_swap((uint32_t)own, (uint32_t)own, false, false);
                const uint32_t pair = a[0] + a[1];
                const auto b2 = __builtin_amdgcn_permlane32_swap(pair, pair, false, false);
                const int before = (q4 & 1 ? (int)a[0] : 0) + (q4 & 2 ? (int)b2[0] : 0);
                int t = running + before;
                uint32_t bitsk = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                    bool keep = bits > tau;
                    if (eq[v]) {
                        keep = (t == 0) || (mass_gt + (float)t * tauf < target);
                        ++t;
                    }
                    bitsk |= keep ? (1u << v) : 0u;
                }
                nib[cg] = bitsk;
                running += (int)(b2[0] + b2[1]);
            }
        } else {
#pragma unroll
            for (int cg = 0; cg < MAXG; ++cg) {
                uint32_t bitsk = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                    bitsk |= (bits > tau || (bits == tau && tau != 0)) ? (1u << v) : 0u;
                }
                nib[cg] = bitsk;
            }
        }
        }

        // ---- mask words: word w covers cube groups 2w, 2w+1; a lane's nibble of group cg sits at bit
        // 16*(cg%2) + 4*q4; the four lanes of a row are OR-ed together
        int kept = 0;
#pragma unroll
        for (int w = 0; w < (MAXG + 1) / 2; ++w) {
            uint32_t word = nib[2 * w] << (4 * q4);
            if (2 * w + 1 < MAXG) word |= nib[2 * w + 1] << (16 + 4 * q4);
            word = selm_quad_or(word);
            kept += __popc(word);
            if (w < g.words && rowg[s] >= 0 && q4 == (w & 3))
                sel_mask[(size_t)rowg[s] * g.words + w] = word | sel_forced_bits(g, w, i);
        }
        // words beyond this kernel's cube groups (grids with more cubes): no candidates there for these rows
        if (rowg[s] >= 0)
            for (int w = (MAXG + 1) / 2 + q4; w < g.words; w += 4)
                sel_mask[(size_t)rowg[s] * g.words + w] = sel_forced_bits(g, w, i);
        if (rowg[s] >= 0 && q4 == 0) sel_count[rowg[s]] = kept + nforced;
    }
}

// ---- More than 256 candidate cubes -----------------------------------------------------------------------
//
// The candidates of a row no longer fit one lane quad's registers, so the SPLIT wavefronts of a workgroup share the
// same 32 query rows and each owns a block of 16 cube groups (256 cubes): wavefront p holds the logits of cubes
// 256p .. 256p+255.  Everything per row that spans the blocks -- maximum, sum, the mass above a threshold
// candidate, the tie counts -- is combined through a small LDS exchange, one workgroup barrier per combination;
// every wavefront adds the parts in the same order, so all of them take the same decisions.  The mean-key operands
// go straight from global memory (L2) into registers, one cube group ahead.
constexpr int SELW_MAXG = 16;
constexpr int SELW_SLABS = 2;
constexpr int SELW_ROWS = 16 * SELW_SLABS;

template <int D, int SPLIT, bool TOPK>
__global__ __launch_bounds__(64 * SPLIT, 2) void cube_select_wide_kernel(
    Geom g, int NG, int i_end, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ ksplit, float top_p,
    int top_k, uint32_t *__restrict__ sel_mask, int32_t *__restrict__ sel_count)
{
    constexpr int KS = D / 32, MAXG = SELW_MAXG, SLABS = SELW_SLABS;
    constexpr int OPS = KS * 3;  // A operands (16 bytes per lane each) of one cube group
    constexpr int XK = 3;        // values per row and wavefront in one exchange
    __shared__ __attribute__((aligned(16))) uint32_t xch[2][SLABS][16][SPLIT * XK];
    // the threshold search's short lists (see the kernel above): SELM_SHORT entries and a dump slot per lane; the
    // two slabs of a wavefront fill it in turn
    __shared__ uint32_t shortlist[SPLIT][SELM_SHORT + 1][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int part = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n16 = lane & 15, q4 = lane >> 4;
    const int nblk_max = (g.G * g.Cmax + SELW_ROWS - 1) / SELW_ROWS;
    const int blk = blockIdx.x % nblk_max;
    const int kv = (blockIdx.x / nblk_max) % g.Hkv;
    const int i = i_end - 1 - blockIdx.x / (nblk_max * g.Hkv);  // this launch covers query cubes [.., i_end)
    const CubeBox qbox = cube_box(g, i);
    const int P = g.G * qbox.size();
    if (blk * SELW_ROWS >= P) return;  // the whole workgroup
    // candidates: the video cubes before the own cube, [Np, cend); text cubes before it are forced
    const SelRange cr = sel_range(g, i);
    const int cend = cr.cend, ncand = cr.ncand, nforced = cr.nforced;

    int rowg[SLABS], rowq[SLABS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        const int rho = blk * SELW_ROWS + s * 16 + n16;
        const int rc = min(rho, P - 1);
        const int rid = token_of(g, qbox, rc / g.G) * g.Hq + kv * g.G + rc % g.G;
        rowg[s] = rho < P ? rid : -1;
        rowq[s] = rid;
    }

    if (ncand == 0 || (TOPK ? (top_k <= 0 || top_k >= ncand) : (top_p <= 0.f || top_p >= 1.f))) {
        // the whole workgroup; wavefront 0 writes
        if (part != 0) return;
        const int keep = (TOPK ? top_k >= ncand : top_p >= 1.f) ? ncand : 0;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            if (rowg[s] < 0) continue;
            for (int w = q4; w < g.words; w += 4)
                sel_mask[(size_t)rowg[s] * g.words + w] = sel_all_candidates(g, w, cr, keep != 0) | sel_forced_bits(g, w, i);
            if (q4 == 0) sel_count[rowg[s]] = keep + nforced;
        }
        return;
    }

    sel_bf16x8 qf[SLABS][KS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s)
#pragma unroll
        for (int c = 0; c < KS; ++c)
            qf[s][c] = *reinterpret_cast<const sel_bf16x8 *>(Q + (size_t)rowq[s] * D + 32 * c + 8 * q4);

    // ---- logits of this wavefront's cube block: acc[s][lg][v] = q(row n16 of slab s) . kbar(cube 16(g0+lg)+4q4+v)
    const int ng = (cend + 15) >> 4;  // cube groups up to the last candidate
    const int g0 = part * MAXG;
    const int nlg = min(max(ng - g0, 0), MAXG);  // of them, in this wavefront's block
    sel_f32x4 acc[SLABS][MAXG];
#pragma unroll
    for (int s = 0; s < SLABS; ++s)
#pragma unroll
        for (int lg = 0; lg < MAXG; ++lg) acc[s][lg] = sel_f32x4{0.f, 0.f, 0.f, 0.f};
    const sel_bf16x8 *src =
        reinterpret_cast<const sel_bf16x8 *>(ksplit) + ((size_t)kv * NG + min(g0, NG - 1)) * (OPS * 64) + lane;
    // operands run half a cube group ahead of the MFMAs: two register buffers of OPS/2 operands each
    constexpr int HALF = OPS / 2, KSH = KS / 2;  // a half covers k-steps [KSH*h, KSH*h + KSH), three terms each
    static_assert(KS % 2 == 0, "a cube group's operands are fetched in two halves");
    sel_bf16x8 buf0[HALF], buf1[HALF];
    if (nlg > 0) {
#pragma unroll
        for (int o = 0; o < HALF; ++o) buf0[o] = src[o * 64];
    }
#pragma unroll
    for (int lg = 0; lg < MAXG; ++lg) {
        if (lg < nlg) {  // uniform for the wavefront
#pragma unroll
            for (int o = 0; o < HALF; ++o) buf1[o] = src[((size_t)lg * OPS + HALF + o) * 64];
#pragma unroll
            for (int o = 0; o < HALF; ++o)
#pragma unroll
                for (int s = 0; s < SLABS; ++s)
                    acc[s][lg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf0[o], qf[s][o / 3], acc[s][lg], 0, 0, 0);
            if (lg + 1 < nlg) {
#pragma unroll
                for (int o = 0; o < HALF; ++o) buf0[o] = src[((size_t)(lg + 1) * OPS + o) * 64];
            }
#pragma unroll
            for (int o = 0; o < HALF; ++o)
#pragma unroll
                for (int s = 0; s < SLABS; ++s)
                    acc[s][lg] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf1[o], qf[s][KSH + o / 3], acc[s][lg], 0, 0, 0);
        }
    }

    // ---- exchange: every wavefront contributes XK values per row; afterwards each lane holds those of its row
    // from all wavefronts.  Two buffers in turn: a wavefront that runs ahead writes the other one.
    int xbuf = 0;
    auto exchange = [&](const uint32_t (&v)[XK][SLABS], uint32_t (&all)[SPLIT][XK][SLABS]) __attribute__((always_inline)) {
        if (q4 == 0) {
#pragma unroll
            for (int s = 0; s < SLABS; ++s)
#pragma unroll
                for (int k = 0; k < XK; ++k) xch[xbuf][s][n16][part * XK + k] = v[k][s];
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < SLABS; ++s)
#pragma unroll
            for (int p = 0; p < SPLIT; ++p)
#pragma unroll
                for (int k = 0; k < XK; ++k) all[p][k][s] = xch[xbuf][s][n16][p * XK + k];
        xbuf ^= 1;
    };
    uint32_t xv[XK][SLABS], xa[SPLIT][XK][SLABS];
#pragma unroll
    for (int k = 0; k < XK; ++k)
#pragma unroll
        for (int s = 0; s < SLABS; ++s) xv[k][s] = 0u;

    // ---- softmax numerators e = exp2(logit*log2(e)/sqrt(D) - max), 0 for non-candidates; kept in acc
    const float scale = 1.44269504088896340736f / sqrtf((float)D);
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        float mx = -INFINITY;
#pragma unroll
        for (int lg = 0; lg < MAXG; ++lg) {
            // a cube group whose 16 cubes are all candidates (most are) needs no test per value: the group-level
            // conditions are the same in every lane and become scalar branches
            const int c0 = 16 * (g0 + lg);
            const bool whole = c0 >= g.Np && c0 + 16 <= cend && (cr.skip >> 4) != g0 + lg;
            if (whole) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = acc[s][lg][v] * scale;
                    acc[s][lg][v] = x;
                    mx = fmaxf(mx, x);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int cube = c0 + 4 * q4 + v;
                    const bool valid = cube >= g.Np && cube < cend && cube != cr.skip;
                    const float x = valid ? acc[s][lg][v] * scale : -INFINITY;
                    acc[s][lg][v] = x;
                    mx = fmaxf(mx, x);
                }
            }
        }
        xv[0][s] = __float_as_uint(selm_quad_max(mx));
        xv[1][s] = 0;
    }
    exchange(xv, xa);
    float target[SLABS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        float mx = -INFINITY;
#pragma unroll
        for (int p = 0; p < SPLIT; ++p) mx = fmaxf(mx, __uint_as_float(xa[p][0][s]));
        float sum = 0.f;
#pragma unroll
        for (int lg = 0; lg < MAXG; ++lg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float x = acc[s][lg][v];
                if (TOPK) {  // rank the logits themselves: their order keys, 0 for non-candidates
                    acc[s][lg][v] = __uint_as_float((x == -INFINITY) ? 0u : sel_order_key(x));
                } else {
                    // (non-candidates hold -inf and the row's maximum is finite: exp2 gives 0)
                    const float e = __builtin_amdgcn_exp2f(x - mx);
                    acc[s][lg][v] = e;
                    sum += e;
                }
            }
        xv[0][s] = __float_as_uint(selm_quad_sum(sum));
    }
    exchange(xv, xa);
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        float z = 0.f;
#pragma unroll
        for (int p = 0; p < SPLIT; ++p) z += __uint_as_float(xa[p][0][s]);
        target[s] = TOPK ? (float)top_k : top_p * z;
    }

    // ---- largest tau (as a bit pattern) with mass{e >= tau} >= target, bit by bit, both slabs in step.  Every
    // decision below is taken on exchanged values, which are the same in all wavefronts (they hold the same rows),
    // so all of them follow the same path through the barriers.
    uint32_t tau[SLABS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s) tau[s] = 0;
    // the row's mass at or above cand[s]: one exchange
    auto mass_at = [&](const uint32_t (&cand)[SLABS], float (&mass)[SLABS]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            float sum = 0.f;
#pragma unroll
            for (int lg = 0; lg < MAXG; ++lg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float e = acc[s][lg][v];
                    sum += (__float_as_uint(e) >= cand[s]) ? (TOPK ? 1.f : e) : 0.f;
                }
            xv[0][s] = __float_as_uint(selm_quad_sum(sum));
        }
        exchange(xv, xa);
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            mass[s] = 0.f;
#pragma unroll
            for (int p = 0; p < SPLIT; ++p) mass[s] += __uint_as_float(xa[p][0][s]);
        }
    };
    bool single = false;  // the search ended early: every row has exactly one element equal to tau
    int b_next = TOPK ? 31 : 29;  // (numerators lie in (0, 1]: bit 30 is never set)
    if (!TOPK) {
        // The same search as in the kernel for up to 256 candidates: a first trial that settles bits 29..26 at once,
        // the bits down to SELM_SWITCH_BIT on all candidates while carrying `above`, the mass beyond the bucket
        // [tau, tau + 2^b), and the rest on a short list of the bucket's elements per lane.
        uint32_t cand[SLABS];
        float mass[SLABS], above[SLABS];
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            cand[s] = 0x3C000000u;
            above[s] = 0.f;
        }
        mass_at(cand, mass);
        bool pass = true;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) pass = pass && mass[s] >= target[s];
        if (__all(pass)) {
#pragma unroll
            for (int s = 0; s < SLABS; ++s) tau[s] = cand[s];
            b_next = 25;
        }
        for (; b_next >= SELM_SWITCH_BIT; --b_next) {
#pragma unroll
            for (int s = 0; s < SLABS; ++s) cand[s] = tau[s] | (1u << b_next);
            mass_at(cand, mass);
#pragma unroll
            for (int s = 0; s < SLABS; ++s) {
                if (mass[s] >= target[s]) tau[s] = cand[s];
                else above[s] = mass[s];
            }
        }
        // ---- the bucket's elements of this lane (its share of this wavefront's 256 cubes), slab by slab through
        // the same LDS list into registers
        uint32_t c[SLABS][SELM_SHORT];
        uint32_t *mine = &shortlist[part][0][lane];
        constexpr uint32_t width = 1u << SELM_SWITCH_BIT;
        int cmax = 0;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
#pragma unroll
            for (int k = 0; k < SELM_SHORT; ++k) mine[k * 64] = 0u;
            int cnt = 0;
#pragma unroll
            for (int lg = 0; lg < MAXG; ++lg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t bits = __float_as_uint(acc[s][lg][v]);
                    const bool inb = bits - tau[s] < width;
                    mine[(inb ? min(cnt, SELM_SHORT) : SELM_SHORT) * 64] = bits;
                    cnt += inb ? 1 : 0;
                }
#pragma unroll
            for (int k = 0; k < SELM_SHORT; ++k) c[s][k] = mine[k * 64];
            cmax = max(cmax, cnt);
        }
        // a list that overflowed anywhere in the workgroup: all wavefronts go on with the plain search below
#pragma unroll
        for (int s = 0; s < SLABS; ++s) xv[0][s] = __any(cmax > SELM_SHORT) ? 1u : 0u;
        exchange(xv, xa);
        uint32_t over = 0u;
#pragma unroll
        for (int p = 0; p < SPLIT; ++p) over |= xa[p][0][0];
        if (!over) {
            // the longest list of the wavefront, rounded up to four, bounds the loops over list entries
            const int kmax = __any(cmax > 12) ? 16 : __any(cmax > 8) ? 12 : __any(cmax > 4) ? 8 : 4;
            for (; b_next >= 0; --b_next) {
                // the bucket's upper half [cand, cand + 2^b): its mass and its number of elements; the lower
                // half's number of elements -- whichever half the bucket becomes, its count is known after the
                // one exchange
                const uint32_t half = 1u << b_next;
#pragma unroll
                for (int s = 0; s < SLABS; ++s) {
                    cand[s] = tau[s] | half;
                    float sum = 0.f;
                    int nup = 0, nlo = 0;
#pragma unroll
                    for (int k4 = 0; k4 < SELM_SHORT / 4; ++k4)
                        if (4 * k4 < kmax) {
#pragma unroll
                            for (int k = 4 * k4; k < 4 * k4 + 4; ++k) {
                                const bool up = c[s][k] - cand[s] < half;
                                sum += up ? __uint_as_float(c[s][k]) : 0.f;
                                nup += up ? 1 : 0;
                                nlo += (c[s][k] - tau[s] < half) ? 1 : 0;
                            }
                        }
                    xv[0][s] = __float_as_uint(selm_quad_sum(sum));
                    xv[1][s] = (uint32_t)selm_quad_sum((float)nup);  // small counts: exact in fp32
                    xv[2][s] = (uint32_t)selm_quad_sum((float)nlo);
                }
                exchange(xv, xa);
                bool one = true;
#pragma unroll
                for (int s = 0; s < SLABS; ++s) {
                    float m = above[s];
                    uint32_t nup = 0u, nlo = 0u;
#pragma unroll
                    for (int p = 0; p < SPLIT; ++p) {
                        m += __uint_as_float(xa[p][0][s]);
                        nup += xa[p][1][s];
                        nlo += xa[p][2][s];
                    }
                    const bool take = m >= target[s];
                    if (take) tau[s] = cand[s];
                    else above[s] = m;
                    one = one && (take ? nup : nlo) == 1u;
                }
                if (__all(one)) {  // one element left in every row's bucket: it is tau
#pragma unroll
                    for (int s = 0; s < SLABS; ++s) {
                        uint32_t it = 0u;
#pragma unroll
                        for (int k = 0; k < SELM_SHORT; ++k) it = (c[s][k] - tau[s] < half) ? c[s][k] : it;
                        xv[0][s] = selm_quad_umax(it);
                    }
                    exchange(xv, xa);
#pragma unroll
                    for (int s = 0; s < SLABS; ++s) {
                        uint32_t it = 0u;
#pragma unroll
                        for (int p = 0; p < SPLIT; ++p) it = max(it, xa[p][0][s]);
                        tau[s] = it;
                    }
                    single = true;
                    break;
                }
            }
            b_next = -1;
        }
#pragma unroll
        for (int s = 0; s < SLABS; ++s) xv[1][s] = xv[2][s] = 0u;
    }
    for (int b = b_next; b >= 0; --b) {
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            const uint32_t cand = tau[s] | (1u << b);
            float sum = 0.f;
#pragma unroll
            for (int lg = 0; lg < MAXG; ++lg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float e = acc[s][lg][v];
                    sum += (__float_as_uint(e) >= cand) ? (TOPK ? 1.f : e) : 0.f;
                }
            xv[0][s] = __float_as_uint(selm_quad_sum(sum));
        }
        exchange(xv, xa);
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            float mass = 0.f;
#pragma unroll
            for (int p = 0; p < SPLIT; ++p) mass += __uint_as_float(xa[p][0][s]);
            if (mass >= target[s]) tau[s] |= 1u << b;
        }
        // tau is the value of one of the row's elements and lies in [tau, tau + 2^b): once that bucket holds a
        // single distinct value for every row, the remaining bits are known
        if (b <= 22 && (b & 3) == 2) {
            const uint32_t width = 1u << b;
#pragma unroll
            for (int s = 0; s < SLABS; ++s) {
                uint32_t mn = 0xffffffffu, mxb = 0u;
#pragma unroll
                for (int lg = 0; lg < MAXG; ++lg)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const uint32_t bits = __float_as_uint(acc[s][lg][v]);
                        const bool inb = bits - tau[s] < width;
                        mn = inb ? min(mn, bits) : mn;
                        mxb = inb ? max(mxb, bits) : mxb;
                    }
                xv[0][s] = selm_quad_umax(~mn);  // min via max of the complement
                xv[1][s] = selm_quad_umax(mxb);
            }
            exchange(xv, xa);
            bool one_value = true;
            uint32_t only[SLABS];
#pragma unroll
            for (int s = 0; s < SLABS; ++s) {
                uint32_t nmn = 0u, mxb = 0u;
#pragma unroll
                for (int p = 0; p < SPLIT; ++p) {
                    nmn = max(nmn, xa[p][0][s]);
                    mxb = max(mxb, xa[p][1][s]);
                }
                only[s] = ~nmn;
                one_value = one_value && (only[s] == mxb);
            }
            if (__all(one_value)) {  // the same in every wavefront: they hold the same rows
#pragma unroll
                for (int s = 0; s < SLABS; ++s) tau[s] = only[s];
                break;
            }
        }
    }

    // ---- mass above tau and the number of elements equal to it: in the whole row, and in the blocks before this
    // wavefront's (ties are kept in cube order).  With a single element equal to tau in every row (`single`) none of
    // that is needed: kept <=> pattern >= tau.
    if (!single) {
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        float sgt = 0.f;
        int neq = 0;
#pragma unroll
        for (int lg = 0; lg < MAXG; ++lg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint32_t bits = __float_as_uint(acc[s][lg][v]);
                sgt += bits > tau[s] ? (TOPK ? 1.f : acc[s][lg][v]) : 0.f;
                neq += (bits == tau[s] && tau[s] != 0) ? 1 : 0;
            }
        xv[0][s] = __float_as_uint(selm_quad_sum(sgt));
        xv[1][s] = (uint32_t)selm_quad_sum((float)neq);  // small counts: exact in fp32
    }
    exchange(xv, xa);
    }
    uint32_t kept_part[SLABS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        float mass_gt = 0.f;
        int neq_row = 0, neq_before = 0;
#pragma unroll
        for (int p = 0; p < SPLIT; ++p) {
            mass_gt += __uint_as_float(xa[p][0][s]);
            neq_row += (int)xa[p][1][s];
            neq_before += p < part ? (int)xa[p][1][s] : 0;
        }
        const float tauf = TOPK ? 1.f : __uint_as_float(tau[s]);  // weight of an element equal to tau
        uint32_t nib[MAXG];  // bit v of nib[lg]: cube 16(g0+lg) + 4q4 + v is kept
        if (single) {
            // (tau - 1) - pattern is negative as a signed number exactly when pattern >= tau (both are below 2^31):
            // its sign bits are shifted into the nibble
            const uint32_t tm1 = tau[s] - 1u;
#pragma unroll
            for (int lg = 0; lg < MAXG; ++lg) {
                uint32_t bitsk = 0u;
#pragma unroll
                for (int v = 3; v >= 0; --v)
                    bitsk = __builtin_amdgcn_alignbit(bitsk, tm1 - __float_as_uint(acc[s][lg][v]), 31);
                nib[lg] = bitsk;
            }
        } else if (__any(neq_row > 1)) {
            int running = neq_before;  // tied elements of this row in earlier cube groups
#pragma unroll
            for (int lg = 0; lg < MAXG; ++lg) {
                int own = 0;
                bool eq[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    eq[v] = __float_as_uint(acc[s][lg][v]) == tau[s] && tau[s] != 0;
                    own += eq[v] ? 1 : 0;
                }
                const auto a = __builtin_amdgcn_permlane16_swap((uint32_t)own, (uint32_t)own, false, false);
                const uint32_t pair = a[0] + a[1];
                const auto b2 = __builtin_amdgcn_permlane32_swap(pair, pair, false, false);
                const int before = (q4 & 1 ? (int)a[0] : 0) + (q4 & 2 ? (int)b2[0] : 0);
                int t = running + before;
                uint32_t bitsk = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t bits = __float_as_uint(acc[s][lg][v]);
                    bool keep = bits > tau[s];
                    if (eq[v]) {
                        keep = (t == 0) || (mass_gt + (float)t * tauf < target[s]);
                        ++t;
                    }
                    bitsk |= keep ? (1u << v) : 0u;
                }
                nib[lg] = bitsk;
                running += (int)(b2[0] + b2[1]);
            }
        } else {
#pragma unroll
            for (int lg = 0; lg < MAXG; ++lg) {
                uint32_t bitsk = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t bits = __float_as_uint(acc[s][lg][v]);
                    bitsk |= (bits > tau[s] || (bits == tau[s] && tau[s] != 0)) ? (1u << v) : 0u;
                }
                nib[lg] = bitsk;
            }
        }
        // mask words of this wavefront's block: word 8*part + w covers its cube groups 2w, 2w+1
        int kept = 0;
#pragma unroll
        for (int w = 0; w < MAXG / 2; ++w) {
            uint32_t word = (nib[2 * w] << (4 * q4)) | (nib[2 * w + 1] << (16 + 4 * q4));
            word = selm_quad_or(word);
            kept += __popc(word);
            const int wg = (MAXG / 2) * part + w;
            if (wg < g.words && rowg[s] >= 0 && q4 == (w & 3))
                sel_mask[(size_t)rowg[s] * g.words + wg] = word | sel_forced_bits(g, wg, i);
        }
        kept_part[s] = (uint32_t)kept;
    }
#pragma unroll
    for (int s = 0; s < SLABS; ++s) {
        xv[0][s] = kept_part[s];
        xv[1][s] = 0;
    }
    exchange(xv, xa);
    if (part == 0 && q4 == 0) {
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            int kept = 0;
#pragma unroll
            for (int p = 0; p < SPLIT; ++p) kept += (int)xa[p][0][s];
            if (rowg[s] >= 0) sel_count[rowg[s]] = kept + nforced;
        }
    }
}

// ---- compact list: row_ptr = exclusive scan of sel_count, cube_idx = set bits of each row --------------------

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 4;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

__device__ inline long long block_exclusive_scan(long long x, long long *total, long long *lds)
{
    const int t = threadIdx.x;
    lds[t] = x;
    __syncthreads();
    for (int off = 1; off < SCAN_THREADS; off <<= 1) {
        const long long v = (t >= off) ? lds[t - off] : 0;
        __syncthreads();
        lds[t] += v;
        __syncthreads();
    }
    const long long incl = lds[t];
    *total = lds[SCAN_THREADS - 1];
    __syncthreads();
    return incl - x;
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_tile_sums_kernel(const int32_t *__restrict__ count, long long R,
                                                                      long long *__restrict__ tile_sum)
{
    __shared__ long long lds[SCAN_THREADS];
    const long long base = (long long)blockIdx.x * SCAN_TILE + (long long)threadIdx.x * SCAN_ITEMS;
    long long s = 0;
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < R) s += count[base + k];
    long long total;
    block_exclusive_scan(s, &total, lds);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// One workgroup turns tile sums into exclusive tile offsets, in place.
__global__ __launch_bounds__(SCAN_THREADS) void scan_tile_offsets_kernel(long long *__restrict__ tile_sum, int tiles)
{
    __shared__ long long lds[SCAN_THREADS];
    long long carry = 0;
    for (int base = 0; base < tiles; base += SCAN_THREADS) {
        const int x = base + threadIdx.x;
        const long long v = x < tiles ? tile_sum[x] : 0;
        long long total;
        const long long excl = block_exclusive_scan(v, &total, lds);
        if (x < tiles) tile_sum[x] = carry + excl;
        carry += total;
    }
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_write_kernel(const int32_t *__restrict__ count, long long R,
                                                                  const long long *__restrict__ tile_off,
                                                                  int64_t *__restrict__ row_ptr)
{
    __shared__ long long lds[SCAN_THREADS];
    const long long base = (long long)blockIdx.x * SCAN_TILE + (long long)threadIdx.x * SCAN_ITEMS;
    int c[SCAN_ITEMS];
    long long s = 0;
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        c[k] = (base + k < R) ? count[base + k] : 0;
        s += c[k];
    }
    long long total;
    long long run = tile_off[blockIdx.x] + block_exclusive_scan(s, &total, lds);
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (base + k < R) row_ptr[base + k] = run;
        run += c[k];
        if (base + k == R - 1) row_ptr[R] = run;
    }
}

// status (device): ADASPARK_ECAPACITY if the rows' lists do not fit `capacity` entries (the overflowing entries are
// dropped), else ADASPARK_OK.
__global__ void csr_fill_kernel(Geom g, long long R, const uint32_t *__restrict__ sel_mask,
                                const int64_t *__restrict__ row_ptr, int32_t *__restrict__ cube_idx, long long capacity,
                                int32_t *__restrict__ status)
{
    const long long row = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (row == 0) *status = row_ptr[R] > capacity ? (int32_t)ADASPARK_ECAPACITY : (int32_t)ADASPARK_OK;
    if (row >= R) return;
    long long out = row_ptr[row];
    const uint32_t *mrow = sel_mask + (size_t)row * g.words;
    for (int w = 0; w < g.words; ++w) {
        uint32_t bits = mrow[w];
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            if (out < capacity) cube_idx[out] = 32 * w + b;
            ++out;
        }
    }
}

// The compact list back into mask rows (the form the attention kernels read): row r gets the bits of
// cube_idx[row_ptr[r] .. row_ptr[r+1]).  Entries that name no cube are ignored.
__global__ void mask_from_csr_kernel(Geom g, long long R, const int64_t *__restrict__ row_ptr,
                                     const int32_t *__restrict__ cube_idx, uint32_t *__restrict__ sel_mask)
{
    const long long row = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= R) return;
    uint32_t *mrow = sel_mask + (size_t)row * g.words;
    const long long p0 = row_ptr[row], p1 = row_ptr[row + 1];
    // the list of a row is ascending: one pass, a word at a time
    long long p = p0;
    for (int w = 0; w < g.words; ++w) {
        uint32_t bits = 0u;
        while (p < p1) {
            const int c = cube_idx[p];
            if (c >= 32 * (w + 1)) break;
            if (c >= 32 * w && c < g.N) bits |= 1u << (c & 31);
            ++p;
        }
        mrow[w] = bits;
    }
}

void launch_mask_from_csr(const Geom &g, const int64_t *row_ptr, const int32_t *cube_idx, uint32_t *sel_mask,
                          hipStream_t st)
{
    const long long R = (long long)g.S * g.Hq;
    hipLaunchKernelGGL(mask_from_csr_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, g, R, row_ptr, cube_idx,
                       sel_mask);
}

static int select_groups(const Geom &g) { return (g.N + 15) / 16; }
static size_t select_ksplit_bytes(const Geom &g)
{
    return (((size_t)g.Hkv * select_groups(g) * (g.D / 32) * 3 * 1024) + 255) / 256 * 256;
}
static long long scan_tiles(const Geom &g) { return ((long long)g.S * g.Hq + SCAN_TILE - 1) / SCAN_TILE; }

size_t select_status_offset(const Geom &g)
{
    // the bf16 split of the mean keys, then the scan's tile sums
    const size_t tiles = (size_t)scan_tiles(g) * sizeof(long long);
    return select_ksplit_bytes(g) + ((tiles + 255) / 256) * 256;
}

size_t select_workspace_bytes(const Geom &g)
{
    return select_status_offset(g) + 256;  // and the status word (in a block of its own)
}

template <int D, bool TOPK>
static void launch_select_d(const Geom &g, int NG, const uint16_t *Q, const uint16_t *ksplit, float top_p, int top_k,
                            uint32_t *sel_mask, int32_t *sel_count, hipStream_t st)
{
    // query cubes below SELM_MAX_CUBES have at most that many candidates: one wavefront holds a row's logits
    // (in non-causal mode every query cube has all video cubes as candidates)
    const int i_narrow = g.N <= SELM_MAX_CUBES ? g.N : (g.causal ? SELM_MAX_CUBES : 0);
    if (i_narrow > 0) {
        const int nblk_max = (g.G * g.Cmax + SELM_ROWS - 1) / SELM_ROWS;
        const dim3 grid((unsigned)((size_t)i_narrow * g.Hkv * nblk_max)), block(SELM_THREADS);
        if (i_narrow <= 64)
            hipLaunchKernelGGL((cube_select_mfma_kernel<D, 4, TOPK>), grid, block, 0, st, g, NG, i_narrow, Q, ksplit,
                               top_p, top_k, sel_mask, sel_count);
        else
            hipLaunchKernelGGL((cube_select_mfma_kernel<D, 16, TOPK>), grid, block, 0, st, g, NG, i_narrow, Q, ksplit,
                               top_p, top_k, sel_mask, sel_count);
    }
    if (g.N > i_narrow) {  // the later query cubes: a row's candidates are spread over 4 or 8 wavefronts
        const int nblk_max = (g.G * g.Cmax + SELW_ROWS - 1) / SELW_ROWS;
        const dim3 grid((unsigned)((size_t)(g.N - i_narrow) * g.Hkv * nblk_max));
        if (g.N <= 4 * 16 * SELW_MAXG)
            hipLaunchKernelGGL((cube_select_wide_kernel<D, 4, TOPK>), grid, dim3(256), 0, st, g, NG, g.N, Q, ksplit,
                               top_p, top_k, sel_mask, sel_count);
        else
            hipLaunchKernelGGL((cube_select_wide_kernel<D, 8, TOPK>), grid, dim3(512), 0, st, g, NG, g.N, Q, ksplit,
                               top_p, top_k, sel_mask, sel_count);
    }
}

size_t scan_tile_sum_bytes(long long n) { return (size_t)((n + SCAN_TILE - 1) / SCAN_TILE) * sizeof(long long); }

// out[0..n] = exclusive prefix sums of count[0..n-1] (out[n] = total); tile_sum: scan_tile_sum_bytes(n) of scratch.
void launch_exclusive_scan(const int32_t *count, long long n, long long *tile_sum, int64_t *out, hipStream_t st)
{
    const int tiles = (int)((n + SCAN_TILE - 1) / SCAN_TILE);
    hipLaunchKernelGGL(scan_tile_sums_kernel, dim3(tiles), dim3(SCAN_THREADS), 0, st, count, n, tile_sum);
    hipLaunchKernelGGL(scan_tile_offsets_kernel, dim3(1), dim3(SCAN_THREADS), 0, st, tile_sum, tiles);
    hipLaunchKernelGGL(scan_write_kernel, dim3(tiles), dim3(SCAN_THREADS), 0, st, count, n, tile_sum, out);
}

// top_k < 0: Top-p selection with threshold top_p; top_k >= 0: fixed Top-K selection (top_p ignored).
hipError_t launch_cube_select(const Geom &g, const uint16_t *Q, const float *kbar, float top_p, int top_k,
                              uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                              int64_t capacity, void *ws, hipStream_t st)
{
    static_assert(ADASPARK_MAX_CUBES <= 8 * 16 * SELW_MAXG, "eight wavefronts hold the candidates of a row");
    const long long R = (long long)g.S * g.Hq;
    long long *tile_sum = reinterpret_cast<long long *>(reinterpret_cast<char *>(ws) + select_ksplit_bytes(g));
    uint16_t *ksplit = reinterpret_cast<uint16_t *>(ws);
    const int NG = select_groups(g);
    const size_t total = (size_t)g.Hkv * NG * (g.D / 32) * 64;
    int32_t *status = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(ws) + select_status_offset(g));
    hipLaunchKernelGGL(kbar_split_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, NG, kbar, ksplit,
                       status);
    if (top_k >= 0) {
        if (g.D == 64) launch_select_d<64, true>(g, NG, Q, ksplit, top_p, top_k, sel_mask, sel_count, st);
        else launch_select_d<128, true>(g, NG, Q, ksplit, top_p, top_k, sel_mask, sel_count, st);
    } else {
        if (g.D == 64) launch_select_d<64, false>(g, NG, Q, ksplit, top_p, top_k, sel_mask, sel_count, st);
        else launch_select_d<128, false>(g, NG, Q, ksplit, top_p, top_k, sel_mask, sel_count, st);
    }

    if (row_ptr != nullptr) {
        launch_exclusive_scan(sel_count, R, tile_sum, row_ptr, st);
        hipLaunchKernelGGL(csr_fill_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, g, R, sel_mask, row_ptr,
                           cube_idx, (long long)capacity, status);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// Group-shared selection (a variant: one set per token and KV head, shared by the group's query heads).  The
// group's queries are added in head order in float32, multiplied by float32(1)/float32(G) and rounded to bf16; the
// selection kernels then run on that query with one "query head" per KV head, and the result is copied to the rows
// of all heads of the group.
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void group_mean_query_kernel(Geom g, float inv_g, const uint16_t *__restrict__ Q,
                                                               uint16_t *__restrict__ Qbar)
{
    const int chunks = g.D / 8;
    const size_t total = (size_t)g.S * g.Hkv * chunks;
    for (size_t x = blockIdx.x * (size_t)blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(x % chunks);
        const size_t nk = x / chunks;  // token * Hkv + kv
        const size_t n = nk / g.Hkv, kv = nk % g.Hkv;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (int h = 0; h < g.G; ++h) {
            const sel_u32x4 v = *reinterpret_cast<const sel_u32x4 *>(Q + ((n * g.Hq + kv * g.G + h) * g.D + 8 * c));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] = acc[2 * e] + __uint_as_float(v[e] << 16);
                acc[2 * e + 1] = acc[2 * e + 1] + __uint_as_float(v[e] & 0xffff0000u);
            }
        }
        sel_u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = (uint32_t)float_to_bf16_bits(acc[2 * e] * inv_g) | ((uint32_t)float_to_bf16_bits(acc[2 * e + 1] * inv_g) << 16);
        *reinterpret_cast<sel_u32x4 *>(Qbar + (nk * g.D + 8 * c)) = o;
    }
}

__global__ __launch_bounds__(256) void group_expand_kernel(Geom g, const uint32_t *__restrict__ mask1,
                                                           const int32_t *__restrict__ count1,
                                                           uint32_t *__restrict__ sel_mask, int32_t *__restrict__ sel_count)
{
    const size_t total = (size_t)g.S * g.Hq * g.words;
    for (size_t x = blockIdx.x * (size_t)blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
        const int w = (int)(x % g.words);
        const size_t r = x / g.words;
        const size_t src = (r / g.Hq) * g.Hkv + (r % g.Hq) / g.G;
        sel_mask[x] = mask1[src * g.words + w];
        if (w == 0) sel_count[r] = count1[src];
    }
}

static Geom one_head_per_group(const Geom &g)
{
    Geom o = g;
    o.Hq = g.Hkv;
    o.G = 1;
    return o;
}

size_t select_shared_workspace_bytes(const Geom &g)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t rows1 = (size_t)g.S * g.Hkv;
    return up(select_workspace_bytes(one_head_per_group(g))) + up(rows1 * g.D * 2) + up(rows1 * g.words * 4) + up(rows1 * 4);
}

hipError_t launch_cube_select_shared(const Geom &g, const uint16_t *Q, const float *kbar, float top_p, uint32_t *sel_mask,
                                     int32_t *sel_count, void *ws, hipStream_t st)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const Geom g1 = one_head_per_group(g);
    const size_t rows1 = (size_t)g.S * g.Hkv;
    unsigned char *p = static_cast<unsigned char *>(ws);
    void *ws1 = p;
    p += up(select_workspace_bytes(g1));
    uint16_t *Qbar = reinterpret_cast<uint16_t *>(p);
    p += up(rows1 * g.D * 2);
    uint32_t *mask1 = reinterpret_cast<uint32_t *>(p);
    p += up(rows1 * g.words * 4);
    int32_t *count1 = reinterpret_cast<int32_t *>(p);
    const float inv_g = 1.0f / (float)g.G;
    const size_t n1 = rows1 * (g.D / 8);
    hipLaunchKernelGGL(group_mean_query_kernel, dim3((unsigned)std::min<size_t>((n1 + 255) / 256, 65536)), dim3(256), 0, st,
                       g, inv_g, Q, Qbar);
    hipError_t e = launch_cube_select(g1, Qbar, kbar, top_p, -1, mask1, count1, nullptr, nullptr, 0, ws1, st);
    if (e != hipSuccess) return e;
    const size_t n2 = (size_t)g.S * g.Hq * g.words;
    hipLaunchKernelGGL(group_expand_kernel, dim3((unsigned)std::min<size_t>((n2 + 255) / 256, 65536)), dim3(256), 0, st, g,
                       mask1, count1, sel_mask, sel_count);
    return hipGetLastError();
}

}  // namespace adaspark
