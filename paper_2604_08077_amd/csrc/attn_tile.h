// Building blocks shared by the two attention kernels (attn_compact.hip, attn_walk.hip): barriers, direct-to-LDS
// tile loads, and the three steps of flash attention on one 64-key tile for 16-row slabs --
//   S^T = K.Q^T, fp32 online softmax (base 2), O^T += V^T.P^T --
// with mfma_f32_16x16x32_bf16: a lane owns one query row (column n16 of the MFMA) and a quarter (q4) of the keys
// of a tile.  K and V^T tiles come from the packed, pre-swizzled copy (kvtile.h).
#pragma once
#include "kvtile.h"

namespace adaspark {

constexpr int FWD_MAX_THREADS = 512;  // workgroup size of both kernels (register budget: 256 per lane)
constexpr int FWD_NS = 2;             // 16-row slabs a wavefront works on at a time

// Tile barrier.  Waits for everything this wavefront has in flight -- its LDS traffic and its direct-to-LDS loads
// of the next tile, started a whole tile ago -- then the workgroup barrier.
__device__ __forceinline__ void tile_barrier()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One wavefront copies 1 KB from global memory straight into LDS: lane l moves the 16 bytes at sbase + voff (sbase:
// wave-uniform, in scalar registers; voff: the lane's own 32-bit byte offset) to lds_addr + 16*l.  lds_addr is
// wave-uniform.  Completion is counted by vmcnt like any vector load.  A stream of tiles advances with two scalar
// adds and no vector arithmetic.
__device__ __forceinline__ void dma_1k_s(uint32_t lds_addr, const void *sbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff),
                 "s"(sbase)
                 : "memory", "m0");
}

// A wave-uniform pointer moved into scalar registers, as dma_1k_s wants its base (readfirstlane returns a signed
// int: each half is widened through uint32_t, or a low half with bit 31 set would smear ones over the high half).
__device__ __forceinline__ const void *uniform_ptr(const void *p)
{
    const uintptr_t u = reinterpret_cast<uintptr_t>(p);
    const uintptr_t r = (uintptr_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)u) |
                        ((uintptr_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(u >> 32)) << 32);
    return reinterpret_cast<const void *>(r);
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

// Score operands are fp16.  The score products S^T = K.Q^T take the packed natural K tile, which kv_pack writes as
// fp16 (K's bf16 values have 8 significant bits and convert exactly while |k| <= 65504, the limit of the format;
// beyond it they saturate there), and Q converted here: times `scale` -- the softmax scale in base 2,
// log2(e)/sqrt(D), in the kernels that fold it in, so that the scores leave the MFMAs in the exponent's units -- and
// rounded to fp16's 11 significant bits (relative 2^-12: an eighth of what a second bf16 rounding would cost every
// product of a score).  The 128-bit operand registers keep the type bf16x8 whatever they hold; score_mfma reads both
// of its operands as fp16.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ f16x8 to_f16(bf16x8 x, float scale)
{
    f16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (_Float16)fminf(fmaxf((float)x[e] * scale, -65504.f), 65504.f);
    return r;
}
__device__ __forceinline__ bf16x8 score_operand(bf16x8 q, float scale) { return __builtin_bit_cast(bf16x8, to_f16(q, scale)); }
__device__ __forceinline__ f32x4 score_mfma(bf16x8 k, bf16x8 q, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, k), __builtin_bit_cast(f16x8, q), c, 0, 0, 0);
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
                sacc[s][kg] = score_mfma(af, qf[s][c], sacc[s][kg]);
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

// Online softmax with the running maximum folded into the MFMA accumulator: the scores arrive as
// s' = (scaled score) - m_run (the S^T MFMAs of a slab start from -m_run, or from -inf for a row that takes no part
// in the tile), so that in the common case -- no score of the tile exceeds the reference m_run by more than
// SOFTMAX_LAZY -- the probabilities are exp2(s') with no arithmetic in between.  m_run is a reference point, not
// the exact maximum: it moves up to a tile's maximum only when that exceeds it by more than SOFTMAX_LAZY (then O
// and l are rescaled), and to the first tile's maximum whatever it is (fresh rows).  Probabilities are at most
// 2^SOFTMAX_LAZY; the final O / l does not depend on the reference.
constexpr float SOFTMAX_LAZY = 1.0f;
// When the reference moves it is put SOFTMAX_HEADROOM above the tile's maximum, so that the scores may rise by
// SOFTMAX_LAZY + SOFTMAX_HEADROOM before it has to move again; probabilities then lie below 2^-SOFTMAX_HEADROOM
// most of the time, which the normalisation cancels.
constexpr float SOFTMAX_HEADROOM = 8.0f;
template <int D, int NS>
__device__ __forceinline__ void softmax_tile_folded(f32x4 (&sacc)[NS][4], bf16x8 (&pf)[NS][2], f32x4 (&oacc)[NS][D / 16],
                                                    float (&m_run)[NS], f32x4 (&l_run)[NS], bool (&fresh)[NS],
                                                    const int (&lim)[NS], int key0, bool need_mask, int q4)
{
    if (need_mask) {
        int kb = key0 + 8 * q4;
        asm volatile("" : "+v"(kb));
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int kg = 0; kg < 4; ++kg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int kr = kb + 32 * (kg >> 1) + 4 * (kg & 1) + v;
                    if (kr > lim[s]) sacc[s][kg][v] = -INFINITY;
                }
    }
    float mx[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(sacc[s][0][0], sacc[s][0][1], sacc[s][0][2]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(mx[s], sacc[s][0][3], sacc[s][1][0]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(mx[s], sacc[s][1][1], sacc[s][1][2]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(mx[s], sacc[s][1][3], sacc[s][2][0]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(mx[s], sacc[s][2][1], sacc[s][2][2]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(mx[s], sacc[s][2][3], sacc[s][3][0]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax3(mx[s], sacc[s][3][1], sacc[s][3][2]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = vmax(mx[s], sacc[s][3][3]);
#pragma unroll
    for (int s = 0; s < NS; ++s) mx[s] = quad_max(mx[s]);
    bool grow[NS];
    unsigned int any = 0u;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        grow[s] = (mx[s] >= SOFTMAX_LAZY) | (fresh[s] & (mx[s] > -INFINITY));
        any |= grow[s] ? 1u : 0u;
    }
    if (__ballot(any != 0u) != 0ull) {  // rare after a row's first tiles: move the reference, rescale O and l
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const float d = grow[s] ? mx[s] + SOFTMAX_HEADROOM : 0.f;
            const float alpha = (grow[s] && !fresh[s]) ? __builtin_amdgcn_exp2f(-d) : 1.f;  // a fresh row has O = l = 0
            m_run[s] += d;
            fresh[s] = fresh[s] && !grow[s];
#pragma unroll
            for (int kg = 0; kg < 4; ++kg)
#pragma unroll
                for (int v = 0; v < 4; ++v) sacc[s][kg][v] -= d;
#pragma unroll
            for (int e = 0; e < D / 16; ++e) oacc[s][e] *= alpha;
            l_run[s] *= alpha;
        }
    }
#pragma unroll
    for (int kg = 0; kg < 4; ++kg)
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int s = 0; s < NS; ++s)
                pf[s][kg >> 1][4 * (kg & 1) + v] = (__bf16)__builtin_amdgcn_exp2f(sacc[s][kg][v]);
}

// The common case of softmax_tile_folded without its row maximum.  The probabilities are taken as exp2(s') straight
// away, rounded to bf16, and only then is the tile checked: a probability of 2 or more -- a score at least
// SOFTMAX_LAZY = 1 above the row's reference -- has the top exponent bit of its bf16 pattern set, and no smaller
// one has, so the OR of the tile's probability words tells whether any row needs its reference moved.  If so
// (rare after a row's first tiles), or if the tile needs masking or some row of the wavefront has no reference yet
// (`settled` false), the function returns false with nothing but pf changed, and the caller runs
// softmax_tile_folded on the untouched scores.  Vector instructions are not hidden behind another wavefront's
// MFMAs on this chip (only the exponentials are), so the maximum's 14 instructions per slab and tile, the lane
// exchanges and the compare are time saved in full.
template <int NS>
__device__ __forceinline__ bool softmax_tile_fast(const f32x4 (&sacc)[NS][4], bf16x8 (&pf)[NS][2], bool settled)
{
    if (!settled) return false;
#pragma unroll
    for (int kg = 0; kg < 4; ++kg)
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int s = 0; s < NS; ++s)
                pf[s][kg >> 1][4 * (kg & 1) + v] = (__bf16)__builtin_amdgcn_exp2f(sacc[s][kg][v]);
    uint32_t big = 0u;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            const u32x4 w = __builtin_bit_cast(u32x4, pf[s][sl]);
            big |= (w[0] | w[1]) | (w[2] | w[3]);
        }
    return __ballot((big & 0x40004000u) != 0u) == 0ull;
}

// The MFMA phase of a wavefront in the counter-phase kernel: P.V of one tile, then S of the next, as one stream
// of operand loads and MFMAs.  A wavefront that is alone in its MFMA phase cannot hide LDS latency behind a
// neighbour, so the operands run PF loads ahead of their use through a ring of registers, and the order written
// here is the order executed (nothing is scheduled across a step).  Step r < RV: V^T operand (sl, e), O^T of every
// slab; step r >= RV: K operand (c, kg), S^T of every slab.  phase_prefetch starts the first PF loads (it may
// run before the barrier that opens the phase when the tiles are known to have landed), mfma_phase does the rest.
template <int D, bool DO_PV, bool DO_QK>
__device__ __forceinline__ bf16x8 phase_operand(const unsigned char *vt, const unsigned char *kt, int n16, int q4, int r)
{
    constexpr int DT = D / 16;
    constexpr int RV = DO_PV ? 2 * DT : 0;
    if (r < RV) {
        const int sl = r / DT, e = r % DT;
        return *reinterpret_cast<const bf16x8 *>(vt + vt_tile_off(16 * e + n16, 4 * sl + q4));
    }
    const int c = (r - RV) / 4, kg = (r - RV) % 4;
    const int krow = 32 * (kg >> 1) + 8 * (n16 >> 2) + 4 * (kg & 1) + (n16 & 3);
    return *reinterpret_cast<const bf16x8 *>(kt + k_tile_off<D>(krow, 4 * c + q4));
}

template <int D, int PF, bool DO_PV, bool DO_QK>
__device__ __forceinline__ void phase_prefetch(const unsigned char *vt, const unsigned char *kt, int n16, int q4,
                                               bf16x8 (&ring)[PF])
{
    constexpr int R = (DO_PV ? 2 * (D / 16) : 0) + (DO_QK ? 4 * (D / 32) : 0);
#pragma unroll
    for (int r = 0; r < PF && r < R; ++r) ring[r] = phase_operand<D, DO_PV, DO_QK>(vt, kt, n16, q4, r);
}

// sinit: what the scores of a slab start from (0, or minus the running maximum: see softmax_tile_folded).
template <int D, int NS, int PF, bool DO_PV, bool DO_QK>
__device__ __forceinline__ void mfma_phase_from(const unsigned char *vt, const unsigned char *kt, int n16, int q4,
                                                bf16x8 (&ring)[PF], const bf16x8 (&pf)[NS][2],
                                                f32x4 (&oacc)[NS][D / 16], f32x4 (&l_run)[NS],
                                                const bf16x8 (&qf)[NS][D / 32], const f32x4 (&sinit)[NS],
                                                f32x4 (&sacc)[NS][4])
{
    constexpr int DT = D / 16, KSTEPS = D / 32;
    constexpr int RV = DO_PV ? 2 * DT : 0, RK = DO_QK ? 4 * KSTEPS : 0, R = RV + RK;
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
                sacc[s][kg] = score_mfma(af, qf[s][c], c == 0 ? sinit[s] : sacc[s][kg]);
        }
        if (r + PF < R) ring[r % PF] = phase_operand<D, DO_PV, DO_QK>(vt, kt, n16, q4, r + PF);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int D, int NS, int PF, bool DO_PV, bool DO_QK>
__device__ __forceinline__ void mfma_phase(const unsigned char *vt, const unsigned char *kt, int n16, int q4,
                                           bf16x8 (&ring)[PF], const bf16x8 (&pf)[NS][2],
                                           f32x4 (&oacc)[NS][D / 16], f32x4 (&l_run)[NS],
                                           const bf16x8 (&qf)[NS][D / 32], f32x4 (&sacc)[NS][4])
{
    f32x4 zero[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) zero[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    mfma_phase_from<D, NS, PF, DO_PV, DO_QK>(vt, kt, n16, q4, ring, pf, oacc, l_run, qf, zero, sacc);
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

}  // namespace adaspark
