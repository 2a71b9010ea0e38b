// Relevance scoring + Top-p cube selection (Eqs. 1-2), and the compact
// cube-index list built from the selection bitmask.
//
// One wavefront per query row (token, query head).  Lane l owns the candidate
// cubes l, l+64, l+128, ...; the row's logits never leave registers.
//   1. logits: q . kbar_j as an fp32 FMA chain over head_dim.  The mean keys are
//      read from a transposed copy [kv_head][d][cube] so the 64 lanes read 64
//      consecutive cubes (coalesced); q[d] is broadcast from the lane that
//      holds it with a scalar lane read.
//   2. softmax numerators e_j = exp2(logit_j*log2(e)/sqrt(D) - max) and their sum Z.
//   3. Top-p without sorting: the kept set is {e_j > tau} plus, in index order,
//      as many cubes with e_j == tau as are needed, where tau is the largest
//      value with mass{e_j >= tau} >= p*Z.  tau is found bit by bit on the fp32
//      pattern (positive floats order like unsigned integers), one wavefront
//      sum per bit.  This equals "sort descending, ties by lower index, keep
//      while the mass before an element is < p".
//   4. the kept flags of each 64-cube chunk are one wave ballot = two mask words.
#include "geom.h"

namespace adaspark {

constexpr int SELECT_THREADS = 256;
constexpr int SELECT_ROWS_PER_BLOCK = SELECT_THREADS / 64;

__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
}

__device__ inline float wave_max(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
}

// kbar [N][Hkv][D] -> kbarT [Hkv][D][Npad], zero in the padding columns.
__global__ void kbar_transpose_kernel(Geom g, int Npad, const float *__restrict__ kbar, float *__restrict__ kbarT)
{
    const size_t total = (size_t)g.Hkv * g.D * Npad;
    for (size_t x = blockIdx.x * (size_t)blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(x % Npad);
        const int d = (int)((x / Npad) % g.D);
        const int kv = (int)(x / ((size_t)Npad * g.D));
        kbarT[x] = j < g.N ? kbar[((size_t)j * g.Hkv + kv) * g.D + d] : 0.f;
    }
}

template <int D, int MAXK>
__global__ __launch_bounds__(SELECT_THREADS) void cube_select_kernel(Geom g, int Npad, const uint16_t *__restrict__ Q,
                                                                     const float *__restrict__ kbarT, float top_p,
                                                                     uint32_t *__restrict__ sel_mask,
                                                                     int32_t *__restrict__ sel_count)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long R = (long long)g.S * g.Hq;
    const long long row = (long long)blockIdx.x * SELECT_ROWS_PER_BLOCK + wave;
    if (row >= R) return;  // whole wavefront leaves together; no barriers below
    const int n = (int)(row / g.Hq), a = (int)(row % g.Hq), kv = a / g.G;
    const int i = cube_of_token(g, n);  // candidates are cubes 0..i-1
    uint32_t *mrow = sel_mask + (size_t)row * g.words;

    if (i == 0 || top_p <= 0.f || top_p >= 1.f) {
        const int keep = (i > 0 && top_p >= 1.f) ? i : 0;  // p>=1: every preceding cube
        for (int w = lane; w < g.words; w += 64) {
            const int lo = 32 * w;
            uint32_t bits = 0;
            if (keep >= lo + 32) bits = 0xffffffffu;
            else if (keep > lo) bits = (1u << (keep - lo)) - 1u;
            mrow[w] = bits;
        }
        if (lane == 0) sel_count[row] = keep;
        return;
    }

    // query row: lane l holds q[l] (and q[l+64] for D = 128)
    const uint16_t *qrow = Q + (size_t)row * D;
    const float q0 = bf16_bits_to_float(qrow[lane]);
    const float q1 = (D > 64) ? bf16_bits_to_float(qrow[64 + lane]) : 0.f;

    const int nch = (i + 63) >> 6;  // 64-cube chunks that hold candidates (wave-uniform)
    const float scale = 1.44269504088896340736f / sqrtf((float)D);
    float e[MAXK];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < MAXK; ++k) {
        e[k] = -INFINITY;
        if (k < nch) {
            const float *col = kbarT + (size_t)kv * D * Npad + 64 * k + lane;
            float acc = 0.f;
#pragma unroll 16
            for (int d = 0; d < 64; ++d)
                acc = fmaf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(q0), d)), col[(size_t)d * Npad], acc);
            if (D > 64) {
#pragma unroll 16
                for (int d = 0; d < 64; ++d)
                    acc = fmaf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(q1), d)),
                               col[(size_t)(64 + d) * Npad], acc);
            }
            if (64 * k + lane < i) {
                e[k] = acc * scale;
                mx = fmaxf(mx, e[k]);
            }
        }
    }
    mx = wave_max(mx);
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < MAXK; ++k) {
        e[k] = (e[k] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(e[k] - mx);
        part += e[k];
    }
    const float Z = wave_sum(part);
    const float target = top_p * Z;

    // largest tau (as a bit pattern) with mass{e >= tau} >= target
    uint32_t tau = 0;
    for (int b = 30; b >= 0; --b) {
        const uint32_t cand = tau | (1u << b);
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < MAXK; ++k) s += (__float_as_uint(e[k]) >= cand) ? e[k] : 0.f;
        if (wave_sum(s) >= target) tau = cand;
    }
    const float tauf = __uint_as_float(tau);
    float sgt = 0.f;
    int n_eq = 0;
#pragma unroll
    for (int k = 0; k < MAXK; ++k) {
        sgt += (__float_as_uint(e[k]) > tau) ? e[k] : 0.f;
        n_eq += __popcll(__ballot(__float_as_uint(e[k]) == tau && tau != 0));
    }
    const float mass_gt = wave_sum(sgt);

    int kept = 0, ties_before = 0;
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int k = 0; k < MAXK; ++k) {
        const uint32_t bits = __float_as_uint(e[k]);
        const bool is_eq = (bits == tau) && tau != 0;
        const unsigned long long eqb = __ballot(is_eq);
        bool keep = bits > tau;
        if (is_eq) {
            // ties are taken in cube-index order while the mass before them is below the target
            const int t = ties_before + __popcll(eqb & lt_mask);
            keep = (t == 0) || (mass_gt + (float)t * tauf < target);
        }
        ties_before += __popcll(eqb);
        const unsigned long long kb = __ballot(keep);
        kept += __popcll(kb);
        if (lane == 0) {
            if (2 * k < g.words) mrow[2 * k] = (uint32_t)kb;
            if (2 * k + 1 < g.words) mrow[2 * k + 1] = (uint32_t)(kb >> 32);
        }
    }
    (void)n_eq;
    if (lane == 0) sel_count[row] = kept;
}

// ---- MFMA path for grids of up to 256 cubes ---------------------------------------------------------------
//
// The logits of 16 query rows against 16 cubes are one 16x16 tile of K-bar.Q^T.  The fp32 mean keys are split
// into three bf16 terms (hi + mid + lo reproduces the fp32 value to 2^-25), so three bf16 MFMAs accumulate the
// fp32-accurate dot product; Q is bf16 already.  A wavefront holds the logits of its 16-row slabs in MFMA
// accumulators: lane (n16, q4) owns row n16 and cubes 16*cg + 4*q4 + v.  Softmax and the Top-p threshold search
// then run per lane over its 4*MAXG values, and a row's four lanes combine with two lane-swap steps: no
// wavefront-wide reductions, no sort.  All rows of a workgroup belong to one query cube, so they share the
// number of candidate cubes.
constexpr int SELM_THREADS = 256;
constexpr int SELM_SLABS = 2;                                      // 16-row slabs per wavefront
constexpr int SELM_ROWS = (SELM_THREADS / 64) * SELM_SLABS * 16;  // rows per workgroup
constexpr int SELM_MAX_CUBES = 256;

typedef __bf16 sel_bf16x8 __attribute__((ext_vector_type(8)));
typedef float sel_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int sel_u32x4 __attribute__((ext_vector_type(4)));

// kbar [N][Hkv][D] fp32 -> ksplit [Hkv][NG][D/32][3][64 lanes][8] bf16: the A operands of
// mfma_f32_16x16x32_bf16 for cube group cg (cubes 16cg..16cg+15), k-step c, term (hi, mid, lo): lane (n16, q4)
// holds cube 16cg + n16, head-dim elements 32c + 8*q4 .. +7.  Cubes beyond N are zero.
__global__ void kbar_split_kernel(Geom g, int NG, const float *__restrict__ kbar, uint16_t *__restrict__ ksplit)
{
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

template <int D, int MAXG>
__global__ __launch_bounds__(SELM_THREADS, 2) void cube_select_mfma_kernel(
    Geom g, int NG, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ ksplit, float top_p,
    uint32_t *__restrict__ sel_mask, int32_t *__restrict__ sel_count)
{
    constexpr int KS = D / 32;
    constexpr int GB = KS * 3 * 1024;            // bytes of one cube group's operands
    constexpr int PIECES = GB / 16;              // 16-byte pieces of a group
    constexpr int PPT = (PIECES + SELM_THREADS - 1) / SELM_THREADS;
    __shared__ __attribute__((aligned(16))) unsigned char abuf[GB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    // workgroup -> (query cube, KV head, block of rows); late cubes (most candidates) first
    const int nblk_max = (g.G * g.Cmax + SELM_ROWS - 1) / SELM_ROWS;
    const int blk = blockIdx.x % nblk_max;
    const int kv = (blockIdx.x / nblk_max) % g.Hkv;
    const int i = g.N - 1 - blockIdx.x / (nblk_max * g.Hkv);
    const CubeBox qbox = cube_box(g, i);
    const int P = g.G * qbox.size();  // rows of this (cube, KV head): rho = rank * G + head-in-group
    if (blk * SELM_ROWS >= P) return;

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

    if (i == 0 || top_p <= 0.f || top_p >= 1.f) {
        const int keep = (i > 0 && top_p >= 1.f) ? i : 0;  // p>=1: every preceding cube
#pragma unroll
        for (int s = 0; s < SELM_SLABS; ++s) {
            if (rowg[s] < 0) continue;
            for (int w = q4; w < g.words; w += 4) {
                const int lo = 32 * w;
                uint32_t bits = 0;
                if (keep >= lo + 32) bits = 0xffffffffu;
                else if (keep > lo) bits = (1u << (keep - lo)) - 1u;
                sel_mask[(size_t)rowg[s] * g.words + w] = bits;
            }
            if (q4 == 0) sel_count[rowg[s]] = keep;
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
    const int ng = (i + 15) >> 4;  // cube groups that hold candidates (the same for every row here)
    sel_f32x4 acc[SELM_SLABS][MAXG];
#pragma unroll
    for (int s = 0; s < SELM_SLABS; ++s)
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg) acc[s][cg] = sel_f32x4{0.f, 0.f, 0.f, 0.f};
    const sel_u32x4 *src = reinterpret_cast<const sel_u32x4 *>(ksplit + (size_t)kv * NG * (GB / 2));
    sel_u32x4 pre[PPT];
#pragma unroll
    for (int u = 0; u < PPT; ++u)
        if (tid + SELM_THREADS * u < PIECES) pre[u] = src[tid + SELM_THREADS * u];
#pragma unroll
    for (int cg = 0; cg < MAXG; ++cg) {
        if (cg < ng) {  // uniform for the workgroup
            __syncthreads();  // the previous group's operands have been consumed
#pragma unroll
            for (int u = 0; u < PPT; ++u)
                if (tid + SELM_THREADS * u < PIECES)
                    reinterpret_cast<sel_u32x4 *>(abuf)[tid + SELM_THREADS * u] = pre[u];
            if (cg + 1 < ng) {
#pragma unroll
                for (int u = 0; u < PPT; ++u)
                    if (tid + SELM_THREADS * u < PIECES)
                        pre[u] = src[(size_t)(cg + 1) * PIECES + tid + SELM_THREADS * u];
            }
            __syncthreads();
#pragma unroll
            for (int c = 0; c < KS; ++c)
#pragma unroll
                for (int term = 0; term < 3; ++term) {
                    const sel_bf16x8 af =
                        *reinterpret_cast<const sel_bf16x8 *>(abuf + ((c * 3 + term) * 64 + lane) * 16);
#pragma unroll
                    for (int s = 0; s < SELM_SLABS; ++s)
                        acc[s][cg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, qf[s][c], acc[s][cg], 0, 0, 0);
                }
        }
    }

    const float scale = 1.44269504088896340736f / sqrtf((float)D);
    const int ng4 = (ng + 3) >> 2;  // groups are processed four at a time below
#pragma unroll
    for (int s = 0; s < SELM_SLABS; ++s) {
        // ---- softmax numerators e = exp2(logit*log2(e)/sqrt(D) - max), 0 for non-candidates; kept in acc
        float mx = -INFINITY;
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool valid = 16 * cg + 4 * q4 + v < i;
                const float x = valid ? acc[s][cg][v] * scale : -INFINITY;
                acc[s][cg][v] = x;
                mx = fmaxf(mx, x);
            }
        mx = selm_quad_max(mx);
        float part = 0.f;
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float x = acc[s][cg][v];
                const float e = (x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(x - mx);
                acc[s][cg][v] = e;
                part += e;
            }
        const float target = top_p * selm_quad_sum(part);

        // ---- largest tau (as a bit pattern) with mass{e >= tau} >= target: positive floats order like
        // unsigned integers, so tau is found bit by bit; every row (four lanes) runs its own search
        uint32_t tau = 0;
        for (int b = 30; b >= 0; --b) {
            const uint32_t cand = tau | (1u << b);
            float sum = 0.f;
#pragma unroll
            for (int k4 = 0; k4 < (MAXG + 3) / 4; ++k4)
                if (k4 < ng4) {
#pragma unroll
                    for (int cg = 4 * k4; cg < 4 * k4 + 4 && cg < MAXG; ++cg)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const float e = acc[s][cg][v];
                            sum += (__float_as_uint(e) >= cand) ? e : 0.f;
                        }
                }
            if (selm_quad_sum(sum) >= target) tau = cand;
            // tau is the value of one of the row's elements, the smallest kept one, and it lies in
            // [tau, tau + 2^b).  Once that bucket holds a single distinct value for every row of the slab the
            // remaining bits are known; looked at every fourth step once the exponent bits are settled.
            if (b <= 22 && (b & 3) == 2) {
                const uint32_t width = 1u << b;
                uint32_t mn = 0xffffffffu, mxb = 0u;
#pragma unroll
                for (int k4 = 0; k4 < (MAXG + 3) / 4; ++k4)
                    if (k4 < ng4) {
#pragma unroll
                        for (int cg = 4 * k4; cg < 4 * k4 + 4 && cg < MAXG; ++cg)
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                                const bool inb = bits - tau < width;
                                mn = inb ? min(mn, bits) : mn;
                                mxb = inb ? max(mxb, bits) : mxb;
                            }
                    }
                // min over the row's four lanes via max of the complement
                mn = ~selm_quad_umax(~mn);
                mxb = selm_quad_umax(mxb);
                if (__all(mn == mxb)) {
                    tau = mn;
                    break;
                }
            }
        }
        const float tauf = __uint_as_float(tau);
        float sgt = 0.f;
        int neq = 0;
#pragma unroll
        for (int cg = 0; cg < MAXG; ++cg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint32_t bits = __float_as_uint(acc[s][cg][v]);
                sgt += bits > tau ? acc[s][cg][v] : 0.f;
                neq += (bits == tau && tau != 0) ? 1 : 0;
            }
        const float mass_gt = selm_quad_sum(sgt);
        const int neq_row = (int)selm_quad_sum((float)neq);  // small counts: exact in fp32

        // ---- kept flags.  An element equal to tau is kept while the mass before it (in cube order among the
        // tied ones) is below the target; with a single such element that is always the case.
        uint32_t nib[MAXG];  // bit v of nib[cg]: cube 16cg + 4q4 + v is kept
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

        // ---- mask words: word w covers cube groups 2w, 2w+1; a lane's nibble of group cg sits at bit
        // 16*(cg%2) + 4*q4; the four lanes of a row are OR-ed together
        int kept = 0;
#pragma unroll
        for (int w = 0; w < (MAXG + 1) / 2; ++w) {
            uint32_t word = nib[2 * w] << (4 * q4);
            if (2 * w + 1 < MAXG) word |= nib[2 * w + 1] << (16 + 4 * q4);
            word = selm_quad_or(word);
            kept += __popc(word);
            if (w < g.words && rowg[s] >= 0 && q4 == (w & 3)) sel_mask[(size_t)rowg[s] * g.words + w] = word;
        }
        if (rowg[s] >= 0 && q4 == 0) sel_count[rowg[s]] = kept;
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

__global__ void csr_fill_kernel(Geom g, long long R, const uint32_t *__restrict__ sel_mask,
                                const int64_t *__restrict__ row_ptr, int32_t *__restrict__ cube_idx, long long capacity)
{
    const long long row = (long long)blockIdx.x * blockDim.x + threadIdx.x;
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

static int select_npad(const Geom &g) { return (g.N + 63) / 64 * 64; }
static bool select_use_mfma(const Geom &g) { return g.N <= SELM_MAX_CUBES; }
static int select_groups(const Geom &g) { return (g.N + 15) / 16; }
static size_t select_ksplit_bytes(const Geom &g)
{
    return (((size_t)g.Hkv * select_groups(g) * (g.D / 32) * 3 * 1024) + 255) / 256 * 256;
}
static long long scan_tiles(const Geom &g) { return ((long long)g.S * g.Hq + SCAN_TILE - 1) / SCAN_TILE; }

size_t select_workspace_bytes(const Geom &g)
{
    // the transposed fp32 mean keys (general path) or their bf16 split (MFMA path), then the scan's tile sums
    const size_t kbarT = (size_t)g.Hkv * g.D * select_npad(g) * sizeof(float);
    const size_t first = select_use_mfma(g) ? select_ksplit_bytes(g) : ((kbarT + 255) / 256) * 256;
    const size_t tiles = (size_t)scan_tiles(g) * sizeof(long long);
    return first + ((tiles + 255) / 256) * 256;
}

template <int D>
static void launch_select_d(const Geom &g, int Npad, const uint16_t *Q, const float *kbarT, float top_p,
                            uint32_t *sel_mask, int32_t *sel_count, hipStream_t st)
{
    const long long R = (long long)g.S * g.Hq;
    const dim3 grid((unsigned)((R + SELECT_ROWS_PER_BLOCK - 1) / SELECT_ROWS_PER_BLOCK)), block(SELECT_THREADS);
#define ADASPARK_SELECT_CASE(MAXK)                                                                          \
    hipLaunchKernelGGL((cube_select_kernel<D, MAXK>), grid, block, 0, st, g, Npad, Q, kbarT, top_p, sel_mask, \
                       sel_count)
    if (g.N <= 64) ADASPARK_SELECT_CASE(1);
    else if (g.N <= 128) ADASPARK_SELECT_CASE(2);
    else if (g.N <= 256) ADASPARK_SELECT_CASE(4);
    else if (g.N <= 512) ADASPARK_SELECT_CASE(8);
    else if (g.N <= 1024) ADASPARK_SELECT_CASE(16);
    else ADASPARK_SELECT_CASE(32);
#undef ADASPARK_SELECT_CASE
}

hipError_t launch_cube_select(const Geom &g, const uint16_t *Q, const float *kbar, float top_p, uint32_t *sel_mask,
                              int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx, int64_t capacity, void *ws,
                              hipStream_t st)
{
    const int Npad = select_npad(g);
    const long long R = (long long)g.S * g.Hq;
    const size_t kbarT_bytes = (((size_t)g.Hkv * g.D * Npad * sizeof(float)) + 255) / 256 * 256;
    const size_t first_bytes = select_use_mfma(g) ? select_ksplit_bytes(g) : kbarT_bytes;
    long long *tile_sum = reinterpret_cast<long long *>(reinterpret_cast<char *>(ws) + first_bytes);

    if (select_use_mfma(g)) {
        uint16_t *ksplit = reinterpret_cast<uint16_t *>(ws);
        const int NG = select_groups(g);
        const size_t total = (size_t)g.Hkv * NG * (g.D / 32) * 64;
        hipLaunchKernelGGL(kbar_split_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, NG, kbar,
                           ksplit);
        const int nblk_max = (g.G * g.Cmax + SELM_ROWS - 1) / SELM_ROWS;
        const dim3 grid((unsigned)((size_t)g.N * g.Hkv * nblk_max)), block(SELM_THREADS);
#define ADASPARK_SELM_CASE(DD, MAXG)                                                                          \
    hipLaunchKernelGGL((cube_select_mfma_kernel<DD, MAXG>), grid, block, 0, st, g, NG, Q, ksplit, top_p, sel_mask, \
                       sel_count)
        if (g.D == 64) {
            if (NG <= 4) ADASPARK_SELM_CASE(64, 4);
            else ADASPARK_SELM_CASE(64, 16);
        } else {
            if (NG <= 4) ADASPARK_SELM_CASE(128, 4);
            else ADASPARK_SELM_CASE(128, 16);
        }
#undef ADASPARK_SELM_CASE
    } else {
        float *kbarT = reinterpret_cast<float *>(ws);
        const size_t total = (size_t)g.Hkv * g.D * Npad;
        hipLaunchKernelGGL(kbar_transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, Npad,
                           kbar, kbarT);
        if (g.D == 64) launch_select_d<64>(g, Npad, Q, kbarT, top_p, sel_mask, sel_count, st);
        else launch_select_d<128>(g, Npad, Q, kbarT, top_p, sel_mask, sel_count, st);
    }

    if (row_ptr != nullptr) {
        const int tiles = (int)scan_tiles(g);
        hipLaunchKernelGGL(scan_tile_sums_kernel, dim3(tiles), dim3(SCAN_THREADS), 0, st, sel_count, R, tile_sum);
        hipLaunchKernelGGL(scan_tile_offsets_kernel, dim3(1), dim3(SCAN_THREADS), 0, st, tile_sum, tiles);
        hipLaunchKernelGGL(scan_write_kernel, dim3(tiles), dim3(SCAN_THREADS), 0, st, sel_count, R, tile_sum, row_ptr);
        hipLaunchKernelGGL(csr_fill_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, g, R, sel_mask, row_ptr,
                           cube_idx, (long long)capacity);
    }
    return hipGetLastError();
}

}  // namespace adaspark
