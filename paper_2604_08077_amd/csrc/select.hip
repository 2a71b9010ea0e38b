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
static long long scan_tiles(const Geom &g) { return ((long long)g.S * g.Hq + SCAN_TILE - 1) / SCAN_TILE; }

size_t select_workspace_bytes(const Geom &g)
{
    const size_t kbarT = (size_t)g.Hkv * g.D * select_npad(g) * sizeof(float);
    const size_t tiles = (size_t)scan_tiles(g) * sizeof(long long);
    return ((kbarT + 255) / 256) * 256 + ((tiles + 255) / 256) * 256;
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
    float *kbarT = reinterpret_cast<float *>(ws);
    const size_t kbarT_bytes = (((size_t)g.Hkv * g.D * Npad * sizeof(float)) + 255) / 256 * 256;
    long long *tile_sum = reinterpret_cast<long long *>(reinterpret_cast<char *>(ws) + kbarT_bytes);

    const size_t total = (size_t)g.Hkv * g.D * Npad;
    hipLaunchKernelGGL(kbar_transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, Npad, kbar,
                       kbarT);
    if (g.D == 64) launch_select_d<64>(g, Npad, Q, kbarT, top_p, sel_mask, sel_count, st);
    else launch_select_d<128>(g, Npad, Q, kbarT, top_p, sel_mask, sel_count, st);

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
