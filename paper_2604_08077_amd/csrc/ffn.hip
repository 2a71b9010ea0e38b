// Adaptive Token-Selective FFN (Sec. 3.3): everything around the two matrix products --
//   ffn_select_kernel   token norms, importance scores, Top-p token selection per cube (Eqs. 4-5)
//   ffn_count_kernel / ffn_fill_kernel   the list of activated tokens in cube order, and every token's place in it
//   ffn_finish_kernel   residual sums and mean compensation (Eqs. 6-7)
// One workgroup per cube in all of them.
#include "ffn.h"

namespace adaspark {

constexpr int SEL_THREADS = 1024;
constexpr int TAB_THREADS = 256;
constexpr int FIN_THREADS = 512;

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// Sum of n floats held in LDS, in a fixed order (the same on every run): per-thread strided partial sums, then a
// tree over the wavefronts.  All threads get the result.  `red` holds one float per wavefront.
template <int THREADS>
__device__ float block_sum(const float *vals, int n, float *red)
{
    float acc = 0.f;
    for (int j = threadIdx.x; j < n; j += THREADS) acc += vals[j];
    acc = wave_sum(acc);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) tot += red[w];
    return tot;
}

// Eqs. 4-5 for cube blockIdx.x.
__global__ __launch_bounds__(SEL_THREADS) void ffn_select_kernel(Geom g, int d_model, const uint16_t *__restrict__ X,
                                                                 float top_p, float eps, uint8_t *__restrict__ keep,
                                                                 float *__restrict__ score, int32_t *__restrict__ keep_count)
{
    extern __shared__ float sm[];
    float *sc = sm;                 // [Cmax] norms, then scores
    float *red = sm + g.Cmax;       // [SEL_THREADS / 64]
    int *cnt = reinterpret_cast<int *>(red + SEL_THREADS / 64);
    const int c = blockIdx.x;
    const CubeBox b = cube_box(g, c);
    const int n = b.size();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunks = d_model / 8;  // 16-byte pieces of a token
    if (threadIdx.x == 0) *cnt = 0;

    // token norms: a wavefront per token, four tokens in flight
    constexpr int NW = SEL_THREADS / 64, INFLIGHT = 4;
    for (int r0 = wave; r0 < n; r0 += INFLIGHT * NW) {
        const uint16_t *x[INFLIGHT];
        float a[INFLIGHT];
#pragma unroll
        for (int u = 0; u < INFLIGHT; ++u) {
            const int r = r0 + u * NW;
            x[u] = X + (size_t)token_of(g, b, r < n ? r : r0) * d_model;
            a[u] = 0.f;
        }
        for (int k = lane; k < chunks; k += 64) {
            u32x4 v[INFLIGHT];
#pragma unroll
            for (int u = 0; u < INFLIGHT; ++u) v[u] = *reinterpret_cast<const u32x4 *>(x[u] + 8 * k);
#pragma unroll
            for (int u = 0; u < INFLIGHT; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = __uint_as_float(v[u][e] << 16), hi = __uint_as_float(v[u][e] & 0xffff0000u);
                    a[u] = fmaf(lo, lo, a[u]);
                    a[u] = fmaf(hi, hi, a[u]);
                }
        }
#pragma unroll
        for (int u = 0; u < INFLIGHT; ++u) {
            const float tot = wave_sum(a[u]);
            const int r = r0 + u * NW;
            if (lane == 0 && r < n) sc[r] = sqrtf(tot);
        }
    }
    __syncthreads();
    const float total = block_sum<SEL_THREADS>(sc, n, red);
    // a cube of zero-norm tokens with eps = 0: every score is 0 (Eq. 4's epsilon is there for this cube)
    const float inv = (total + eps > 0.f) ? 1.0f / (total + eps) : 0.f;
    __syncthreads();
    for (int j = threadIdx.x; j < n; j += SEL_THREADS) sc[j] = sc[j] * inv;
    __syncthreads();

    const bool text = b.t0 < 0;
    int mine = 0;
    for (int j = threadIdx.x; j < n; j += SEL_THREADS) {
        const float sj = sc[j];
        bool k = true;
        if (!text && top_p < 1.0f) {
            float before = 0.f;  // mass of the tokens ranked before j: larger score, or equal score and lower rank
            for (int i = 0; i < n; ++i) {
                const float si = sc[i];
                if (si > sj || (si == sj && i < j)) before += si;
            }
            k = before < top_p;
        }
        const int tok = token_of(g, b, j);
        keep[tok] = k ? 1 : 0;
        if (score) score[tok] = sj;
        mine += k ? 1 : 0;
    }
    if (keep_count) {
        if (mine) atomicAdd(cnt, mine);
        __syncthreads();
        if (threadIdx.x == 0) keep_count[c] = *cnt;
    }
}

// Activated tokens per cube.
__global__ __launch_bounds__(TAB_THREADS) void ffn_count_kernel(Geom g, const uint8_t *__restrict__ keep,
                                                                int32_t *__restrict__ cnt)
{
    __shared__ int tot;
    const CubeBox b = cube_box(g, blockIdx.x);
    const int n = b.size();
    if (threadIdx.x == 0) tot = 0;
    __syncthreads();
    int mine = 0;
    if (keep == nullptr) {
        if (threadIdx.x == 0) mine = n;
    } else {
        for (int j = threadIdx.x; j < n; j += TAB_THREADS) mine += keep[token_of(g, b, j)] != 0;
    }
    if (mine) atomicAdd(&tot, mine);
    __syncthreads();
    if (threadIdx.x == 0) cnt[blockIdx.x] = tot;
}

// cube_ptr[c] = activated tokens of the cubes before c; active[cube_ptr[c] + k] = k-th activated token of cube c in
// rank order; slot[token] = its index in `active`, or -1.  The last cube also writes cube_ptr[N] and pads `active`
// with token 0 up to a multiple of FFN_ROW_TILE (rows that the matrix products compute and nobody reads).
__global__ __launch_bounds__(TAB_THREADS) void ffn_fill_kernel(Geom g, const uint8_t *__restrict__ keep,
                                                               const int32_t *__restrict__ cnt,
                                                               int32_t *__restrict__ cube_ptr, int32_t *__restrict__ active,
                                                               int32_t *__restrict__ slot)
{
    __shared__ int part[TAB_THREADS];
    __shared__ int base_s;
    const int c = blockIdx.x;
    const CubeBox b = cube_box(g, c);
    const int n = b.size();
    // offset of this cube: sum of the counts of the cubes before it
    int acc = 0;
    for (int i = threadIdx.x; i < c; i += TAB_THREADS) acc += cnt[i];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int d = TAB_THREADS / 2; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) part[threadIdx.x] += part[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) base_s = part[0];
    __syncthreads();
    const int base = base_s;
    __syncthreads();

    // every thread takes a run of consecutive ranks; exclusive scan of the runs' counts
    const int per = (n + TAB_THREADS - 1) / TAB_THREADS;
    const int j0 = min(n, (int)threadIdx.x * per), j1 = min(n, j0 + per);
    int mine = 0;
    for (int j = j0; j < j1; ++j) mine += keep == nullptr || keep[token_of(g, b, j)] != 0;
    part[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < TAB_THREADS; d <<= 1) {
        const int v = (int)threadIdx.x >= d ? part[threadIdx.x - d] : 0;
        __syncthreads();
        part[threadIdx.x] += v;
        __syncthreads();
    }
    int pos = base + part[threadIdx.x] - mine;
    for (int j = j0; j < j1; ++j) {
        const int tok = token_of(g, b, j);
        if (keep == nullptr || keep[tok] != 0) {
            active[pos] = tok;
            slot[tok] = pos++;
        } else {
            slot[tok] = -1;
        }
    }
    if (threadIdx.x == 0) cube_ptr[c] = base;
    if (c == g.N - 1) {
        const int total = base + part[TAB_THREADS - 1];
        if (threadIdx.x == 0) cube_ptr[g.N] = total;
        const int padded = (total + FFN_ROW_TILE - 1) / FFN_ROW_TILE * FFN_ROW_TILE;
        for (int i = total + threadIdx.x; i < padded; i += TAB_THREADS) active[i] = 0;
    }
}

// Eqs. 6-7 for cube blockIdx.x: F holds FFN(x) of the activated tokens (fp32, row = index in the active list).
// A thread owns eight columns (per block of 8 * FIN_THREADS columns): it walks the cube's activated rows once,
// writing y = x + F and summing F (rows in list order), then gives the bypassed tokens x + mean.
__global__ __launch_bounds__(FIN_THREADS) void ffn_finish_kernel(Geom g, int d_model, const uint16_t *__restrict__ X,
                                                                 const float *__restrict__ F,
                                                                 const int32_t *__restrict__ cube_ptr,
                                                                 const int32_t *__restrict__ active,
                                                                 const int32_t *__restrict__ slot, uint16_t *__restrict__ Y)
{
    const int c = blockIdx.x;
    const CubeBox b = cube_box(g, c);
    const int n = b.size();
    const int first = cube_ptr[c], count = cube_ptr[c + 1] - first;
    const float inv = count > 0 ? 1.0f / (float)count : 0.f;
    auto add_store = [&](int tok, int col, const f32x4 &f0, const f32x4 &f1) __attribute__((always_inline)) {
        const u32x4 xv = *reinterpret_cast<const u32x4 *>(X + (size_t)tok * d_model + col);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = __uint_as_float(xv[e] << 16) + (e < 2 ? f0[2 * e] : f1[2 * e - 4]);
            const float hi = __uint_as_float(xv[e] & 0xffff0000u) + (e < 2 ? f0[2 * e + 1] : f1[2 * e - 3]);
            o[e] = (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
        }
        *reinterpret_cast<u32x4 *>(Y + (size_t)tok * d_model + col) = o;
    };
    for (int col = 8 * threadIdx.x; col < d_model; col += 8 * FIN_THREADS) {
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        const float *f = F + (size_t)first * d_model + col;
        int r = 0;
        for (; r + 4 <= count; r += 4) {
            f32x4 v0[4], v1[4];
            int tok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v0[u] = *reinterpret_cast<const f32x4 *>(f + (size_t)(r + u) * d_model);
                v1[u] = *reinterpret_cast<const f32x4 *>(f + (size_t)(r + u) * d_model + 4);
                tok[u] = active[first + r + u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc0 += v0[u];
                acc1 += v1[u];
                add_store(tok[u], col, v0[u], v1[u]);
            }
        }
        for (; r < count; ++r) {
            const f32x4 v0 = *reinterpret_cast<const f32x4 *>(f + (size_t)r * d_model);
            const f32x4 v1 = *reinterpret_cast<const f32x4 *>(f + (size_t)r * d_model + 4);
            acc0 += v0;
            acc1 += v1;
            add_store(active[first + r], col, v0, v1);
        }
        const f32x4 mean0 = acc0 * inv, mean1 = acc1 * inv;
        for (int j = 0; j < n; ++j) {
            const int tok = token_of(g, b, j);
            if (slot[tok] < 0) add_store(tok, col, mean0, mean1);
        }
    }
}

hipError_t launch_ffn_select(const Geom &g, int d_model, const uint16_t *X, float top_p, float eps, uint8_t *keep,
                             float *score, int32_t *keep_count, hipStream_t st)
{
    const size_t lds = (size_t)(g.Cmax + SEL_THREADS / 64 + 4) * sizeof(float);
    hipLaunchKernelGGL(ffn_select_kernel, dim3(g.N), dim3(SEL_THREADS), lds, st, g, d_model, X, top_p, eps, keep, score,
                       keep_count);
    return hipGetLastError();
}

FfnWorkspace ffn_workspace(const Geom &g, int d_model, int d_ff, void *ws)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t rows = ((size_t)g.S + FFN_ROW_TILE - 1) / FFN_ROW_TILE * FFN_ROW_TILE;
    FfnWorkspace w;
    unsigned char *p = static_cast<unsigned char *>(ws);
    size_t off = 0;
    w.cnt = reinterpret_cast<int32_t *>(p + off); off = up(off + (size_t)g.N * 4);
    w.cube_ptr = reinterpret_cast<int32_t *>(p + off); off = up(off + (size_t)(g.N + 1) * 4);
    w.active = reinterpret_cast<int32_t *>(p + off); off = up(off + rows * 4);
    w.slot = reinterpret_cast<int32_t *>(p + off); off = up(off + (size_t)g.S * 4);
    w.H = reinterpret_cast<uint16_t *>(p + off); off = up(off + rows * (size_t)d_ff * 2);
    w.F = reinterpret_cast<float *>(p + off); off = up(off + rows * (size_t)d_model * 4);
    w.bytes = off;
    w.rows = (long long)rows;
    return w;
}

hipError_t launch_ffn_sparse(const Geom &g, int d_model, int d_ff, const uint16_t *X, const uint16_t *Wg,
                             const uint16_t *Wu, const uint16_t *Wd, const uint8_t *keep, uint16_t *Y, void *ws,
                             hipStream_t st)
{
    const FfnWorkspace w = ffn_workspace(g, d_model, d_ff, ws);
    hipLaunchKernelGGL(ffn_count_kernel, dim3(g.N), dim3(TAB_THREADS), 0, st, g, keep, w.cnt);
    hipLaunchKernelGGL(ffn_fill_kernel, dim3(g.N), dim3(TAB_THREADS), 0, st, g, keep, w.cnt, w.cube_ptr, w.active,
                       w.slot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int m_tiles = (int)(w.rows / FFN_ROW_TILE);
    // hidden activations of the activated tokens, then the layer's output for them
    e = launch_ffn_gemm_gated(X, w.active, Wg, Wu, d_model, d_ff, m_tiles, w.cube_ptr + g.N, w.H, st);
    if (e != hipSuccess) return e;
    e = launch_ffn_gemm_down(w.H, Wd, d_ff, d_model, m_tiles, w.cube_ptr + g.N, w.F, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ffn_finish_kernel, dim3(g.N), dim3(FIN_THREADS), 0, st, g, d_model, X, w.F, w.cube_ptr, w.active,
                       w.slot, Y);
    return hipGetLastError();
}

}  // namespace adaspark
