// The two matrix products of the token-selective FFN (Sec. 3.3, Eq. 6) on the activated tokens:
//   gated:  H[r][n] = silu(sum_k X[active[r]][k] Wg[n][k]) * (sum_k X[active[r]][k] Wu[n][k])   bf16 out
//   down :  F[r][n] = sum_k H[r][k] Wd[n][k]                                                    fp32 out
// Both are C = A.B^T with A (activations) and B (weights) stored row-major with the reduction index contiguous.
//
// Workgroup = 256 activation rows x 256 weight rows, 64 reduction elements per step, 8 wavefronts (2 along the
// activation rows x 4 along the weight rows, 128 x 64 each).  Tiles go from global memory straight into LDS
// (global_load_lds_dwordx4), two stages, one workgroup barrier per step; the 16-byte chunks of a tile row are
// XOR-swizzled by the choice of which chunk a lane fetches, so that the MFMA operand reads are conflict-free.
// mfma_f32_16x16x32_bf16 with the weights on the M side and the activations on the N side: a lane ends up with four
// consecutive output features of one token, which is what a row-major store wants.  For the gated product a tile's
// weight rows are 128 rows of W_gate and the same 128 rows of W_up, and every wavefront holds matching pairs.
#include "attn_tile.h"
#include "ffn.h"

namespace adaspark {

constexpr int GT = FFN_ROW_TILE;            // rows of a tile, both operands
constexpr int GK = 64;                      // reduction elements per step: 128 bytes per row
constexpr int GEMM_THREADS = 512;
constexpr int TILE_BYTES = GT * GK * 2;     // 32 KB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // activations, weights
constexpr int GEMM_LDS = 2 * STAGE_BYTES;   // 128 KB

template <bool GATED>
__global__ __launch_bounds__(GEMM_THREADS) void ffn_gemm_kernel(const uint16_t *__restrict__ A,
                                                                const int32_t *__restrict__ gather,
                                                                const uint16_t *__restrict__ W0,
                                                                const uint16_t *__restrict__ W1, int K, int n_tiles,
                                                                int m_tiles, const int32_t *__restrict__ n_rows_ptr,
                                                                void *__restrict__ out, int ldo)
{
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
    // Workgroup -> tile.  Consecutive workgroups go to different XCDs (each with its own L2), so the 32 tiles of a
    // 4 x 8 block -- four row tiles that share their weights with eight weight tiles that share their rows -- are
    // given to one XCD: block k of 32 goes to XCD k % 8.
    const int total = (m_tiles + 3) / 4 * 4 * n_tiles;
    const int idx = blockIdx.x >> 3;
    const int logical = (((idx >> 5) * 8 + (blockIdx.x & 7)) << 5) + (idx & 31);
    if (logical >= total) return;
    const int tm = logical / (4 * n_tiles) * 4 + (logical & 3);
    const int tn = (logical >> 2) % n_tiles;
    if (tm >= m_tiles || tm * GT >= *n_rows_ptr) return;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n16 = lane & 15, q4 = lane >> 4;
    const int wm = wave >> 2, wn = wave & 3;

    // Tile loads: wavefront w fills the 4 KB [4w, 4w+4) KB of either tile: rows 32w .. 32w+31.  Physical 16-byte slot
    // x of a tile holds chunk `chunk` of row `row` (vt_tile_coords); a lane's four sources stay fixed over the loop.
    uint32_t voffA[4], voffW[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row, chunk;
        vt_tile_coords((wave * 4 + i) * 64 + lane, row, chunk);
        const long long arow = gather ? (long long)gather[tm * GT + row] : (long long)row;
        voffA[i] = (uint32_t)(arow * K * 2 + chunk * 16);
        voffW[i] = (uint32_t)((GATED ? (row & 127) : row) * K * 2 + chunk * 16);
    }
    const unsigned char *baseA = reinterpret_cast<const unsigned char *>(A) + (gather ? 0 : (size_t)tm * GT * K * 2);
    const unsigned char *baseW =
        GATED ? reinterpret_cast<const unsigned char *>(wave < 4 ? W0 : W1) + (size_t)tn * 128 * K * 2
              : reinterpret_cast<const unsigned char *>(W0) + (size_t)tn * GT * K * 2;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + (uint32_t)(wave * 4096));
    auto issue = [&](int stage, int kstep) __attribute__((always_inline)) {
        const void *sa = uniform_ptr(baseA + (size_t)kstep * (GK * 2));
        const void *sw = uniform_ptr(baseW + (size_t)kstep * (GK * 2));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma_1k_s(lds0 + (uint32_t)(stage * STAGE_BYTES + i * 1024), sa, voffA[i]);
            dma_1k_s(lds0 + (uint32_t)(stage * STAGE_BYTES + TILE_BYTES + i * 1024), sw, voffW[i]);
        }
    };

    // Operand reads: row rb + n16 (rb a multiple of 16), chunk 4c + q4 -> rb * 128 + lo[c]
    uint32_t lo[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
        lo[c] = (uint32_t)((n16 >> 1) * 256 + (((((n16 & 1) << 3) | (4 * c + q4)) ^ ((n16 >> 1) & 7)) << 4));
    int wrow[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) wrow[g] = GATED ? (g >> 1) * 128 + wn * 32 + (g & 1) * 16 : wn * 64 + g * 16;

    f32x4 acc[8][4];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[s][g] = f32x4{0.f, 0.f, 0.f, 0.f};

    // One reduction step: 16 groups of four MFMAs (half c of the step, slab s), each needing one activation operand
    // and the half's four weight operands.  Operand loads run three groups ahead of their use through a ring of
    // four registers, the second half's weights arrive under the first half's MFMAs, and the written order is kept.
    auto compute = [&](int stage) __attribute__((always_inline)) {
        const unsigned char *ta = smem + stage * STAGE_BYTES + wm * (128 * 128);
        const unsigned char *tw = smem + stage * STAGE_BYTES + TILE_BYTES;
        auto load_a = [&](int i) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8 *>(ta + (i & 7) * 2048 + lo[i >> 3]);
        };
        auto load_w = [&](int c, int g) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8 *>(tw + wrow[g] * 128 + lo[c]);
        };
        bf16x8 wf[2][4], ring[4];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < 4; ++g) wf[0][g] = load_w(0, g);
#pragma unroll
        for (int i = 0; i < 3; ++i) ring[i] = load_a(i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int c = i >> 3, sl = i & 7;
#pragma unroll
            for (int g = 0; g < 4; ++g)
                acc[sl][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[c][g], ring[i & 3], acc[sl][g], 0, 0, 0);
            if (i + 3 < 16) ring[(i + 3) & 3] = load_a(i + 3);
            if (i >= 1 && i <= 4) wf[1][i - 1] = load_w(1, i - 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int nk = K / GK;
    issue(0, 0);
    for (int k = 0; k < nk; k += 2) {
        tile_barrier();  // step k has landed in stage 0; every wavefront is done reading stage 1
        if (k + 1 < nk) issue(1, k + 1);
        compute(0);
        if (k + 1 < nk) {
            tile_barrier();
            if (k + 2 < nk) issue(0, k + 2);
            compute(1);
        }
    }

    // Results: a lane holds output features 4*q4 .. 4*q4+3 of weight group g for the token of row n16 of slab s.
    const size_t row0 = (size_t)tm * GT + wm * 128 + n16;
    if (GATED) {
        uint16_t *H = static_cast<uint16_t *>(out);
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                bf16x2 p0, p1;
                float h[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float z = acc[s][g][v];
                    h[v] = z / (1.0f + __expf(-z)) * acc[s][g + 2][v];
                }
                p0[0] = (__bf16)h[0]; p0[1] = (__bf16)h[1]; p1[0] = (__bf16)h[2]; p1[1] = (__bf16)h[3];
                uint2 o;
                o.x = *reinterpret_cast<uint32_t *>(&p0);
                o.y = *reinterpret_cast<uint32_t *>(&p1);
                *reinterpret_cast<uint2 *>(H + (row0 + s * 16) * ldo + tn * 128 + wn * 32 + g * 16 + 4 * q4) = o;
            }
    } else {
        float *F = static_cast<float *>(out);
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<f32x4 *>(F + (row0 + s * 16) * ldo + tn * GT + wn * 64 + g * 16 + 4 * q4) = acc[s][g];
    }
}

template <bool GATED>
hipError_t launch_gemm(const uint16_t *A, const int32_t *gather, const uint16_t *W0, const uint16_t *W1, int K,
                       int n_tiles, int m_tiles, const int32_t *n_rows, void *out, int ldo, hipStream_t st)
{
    static LdsOptIn opted;  // one per instantiation
    const hipError_t e = opted.ensure(reinterpret_cast<const void *>(&ffn_gemm_kernel<GATED>), GEMM_LDS);
    if (e != hipSuccess) return e;
    const long long total = (long long)((m_tiles + 3) / 4 * 4) * n_tiles;
    const long long blocks32 = ((total + 31) / 32 + 7) / 8 * 8;  // whole rounds over the eight XCDs
    hipLaunchKernelGGL((ffn_gemm_kernel<GATED>), dim3((unsigned)(blocks32 * 32)), dim3(GEMM_THREADS), GEMM_LDS, st, A,
                       gather, W0, W1, K, n_tiles, m_tiles, n_rows, out, ldo);
    return hipGetLastError();
}

hipError_t launch_ffn_gemm_gated(const uint16_t *X, const int32_t *active, const uint16_t *Wg, const uint16_t *Wu,
                                 int d_model, int d_ff, int m_tiles, const int32_t *n_rows, uint16_t *H, hipStream_t st)
{
    return launch_gemm<true>(X, active, Wg, Wu, d_model, d_ff / 128, m_tiles, n_rows, H, d_ff, st);
}

hipError_t launch_ffn_gemm_down(const uint16_t *H, const uint16_t *Wd, int d_ff, int d_model, int m_tiles,
                                const int32_t *n_rows, float *F, hipStream_t st)
{
    return launch_gemm<false>(H, nullptr, Wd, nullptr, d_ff, d_model / GT, m_tiles, n_rows, F, d_model, st);
}

}  // namespace adaspark
