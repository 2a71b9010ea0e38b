// Cube geometry shared by the kernels of this library (Sec. 3.1, video cube
// partition).  Host code fills a Geom from the caller's adaspark_shape; device
// code maps (cube, rank) <-> raster token index with it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/adaspark.h"

namespace adaspark {

constexpr int KEY_TILE = 64;  // keys per staged K/V tile; cubes are padded to a multiple of it in the packed KV layout

struct Geom {
    int T, H, W;        // video token grid
    int ct, ch, cw;     // cube shape
    int Hq, Hkv, D, G;  // heads, head_dim, group size Hq/Hkv
    int nTb, nHb, nWb;  // video cubes along each axis
    int Nv, Sv;         // video cubes, video tokens
    int Sp, Np;         // text tokens before the video, cut into Np text cubes of up to Cmax tokens
    int St;             // text tokens after the video, cut into text cubes the same way
    int N;              // cubes: leading text cubes, video cubes, trailing text cubes
    int S;              // tokens: leading text, video (raster order), trailing text
    int Cmax;           // tokens in an unclipped cube
    int TPC;            // key tiles per cube in the packed layout = ceil(Cmax / KEY_TILE)
    int words;          // u32 words per selection-mask row = ceil(N / 32)
    int ragged;         // some cubes are smaller than Cmax (clipped at the grid edge, or the last text cube)
    int causal;         // 1: the paper's operator.  0 (selection and forward attention only): candidates are all other
                        // video cubes, the own cube is attended in full
};

inline Geom make_geom(const adaspark_shape &s)
{
    Geom g;
    g.T = s.frames; g.H = s.height; g.W = s.width;
    g.ct = s.cube_t; g.ch = s.cube_h; g.cw = s.cube_w;
    g.Hq = s.q_heads; g.Hkv = s.kv_heads; g.D = s.head_dim; g.G = s.q_heads / s.kv_heads;
    g.nTb = (g.T + g.ct - 1) / g.ct; g.nHb = (g.H + g.ch - 1) / g.ch; g.nWb = (g.W + g.cw - 1) / g.cw;
    g.Nv = g.nTb * g.nHb * g.nWb;
    g.Sv = g.T * g.H * g.W;
    g.Sp = s.prefix_tokens;
    g.St = s.text_tokens;
    g.Cmax = g.ct * g.ch * g.cw;
    g.Np = (g.Sp + g.Cmax - 1) / g.Cmax;
    g.N = g.Np + g.Nv + (g.St + g.Cmax - 1) / g.Cmax;
    g.S = g.Sp + g.Sv + g.St;
    g.TPC = (g.Cmax + KEY_TILE - 1) / KEY_TILE;
    g.words = (g.N + 31) / 32;
    g.causal = 1;
    g.ragged = (g.T % g.ct != 0) || (g.H % g.ch != 0) || (g.W % g.cw != 0) || (g.St % g.Cmax != 0) ||
               (g.Sp % g.Cmax != 0);
    return g;
}

// Clipped extents and origin of cube c.  A text cube is a run of consecutive tokens: t0 < 0, w0 = its first
// token, ew = its length.  Video cubes are numbered from Np; their box is in video-grid coordinates.
struct CubeBox {
    int t0, h0, w0;  // origin in the token grid
    int et, eh, ew;  // extents after clipping at the grid edge
    __host__ __device__ int size() const { return et * eh * ew; }
};

__host__ __device__ inline CubeBox cube_box(const Geom &g, int c)
{
    CubeBox b;
    if (c < g.Np) {
        const int first = c * g.Cmax;
        b.t0 = -1; b.h0 = 0; b.w0 = first;
        b.et = 1; b.eh = 1; b.ew = min(g.Cmax, g.Sp - first);
        return b;
    }
    c -= g.Np;
    if (c >= g.Nv) {
        const int first = (c - g.Nv) * g.Cmax;
        b.t0 = -1; b.h0 = 0; b.w0 = g.Sp + g.Sv + first;
        b.et = 1; b.eh = 1; b.ew = min(g.Cmax, g.St - first);
        return b;
    }
    const int wb = c % g.nWb, hb = (c / g.nWb) % g.nHb, tb = c / (g.nWb * g.nHb);
    b.t0 = tb * g.ct; b.h0 = hb * g.ch; b.w0 = wb * g.cw;
    b.et = min(g.ct, g.T - b.t0); b.eh = min(g.ch, g.H - b.h0); b.ew = min(g.cw, g.W - b.w0);
    return b;
}

// Token index of the token with rank `rank` in the cube described by b.
__host__ __device__ inline int token_of(const Geom &g, const CubeBox &b, int rank)
{
    if (b.t0 < 0) return b.w0 + rank;
    const int lw = rank % b.ew, lh = (rank / b.ew) % b.eh, lt = rank / (b.ew * b.eh);
    return g.Sp + ((b.t0 + lt) * g.H + (b.h0 + lh)) * g.W + (b.w0 + lw);
}

// Cube of token n (rank not needed by the callers of this one).
__host__ __device__ inline int cube_of_token(const Geom &g, int n)
{
    if (n < g.Sp) return n / g.Cmax;
    n -= g.Sp;
    if (n >= g.Sv) return g.Np + g.Nv + (n - g.Sv) / g.Cmax;
    const int w = n % g.W, h = (n / g.W) % g.H, t = n / (g.W * g.H);
    return g.Np + ((t / g.ct) * g.nHb + (h / g.ch)) * g.nWb + (w / g.cw);
}

// bf16 <-> fp32 bit helpers.
__device__ inline float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ inline uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
    return (uint16_t)(u >> 16);
}

// Kernel launchers (defined one per .hip file).  All return hipError_t from the launch.
hipError_t launch_cube_pool(const Geom &g, const uint16_t *K, float *kbar, hipStream_t st);
size_t select_workspace_bytes(const Geom &g);
// byte offset of the call's int32 status word inside that workspace (ADASPARK_OK or ADASPARK_ECAPACITY, on the device)
size_t select_status_offset(const Geom &g);
// sel_mask rows from a compact list (row_ptr, cube_idx as launch_cube_select writes them)
void launch_mask_from_csr(const Geom &g, const int64_t *row_ptr, const int32_t *cube_idx, uint32_t *sel_mask,
                          hipStream_t st);
// top_k < 0: Top-p selection with threshold top_p; top_k >= 0: fixed Top-K selection (top_p ignored).
hipError_t launch_cube_select(const Geom &g, const uint16_t *Q, const float *kbar, float top_p, int top_k,
                              uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                              int64_t capacity, void *ws, hipStream_t st);
// Group-shared variant: one selection per (token, KV head) from the group's mean query, copied to the group's rows.
size_t select_shared_workspace_bytes(const Geom &g);
hipError_t launch_cube_select_shared(const Geom &g, const uint16_t *Q, const float *kbar, float top_p, uint32_t *sel_mask,
                                     int32_t *sel_count, void *ws, hipStream_t st);
// out[0..n] = exclusive prefix sums of count[0..n-1]; tile_sum: scan_tile_sum_bytes(n) bytes of scratch (select.hip)
size_t scan_tile_sum_bytes(long long n);
void launch_exclusive_scan(const int32_t *count, long long n, long long *tile_sum, int64_t *out, hipStream_t st);
size_t attn_workspace_bytes(const Geom &g);
hipError_t launch_kv_pack(const Geom &g, const uint16_t *K, const uint16_t *V, void *ws, bool natural_f16, hipStream_t st);
// Kernel-choice flags of the sparse attention entries (ints, written and read on the device only):
//   [FLAG_MODE]      the row-stationary kernel that runs: 1 compaction, 2 masked walk
//   [FLAG_ESTIMATE]  smallest share of selected candidate cubes over the KV heads, permille, from a sample of rows
//   [FLAG_ACTIVE]    1 if some KV head is the key-stationary kernel's
//   [FLAG_UNION]     share of the candidate cubes that some row of a masked-walk workgroup selected (that kernel skips
//                    the others), permille, from a sample of workgroups; 1000 where rows select independently
//   [FLAG_KV + kv]   3: the rows of KV head kv are left to the key-stationary kernel; 0: to the kernel above
// The per-head part exists only where the caller's workspace has room for the key-stationary kernel's tables
// (kernels take `kv_modes` = 1); the block is then 512 bytes long and followed by that kernel's per-head pair
// totals, u64 [Hkv], which the kernel that fills the first two flags also clears.  Otherwise the block is the
// four ints at the end of the minimum workspace.
constexpr int FLAG_MODE = 0, FLAG_ESTIMATE = 1, FLAG_ACTIVE = 2, FLAG_UNION = 3, FLAG_KV = 4;
constexpr int PAIRS_MAX_KV_HEADS = 64;
constexpr int FLAG_BLOCK_BYTES = 512;

// A kernel that uses more than 64 KB of dynamic LDS has to be allowed to, once per device, before its first launch.
// One object per kernel: ensure() asks the runtime only the first time a device (or a larger size) comes by, so a
// launch costs no runtime call beyond itself afterwards.  Thread-safe without a lock: the worst a race does is ask
// twice.
struct LdsOptIn {
    static constexpr int MAX_DEVICES = 64;
    std::atomic<int> bytes_set[MAX_DEVICES] = {};
    hipError_t ensure(const void *kernel, int bytes)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < MAX_DEVICES;
        if (tracked && bytes_set[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess && tracked) bytes_set[dev].store(bytes, std::memory_order_release);
        return e;
    }
};

// Number of candidate (row, cube) pairs of a causal selection: every row of cube i has i preceding cubes.
unsigned long long candidate_pairs(const Geom &g);

// sel_mask == nullptr: dense (every preceding cube attended); otherwise sparse_kernel is an adaspark_sparse_kernel.
// The automatic choice writes a flag into the last 16 bytes of the packed workspace.  scratch (256-byte aligned, may
// be null): memory for the key-stationary kernel's records.
hipError_t launch_attn(const Geom &g, const uint16_t *Q, void *packed, const uint32_t *sel_mask, int sparse_kernel,
                       void *scratch, size_t scratch_bytes, uint16_t *O, float *lse, hipStream_t st);
// The compacting sparse kernel alone (attn_compact.hip).  flags (device, may be null): the flag block above; a
// workgroup runs only if flags[FLAG_MODE] == my_mode and (kv_modes) its KV head is not the key-stationary kernel's.
hipError_t launch_attn_compact(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask,
                               const int *flags, int my_mode, int kv_modes, uint16_t *O, float *lse, hipStream_t st);
// The key-stationary sparse kernel (attn_pairs.hip).  pairs_scratch_bytes: scratch for max_selected selected (row,
// cube) pairs.  pairs_flags: the flag block inside the scratch memory (with the per-head part), or null if the
// scratch memory does not hold the tables or the geometry is not covered.  launch_attn_pairs expects
// flags[FLAG_MODE], flags[FLAG_ESTIMATE] set and flags[FLAG_KV ...] zero; it enqueues kernels that -- unless the
// estimate is well above pairs_below_permille and force is 0 -- count the pairs exactly per KV head, hand the heads
// whose share is below pairs_below_permille (all heads, if force) to this path as long as their records fit, and run
// it for those heads.
bool pairs_supported(const Geom &g);
size_t pairs_scratch_bytes(const Geom &g, long long max_selected);
int *pairs_flags(const Geom &g, void *scratch, size_t scratch_bytes);
hipError_t launch_attn_pairs(const Geom &g, const uint16_t *Q, const void *packed, const uint32_t *sel_mask, void *scratch,
                             size_t scratch_bytes, int force, int pairs_below_permille, uint16_t *O, float *lse,
                             hipStream_t st);

// Backward of the attention entries (attn_bwd.hip): dQ, dK, dV in bf16 from Q, K, V, the forward's O and
// log-sum-exp, and dO.  sel_mask == nullptr: dense causal attention.  ws: attn_bwd_workspace_bytes(g).
size_t attn_bwd_workspace_bytes(const Geom &g);
hipError_t launch_attn_bwd(const Geom &g, const uint16_t *Q, const uint16_t *K, const uint16_t *V, const uint16_t *O,
                           const float *lse, const uint16_t *dO, const uint32_t *sel_mask, uint16_t *dQ, uint16_t *dK,
                           uint16_t *dV, void *ws, hipStream_t st);

}  // namespace adaspark
