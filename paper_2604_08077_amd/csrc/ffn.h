// Internal interface of the token-selective FFN (Sec. 3.3): ffn.hip (selection, tables, mean compensation) and
// ffn_gemm.hip (the two matrix products on the activated tokens).
#pragma once
#include "kvtile.h"

namespace adaspark {

constexpr int FFN_ROW_TILE = 256;        // activated tokens per workgroup of the matrix products
constexpr int FFN_MAX_CUBE_TOKENS = 4096;

// Views into the caller's workspace.
struct FfnWorkspace {
    int32_t *cnt;       // [N]      activated tokens per cube
    int32_t *cube_ptr;  // [N + 1]  exclusive prefix sums of cnt; cube_ptr[N] = number of activated tokens
    int32_t *active;    // [rows]   activated tokens, cube by cube in rank order, padded to a multiple of FFN_ROW_TILE
    int32_t *slot;      // [S]      index of a token in `active`, or -1
    uint16_t *H;        // [rows][d_ff]     bf16 hidden activations silu(gate) * up
    float *F;           // [rows][d_model]  fp32 FFN(x) of the activated tokens
    long long rows;     // S rounded up to a multiple of FFN_ROW_TILE
    size_t bytes;
};
FfnWorkspace ffn_workspace(const Geom &g, int d_model, int d_ff, void *ws);

hipError_t launch_ffn_select(const Geom &g, int d_model, const uint16_t *X, float top_p, float eps, uint8_t *keep,
                             float *score, int32_t *keep_count, hipStream_t st);
hipError_t launch_ffn_sparse(const Geom &g, int d_model, int d_ff, const uint16_t *X, const uint16_t *Wg,
                             const uint16_t *Wu, const uint16_t *Wd, const uint8_t *keep, uint16_t *Y, void *ws,
                             hipStream_t st);

// H[r][:] = silu(W_gate . x) * (W_up . x) for x = X[active[r]], r < *n_rows (rows up to the next multiple of
// FFN_ROW_TILE are computed too, from the padding of `active`).  m_tiles: upper bound of row tiles (grid size).
hipError_t launch_ffn_gemm_gated(const uint16_t *X, const int32_t *active, const uint16_t *Wg, const uint16_t *Wu,
                                 int d_model, int d_ff, int m_tiles, const int32_t *n_rows, uint16_t *H, hipStream_t st);
// F[r][:] = W_down . H[r][:] in fp32.
hipError_t launch_ffn_gemm_down(const uint16_t *H, const uint16_t *Wd, int d_ff, int d_model, int m_tiles,
                                const int32_t *n_rows, float *F, hipStream_t st);

}  // namespace adaspark
