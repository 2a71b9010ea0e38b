/*
 * adaspark.h -- C ABI of the AdaS-Attn library for AMD MI355X (gfx950).
 *
 * Adaptive Cube-Selective Attention (AdaSpark, Sec. 3.1-3.2): video tokens on a
 * frames x height x width grid are grouped into 3D cubes (Sec. 3.1); every key
 * cube is mean-pooled; every (query token, query head) scores all preceding
 * cubes (Eq. 1), keeps a Top-p nucleus of them (Eq. 2) and runs exact softmax
 * attention over the kept cubes plus the causal part of its own cube (Eq. 3).
 *
 * Conventions shared by all entry points
 *   - Every data pointer is a DEVICE pointer owned by the caller, contiguous,
 *     16-byte aligned.  The library never allocates or frees device memory and
 *     keeps no state between calls (beyond remembering, per device, which of its
 *     kernels have been granted their large LDS and where its one static scratch
 *     array lies); scratch space is the caller's `workspace`
 *     (size from adaspark_workspace_bytes; contents need not be initialised and
 *     are undefined afterwards).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue kernels on it; they never synchronise with the host.
 *   - Token index n = (t*height + h)*width + w ("raster order").  Tensors are
 *     Q,O: bf16 [tokens][q_heads][head_dim]; K,V: bf16 [tokens][kv_heads][head_dim].
 *     Query head a uses KV head a / (q_heads / kv_heads).
 *   - Cubes are numbered (tb*ceil(H/cube_h) + hb)*ceil(W/cube_w) + wb; edge
 *     cubes are clipped.  Inside a cube tokens are ranked in local (t,h,w)
 *     raster order.  "Preceding" / causal order everywhere in this library is
 *     cube-major: all tokens of cube j < i precede all tokens of cube i, and
 *     inside a cube lower rank precedes higher rank.
 *   - Text tokens (end of Sec. 3.2: cube-wise attention to the preceding visual
 *     tokens, token-wise attention to text tokens): the sequence is
 *     `prefix_tokens` text tokens, then the T*H*W video tokens (token index
 *     prefix_tokens + raster index), then `text_tokens` text tokens.  Each text
 *     span is cut into runs of cube_t*cube_h*cube_w tokens ("text cubes"; the
 *     last of a span may be shorter) and cubes are numbered in sequence order:
 *     the prefix's text cubes, the video cubes, the trailing text cubes.  The
 *     candidates of the selection rule (Eqs. 1-2) are, for every query, the
 *     VIDEO cubes before its own cube: a query in the trailing text scores all
 *     video cubes, a query in the prefix none.  Text is attended token-wise:
 *     a row's selection always contains every text cube before its own, and an
 *     own text cube is attended causally like any own cube.  Text cubes are
 *     never candidates; a video query with no prefix is unaffected.
 *   - Query row id r = n*q_heads + a.
 *   - Return value: ADASPARK_OK (0) or a negative adaspark_status.  Arguments
 *     are validated before anything is enqueued; on a validation error nothing
 *     was launched.  No exceptions, no process exit.
 */
#ifndef ADASPARK_H
#define ADASPARK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t frames, height, width;       /* video token grid T, H, W                            */
    int32_t cube_t, cube_h, cube_w;      /* cube shape along frames, height, width (Sec. 3.1)  */
    int32_t q_heads, kv_heads, head_dim; /* q_heads % kv_heads == 0; head_dim in {64, 128}     */
    int32_t text_tokens;                 /* text tokens that follow the video tokens (0: none)  */
    int32_t prefix_tokens;               /* text tokens that precede the video tokens (0: none); */
                                         /* tokens = prefix_tokens + T*H*W + text_tokens         */
} adaspark_shape;

typedef enum {
    ADASPARK_OK = 0,
    ADASPARK_EINVAL = -1,       /* null/misaligned pointer, bad shape, top_p outside [0,1]     */
    ADASPARK_EUNSUPPORTED = -2, /* valid request outside what the kernels cover (see below)    */
    ADASPARK_EWORKSPACE = -3,   /* workspace missing or smaller than adaspark_workspace_bytes  */
    ADASPARK_EHIP = -4,         /* the HIP runtime refused a launch                            */
    ADASPARK_ECAPACITY = -5     /* never returned by a call: the value a selection call leaves */
                                /* in its device status word when the compact list overflowed  */
} adaspark_status;

typedef enum {
    ADASPARK_CALL_CUBE_POOL = 0,
    ADASPARK_CALL_CUBE_SELECT = 1,
    ADASPARK_CALL_SPARSE_ATTN = 2,
    ADASPARK_CALL_DENSE_ATTN = 3,
    ADASPARK_CALL_ATTN_BWD = 4,
    ADASPARK_CALL_CUBE_SELECT_SHARED = 5,
    ADASPARK_CALL_SPARSE_ATTN_CSR = 6
} adaspark_call;

/* Which kernel a sparse-attention call runs.  All compute the same result (Eq. 3).
 *   COMPACT  row blocks walk the key cubes; per cube the rows that selected it are gathered into dense MFMA
 *            tiles.  Pays only when very few cubes are selected.
 *   MASKED   every row walks every preceding cube and its selection bits act as a mask: dense work, none of
 *            the gathering cost; the better choice when most cubes are selected.
 *   PAIRS    key-stationary: a workgroup keeps one key cube on chip and runs the rows that selected it; every
 *            (row, selected cube) pair leaves a partial result of 2 * head_dim + 16 bytes in scratch memory (an
 *            fp16 vector scaled by its fp32 maximum) and a second kernel merges them per row.  Work follows the selection; the better choice when less than
 *            about 40 % of the cubes are selected.  Needs extra workspace (adaspark_pairs_workspace_bytes) and
 *            cubes of at most 256 tokens.  If the selection turns out to hold more pairs than the scratch
 *            memory was sized for, the call runs MASKED instead (decided on the device).
 *   AUTO     the choice is made on the device from the selected share (no host synchronisation).  PAIRS is
 *            among the candidates iff the workspace is large enough for it, and the choice is then made per KV
 *            head: heads whose rows select little go to PAIRS, the others to MASKED (or COMPACT). */
typedef enum {
    ADASPARK_SPARSE_AUTO = 0,
    ADASPARK_SPARSE_COMPACT = 1,
    ADASPARK_SPARSE_MASKED = 2,
    ADASPARK_SPARSE_PAIRS = 3
} adaspark_sparse_kernel;

/* Limits: head_dim in {64,128}; number of cubes (text cubes included) <= ADASPARK_MAX_CUBES;
 * tokens*q_heads < 2^31.
 * causal: non-zero is the paper's operator (candidates: the video cubes before the own cube; the own cube up to the
 * row's rank).  causal == 0 is a variant of the selection and forward attention entries: the candidates of Eqs. 1-2 are
 * ALL video cubes other than the row's own, every text cube other than the own one is attended (its bit set), the own
 * cube is attended in full, and the dense entries are plain attention over all tokens; it runs on the masked-walk /
 * dense kernel (a forced COMPACT or PAIRS gives ADASPARK_EUNSUPPORTED), and the backward entry is causal only. */
#define ADASPARK_MAX_CUBES 2048

/* Host-only helpers (no GPU work). */
int adaspark_num_cubes(const adaspark_shape *shape, int32_t *n_cubes);
int adaspark_workspace_bytes(const adaspark_shape *shape, int which_call /* adaspark_call */, size_t *bytes);
const char *adaspark_status_string(int status);
/* Workspace size for the sparse attention entries that also lets the key-stationary kernel (ADASPARK_SPARSE_PAIRS)
 * run for selections of up to max_selected selected (row, cube) pairs in total (the sum of sel_count):
 * adaspark_workspace_bytes(ADASPARK_CALL_SPARSE_ATTN) plus, per row, 12 bytes of tables and a scaled copy of its
 * Q vector, plus 2 * head_dim + 24 bytes per pair and per row.  The sparse entries use whatever lies beyond the minimum size this way. */
int adaspark_pairs_workspace_bytes(const adaspark_shape *shape, int64_t max_selected, size_t *bytes);

/*
 * Cube mean keys (Eq. 1: k-bar_j = Mean(k in K_j)), per KV head.
 *   K    in   bf16 [tokens][kv_heads][head_dim]
 *   kbar out  fp32 [cubes][kv_heads][head_dim]   (fp32 accumulation, never rounded to bf16)
 */
int adaspark_cube_pool(const adaspark_shape *shape, const void *K, float *kbar, void *stream);

/*
 * Relevance scoring and Top-p cube selection (Eqs. 1-2) for every query row.
 * For row r = (token n in cube i, head a): logits q.kbar_j/sqrt(head_dim) over
 * cubes j < i, softmax, then the minimal set of highest-probability cubes whose
 * mass reaches top_p (ties: lower cube index first).  top_p >= 1 keeps every
 * preceding cube, top_p == 0 keeps none; rows of cube 0 keep none.
 *   Q         in   bf16 [tokens][q_heads][head_dim]
 *   kbar      in   fp32 [cubes][kv_heads][head_dim]
 *   sel_mask  out  u32  [tokens*q_heads][ceil(cubes/32)]; bit (j%32) of word j/32 set
 *                  iff cube j is selected.  The own cube's bit is never set.
 *   sel_count out  i32  [tokens*q_heads] number of selected cubes (for a text row: including the
 *                  text cubes before its own, which are always set)
 *   row_ptr   out  i64  [tokens*q_heads + 1] exclusive prefix sum of sel_count, or NULL
 *   cube_idx  out  i32  [capacity] selected cube ids, ascending inside each row,
 *                  row r at [row_ptr[r], row_ptr[r+1]); entries at positions
 *                  >= capacity are dropped, so the list is complete iff
 *                  row_ptr[tokens*q_heads] <= capacity.  NULL iff row_ptr is NULL.
 *   workspace      adaspark_workspace_bytes(ADASPARK_CALL_CUBE_SELECT)
 * Overflow of the compact list is found on the device (the call never waits for it): every selection call leaves
 * an int32 status word in its workspace, at byte adaspark_select_status_offset(shape): ADASPARK_OK, or
 * ADASPARK_ECAPACITY if the rows' lists needed more than `capacity` entries.  The caller reads it (a 4-byte copy)
 * after the stream has reached the end of the call.  The mask and the counts are complete either way.
 */
int adaspark_cube_select(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int causal,
                         uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                         int64_t capacity, void *workspace, size_t workspace_bytes, void *stream);
/* Host-only: where in the selection workspace the device status word of the call lies. */
int adaspark_select_status_offset(const adaspark_shape *shape, size_t *offset);

/*
 * adaspark_cube_select for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and so cannot bring a workspace: the same kernels and the same results,
 * with the workspace -- the bf16 split of the mean keys and the tile sums of the compact list's scan -- in a device
 * array that is part of the library (ADASPARK_NOALLOC_SCRATCH_BYTES per GPU, held from the library's load to the end
 * of the process).  The call allocates and frees nothing.  A shape whose selection workspace
 * (adaspark_workspace_bytes(ADASPARK_CALL_CUBE_SELECT)) exceeds that size is refused with ADASPARK_EWORKSPACE before
 * anything is enqueued; 4 MiB covers 262,144 tokens in 1,024 cubes with 4 KV heads of 128.  All calls on one GPU share
 * that GPU's array: it holds whatever the last call left, every call rewrites what it reads, and two calls that
 * overlap in time on one GPU (different streams or threads) race -- serialise them, or use adaspark_cube_select
 * with a workspace each.  Other arguments and outputs as adaspark_cube_select, except that the status word of the
 * call lies in the library's array, out of the caller's reach: whether the compact list fitted is read off the list
 * itself (row_ptr[tokens*q_heads] <= capacity).
 */
#define ADASPARK_NOALLOC_SCRATCH_BYTES (4u << 20)
int adaspark_cube_select_noalloc(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int causal,
                                 uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                                 int64_t capacity, void *stream);

/*
 * Fixed Top-K cube selection, the comparison baseline of the paper's ablation
 * "Effect of Top-P Adaptive Selection" (Sec. 4) and of its table of selection
 * strategies: row r keeps the top_k preceding cubes of highest relevance (Eq. 1),
 * ties by lower cube index; all of them if it has no more than top_k.  Same
 * outputs, workspace and conventions as adaspark_cube_select; the result feeds
 * adaspark_sparse_attn unchanged.  top_k = 0 keeps nothing (local attention
 * only); top_k < 0 is ADASPARK_EINVAL.
 */
int adaspark_cube_select_topk(const adaspark_shape *shape, const void *Q, const float *kbar, int32_t top_k, int causal,
                              uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                              int64_t capacity, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Group-shared Top-p selection: a variant in which the query heads of a GQA group share one set of cubes per token
 * (the paper selects per query head and does not discuss grouped-query attention).  The cubes are scored by the
 * group's mean query -- equivalently, by the mean of the group's logits of Eq. 1 -- and Eq. 2 is applied once per
 * (token, KV head); every row of the group gets that set.  The mean query is part of the definition, precision
 * included: the group's bf16 queries added in head order in float32, times float32(1)/float32(group size), rounded
 * to bf16 (nearest even).  With one query head per KV head this is adaspark_cube_select.
 *   outputs as adaspark_cube_select (no compact list);
 *   workspace  adaspark_workspace_bytes(ADASPARK_CALL_CUBE_SELECT_SHARED)
 */
int adaspark_cube_select_shared(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int causal,
                                uint32_t *sel_mask, int32_t *sel_count, void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * Sparse attention (Eq. 3 plus the own-cube rule of Sec. 3.2): row r attends
 * all tokens of the cubes set in its sel_mask row and the tokens of its own
 * cube with rank <= its own rank; softmax(q.K_att^T/sqrt(head_dim)).V_att with
 * bf16 inputs, fp32 accumulation and fp32 softmax.
 *   Q,K,V     in   bf16 (layouts above)
 *   sel_mask  in   as written by adaspark_cube_select
 *   O         out  bf16 [tokens][q_heads][head_dim]
 *   lse       out  fp32 [tokens*q_heads] natural-log sum-exp of the scaled logits, or NULL.  (The masked-walk,
 *                  dense and key-stationary kernels multiply Q by the softmax scale and round it to fp16: a score,
 *                  and with it this value, is accurate to about 2^-12 * sum_d |q_d k_d| / sqrt(head_dim).)
 * The score products q.k take fp16 operands: K converts exactly while |k| <= 65504, the limit of that format; larger
 * magnitudes, in K or in the scaled Q, saturate there.  P.V takes bf16 operands as they are.
 *   workspace      adaspark_workspace_bytes(ADASPARK_CALL_SPARSE_ATTN), or more: with
 *                  adaspark_pairs_workspace_bytes(...) the key-stationary kernel becomes a candidate
 */
int adaspark_sparse_attn(const adaspark_shape *shape, const void *Q, const void *K, const void *V,
                         const uint32_t *sel_mask, int causal, void *O, float *lse,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * adaspark_sparse_attn fed the compact list instead of the mask rows (Eq. 3 on the sets S_r as
 * adaspark_cube_select lists them): row r attends the cubes cube_idx[row_ptr[r] .. row_ptr[r+1]) -- ascending,
 * complete (status word ADASPARK_OK) -- and the causal part of its own cube.  The list is first turned back into
 * mask rows inside the workspace; results are bit-identical to the mask-fed entry.
 *   row_ptr   in   i64  [tokens*q_heads + 1];   cube_idx  in  i32  [row_ptr[tokens*q_heads]]
 *   workspace      adaspark_workspace_bytes(ADASPARK_CALL_SPARSE_ATTN_CSR) (the packed K/V copy and the mask rows),
 *                  or more: what lies beyond is scratch for the key-stationary kernel, as above
 */
int adaspark_sparse_attn_csr(const adaspark_shape *shape, const void *Q, const void *K, const void *V,
                             const int64_t *row_ptr, const int32_t *cube_idx, int causal, void *O, float *lse,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Dense causal attention in the same cube-major order (the comparison point of
 * the paper's FLOPs analysis, supp. "Detail of FLOPs Calculation"): row r
 * attends every token that precedes it in cube-major order, and itself.
 * Built from the same kernels as adaspark_sparse_attn with every preceding
 * cube taken as selected.  Arguments as above, without sel_mask.
 */
int adaspark_dense_attn(const adaspark_shape *shape, const void *Q, const void *K, const void *V,
                        int causal, void *O, float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Split-phase form of the two attention entries.  Both attention entries first
 * gather K and V into a cube-major, tile-blocked copy inside the workspace (the
 * layout Alg. 1 calls "Reshape K,V into Cubes") and then run the attention
 * kernel on that copy.  A caller that attends the same K,V more than once (a
 * Top-p sweep, sparse and dense side by side) can pack once:
 *   adaspark_kv_pack            fills `workspace` (same size as for the attention entries)
 *   adaspark_sparse_attn_packed / adaspark_dense_attn_packed
 *                               read a workspace filled by adaspark_kv_pack for the same shape.  The K/V copy
 *                               in it is only read; the sparse entries use the last 16 bytes of the minimum size
 *                               and everything beyond it as scratch, so two sparse calls on one workspace must
 *                               not overlap in time.
 *   adaspark_sparse_attn_packed_with
 *                               the same with an explicit adaspark_sparse_kernel (the plain entry uses AUTO).
 * adaspark_sparse_attn(...) == adaspark_kv_pack(...) followed by adaspark_sparse_attn_packed(...).
 */
int adaspark_kv_pack(const adaspark_shape *shape, const void *K, const void *V,
                     void *workspace, size_t workspace_bytes, void *stream);
int adaspark_sparse_attn_packed(const adaspark_shape *shape, const void *Q, void *packed, size_t packed_bytes,
                                const uint32_t *sel_mask, int causal, void *O, float *lse, void *stream);
int adaspark_sparse_attn_packed_with(const adaspark_shape *shape, const void *Q, void *packed, size_t packed_bytes,
                                     const uint32_t *sel_mask, int causal, int sparse_kernel, void *O, float *lse,
                                     void *stream);
int adaspark_dense_attn_packed(const adaspark_shape *shape, const void *Q, const void *packed, size_t packed_bytes,
                               int causal, void *O, float *lse, void *stream);

/*
 * Backward pass of the attention entries (the paper post-trains through the operator: supplementary material,
 * "AdaSpark Training Algorithm"; it states no gradient of its own).  Eq. 3 differentiated with the selected sets held
 * constant -- the Top-p rule is piecewise constant in Q and K.  For row r with attended keys A_r, c = 1/sqrt(head_dim):
 *   p = softmax(c q.k_j over A_r),  delta = dO.O,
 *   dV_j += p_j dO,   dS_j = p_j (dO.v_j - delta),   dQ = c sum_j dS_j k_j,   dK_j += c dS_j q
 * (dK, dV summed over all rows and all query heads of the KV head's group).
 *   Q, dO, O   in   bf16 [tokens][q_heads][head_dim]   (O and lse as the forward entry returned them)
 *   K, V       in   bf16 [tokens][kv_heads][head_dim]
 *   lse        in   fp32 [tokens*q_heads]   natural-log sum-exp of the scaled logits over A_r
 *   sel_mask   in   u32  [tokens*q_heads][ceil(cubes/32)], or NULL for dense causal attention
 *   dQ         out  bf16 [tokens][q_heads][head_dim];  dK, dV  out  bf16 [tokens][kv_heads][head_dim]
 *   workspace       adaspark_workspace_bytes(ADASPARK_CALL_ATTN_BWD): packed copies of K, V (natural and
 *                   transposed), of Q and dO (natural and transposed, in cube order) and two floats per row
 * p is rebuilt from lse in fp32 from exact score products (bf16 x bf16 accumulated in fp32, the softmax scale applied
 * in fp32); p and dS are rounded to bf16 for the other MFMA products, sums are fp32, outputs are rounded to bf16
 * once.  Limits as for the forward, and tokens*q_heads*ceil(cubes/32) < 2^30; causal != 0 only.
 */
int adaspark_sparse_attn_bwd(const adaspark_shape *shape, const void *Q, const void *K, const void *V, const void *O,
                             const float *lse, const void *dO, const uint32_t *sel_mask, int causal, void *dQ,
                             void *dK, void *dV, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Adaptive Token-Selective FFN (AdaS-FFN, Sec. 3.3, Eqs. 4-7).  Inside every video cube the tokens with the largest
 * L2 norms, a Top-p nucleus of the cube's importance distribution, take the feed-forward layer; the others receive
 * the mean of what the layer added to the activated tokens of their cube.
 *
 * The token sequence and its cubes are those of the attention entries (same adaspark_shape; q_heads, kv_heads and
 * head_dim must be valid but are not used).  The layer is the gated MLP of the backbone the paper builds on:
 *   FFN(x) = W_down . (silu(W_gate . x) * (W_up . x)),  no biases,
 *   X, Y      bf16 [tokens][d_model]
 *   W_gate, W_up  bf16 [d_ff][d_model];  W_down  bf16 [d_model][d_ff]   (row = output feature)
 * Products accumulate in fp32; the hidden activations silu(.)*(.) are rounded to bf16 once, between the two
 * matrix products; the residual sum is rounded to bf16 once, on output.
 * Limits: d_model a multiple of 256 up to 16384; d_ff a multiple of 128 up to 65536; a cube of at most 4096 tokens;
 * tokens * d_model < 2^30.  Otherwise ADASPARK_EUNSUPPORTED.
 */
typedef struct {
    int32_t d_model; /* width of a token embedding                      */
    int32_t d_ff;    /* hidden width of the feed-forward layer          */
} adaspark_ffn_dims;

/* Workspace of adaspark_ffn_sparse: tables of the activated tokens, their hidden activations (bf16, d_ff per
 * token) and the layer's output for them (fp32, d_model per token), sized for all tokens activated. */
int adaspark_ffn_workspace_bytes(const adaspark_shape *shape, const adaspark_ffn_dims *dims, size_t *bytes);

/*
 * Importance scores and Top-p token selection (Eqs. 4-5).  For every video cube C_i:
 * s_j = ||x_j||_2 / (sum over the cube of ||x_k||_2 + eps) in fp32; tokens ranked by s_j descending (ties: lower rank
 * inside the cube first); a token is activated iff the scores ranked before it sum to less than top_p.  top_p >= 1
 * activates every token, top_p == 0 none.  Text tokens are always activated (end of Sec. 3.3).
 *   X          in   bf16 [tokens][d_model]
 *   keep       out  u8   [tokens]   1: activated (set M_i), 0: bypassed (set R_i)
 *   score      out  fp32 [tokens]   s_j, or NULL
 *   keep_count out  i32  [cubes]    activated tokens per cube, or NULL
 * eps must be >= 0 and top_p in [0, 1].  No workspace.
 */
int adaspark_ffn_select(const adaspark_shape *shape, const adaspark_ffn_dims *dims, const void *X, float top_p,
                        float eps, uint8_t *keep, float *score, int32_t *keep_count, void *stream);

/*
 * The layer with mean compensation (Eqs. 6-7):
 *   y_j = x_j + FFN(x_j)                                   for activated tokens (keep[j] != 0),
 *   y_k = x_k + mean over the activated tokens of k's cube of FFN(x_j)   for the others;
 * a cube without activated tokens is copied unchanged.  keep == NULL activates every token: the dense layer
 * y = x + FFN(x), the comparison point.  `keep` is honoured as given, for text cubes too.
 *   Y          out  bf16 [tokens][d_model]   (must not alias X)
 *   workspace       adaspark_ffn_workspace_bytes
 */
int adaspark_ffn_sparse(const adaspark_shape *shape, const adaspark_ffn_dims *dims, const void *X, const void *W_gate,
                        const void *W_up, const void *W_down, const uint8_t *keep, void *Y, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * Measurement probes (not part of the method: they exist so that a benchmark can state what this GPU sustains next
 * to the datasheet peaks its kernels are priced against).
 *   adaspark_probe_copy  a plain streaming copy of `bytes` bytes (a multiple of 16) from src to dst, device buffers
 *                        that do not overlap; bytes read + bytes written over its duration is the attainable HBM rate.
 *   adaspark_probe_mfma  `workgroups` workgroups of eight wavefronts each run 16 * trips back-to-back
 *                        mfma_f32_16x16x32_bf16 on independent accumulators; *flops (host, may be NULL) receives the
 *                        floating-point operations of the launch; out: device, `workgroups` floats, overwritten.
 */
int adaspark_probe_copy(void *dst, const void *src, size_t bytes, void *stream);
int adaspark_probe_mfma(float *out, int32_t workgroups, int32_t trips, double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ADASPARK_H */
