/*
 * AdaS-Attn fp64 oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of Adaptive Cube-Selective
 * Attention (AdaSpark, Sec. 3.1-3.2, Eqs. 1-3; dense comparison point from the
 * supplementary "Detail of FLOPs Calculation").  Every floating-point step is
 * fp64; inputs are bf16 bit patterns (uint16) widened exactly.  Nothing here is
 * blocked, fused or reordered beyond what the equations state; the only
 * parallelism is an OpenMP "parallel for" over independent query rows.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP library.
 *
 * Readings fixed where the paper is silent or ambiguous (same list as in the
 * design notes of this repository):
 *   - token grid is frames x height x width, token index n = (t*H + h)*W + w;
 *     the cube shape is given explicitly as (cube_t, cube_h, cube_w)
 *     (the paper writes it h x w x t in Sec. 3.1 and (t,h,w) in Alg. 1);
 *   - edge cubes are clipped, never padded or merged;
 *   - cubes are ordered by (tb, hb, wb) raster, tokens inside a cube by local
 *     (t, h, w) raster; "preceding" (Sec. 3.2, j < i) means this cube-major
 *     order, which is what makes Eq. 3 with all preceding cubes selected equal
 *     to ordinary causal attention;
 *   - K_i^{<q} includes the query token itself (rank <= rank(q));
 *   - the own cube is not part of P_i (Eq. 1 lists cubes 1..i-1 only);
 *   - the first cube has no distribution: S = {} and attention is local only;
 *   - Top-p (Eq. 2): sort by probability descending, ties by ascending cube
 *     index; element k is kept iff the mass ranked strictly before it is < p,
 *     i.e. the minimal prefix whose mass reaches p; p >= 1 keeps every
 *     preceding cube, p = 0 keeps none;
 *   - fixed Top-K (the ablation baseline): the k highest-ranked preceding cubes
 *     in the same order, all of them if there are no more than k;
 *   - text tokens (end of Sec. 3.2) come before the video (`lead`) and after it
 *     (`text`): the sequence is leading text, video in raster order, trailing
 *     text.  Each text span is cut into runs of one full cube's length, numbered
 *     as cubes in sequence order (leading text cubes, video cubes, trailing text
 *     cubes).  Every query selects among the video cubes before its own cube (a
 *     trailing-text query: all video cubes) and always attends the text cubes
 *     before its own plus the causal part of its own: cube-wise attention to
 *     the video, token-wise attention to text;
 *   - selection is per (token, query head); with grouped-query attention query
 *     head a reads K, V and the mean keys of KV head a / (Hq / Hkv);
 *   - both the relevance score and the attention logits are scaled by
 *     1/sqrt(head_dim) (Eq. 1, Eq. 3);
 *   - mean keys stay in full precision (never rounded to bf16).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int T, H, W;      /* token grid: frames, height, width            */
    int ct, ch, cw;   /* cube shape along frames, height, width       */
    int Hq, Hkv, D;   /* query heads, KV heads, head dimension        */
    int text;         /* text tokens that follow the video tokens     */
    int lead;         /* text tokens that precede the video tokens    */
} oracle_shape;

static int video_tokens(const oracle_shape *s) { return s->T * s->H * s->W; }
static int all_tokens(const oracle_shape *s) { return s->lead + s->T * s->H * s->W + s->text; }
static int cube_tokens(const oracle_shape *s) { return s->ct * s->ch * s->cw; }

static double bf16_widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

int oracle_num_video_cubes(const oracle_shape *s)
{
    return ceil_div(s->T, s->ct) * ceil_div(s->H, s->ch) * ceil_div(s->W, s->cw);
}

/* leading text in runs of one full cube's length ("text cubes"), video cubes, trailing text cubes */
int oracle_num_lead_cubes(const oracle_shape *s) { return ceil_div(s->lead, cube_tokens(s)); }
int oracle_num_cubes(const oracle_shape *s)
{
    return oracle_num_lead_cubes(s) + oracle_num_video_cubes(s) + ceil_div(s->text, cube_tokens(s));
}

/* ---------------------------------------------------------------------------
 * Video cube partition (Sec. 3.1; Alg. 1 "Reshape K,V into Cubes"), between the
 * leading and the trailing text cubes.  For every token n (leading text, video
 * tokens in raster order, trailing text) writes the cube it falls in and its rank
 * inside that cube; for every cube its size; start[c] = sum of sizes of cubes
 * before c (start has N+1 entries).  Cube-major position of a token is
 * start[cube] + rank.
 * ------------------------------------------------------------------------- */
void oracle_cube_map(const oracle_shape *s, int32_t *cube_of, int32_t *rank_of,
                     int32_t *size_of, int64_t *start)
{
    const int nHb = ceil_div(s->H, s->ch), nWb = ceil_div(s->W, s->cw);
    const int N = oracle_num_cubes(s), Nv = oracle_num_video_cubes(s), Np = oracle_num_lead_cubes(s);
    for (int c = 0; c < N; ++c) size_of[c] = 0;
    /* text tokens (end of Sec. 3.2): run k of cube_tokens consecutive tokens of the leading text is cube k, of
     * the trailing text cube Np + Nv + k; rank = position in the run */
    for (int x = 0; x < s->lead; ++x) {
        const int c = x / cube_tokens(s);
        cube_of[x] = c;
        rank_of[x] = x % cube_tokens(s);
        size_of[c] += 1;
    }
    for (int x = 0; x < s->text; ++x) {
        const int n = s->lead + video_tokens(s) + x, c = Np + Nv + x / cube_tokens(s);
        cube_of[n] = c;
        rank_of[n] = x % cube_tokens(s);
        size_of[c] += 1;
    }
    for (int t = 0; t < s->T; ++t)
        for (int h = 0; h < s->H; ++h)
            for (int w = 0; w < s->W; ++w) {
                const int n = s->lead + (t * s->H + h) * s->W + w;
                const int tb = t / s->ct, hb = h / s->ch, wb = w / s->cw;
                const int c = Np + (tb * nHb + hb) * nWb + wb;
                /* clipped extents of this cube along height and width */
                int eh = s->H - hb * s->ch; if (eh > s->ch) eh = s->ch;
                int ew = s->W - wb * s->cw; if (ew > s->cw) ew = s->cw;
                const int lt = t - tb * s->ct, lh = h - hb * s->ch, lw = w - wb * s->cw;
                cube_of[n] = c;
                rank_of[n] = (lt * eh + lh) * ew + lw;
                size_of[c] += 1;
            }
    start[0] = 0;
    for (int c = 0; c < N; ++c) start[c + 1] = start[c] + size_of[c];
}

/* ---------------------------------------------------------------------------
 * Mean key of every cube (Eq. 1, "k-bar_j = Mean(k in K_j)"), per KV head.
 * K: bf16 bits [S][Hkv][D].  kbar: fp64 [N][Hkv][D].
 * ------------------------------------------------------------------------- */
void oracle_cube_pool(const oracle_shape *s, const uint16_t *K, double *kbar)
{
    const int S = all_tokens(s), N = oracle_num_cubes(s);
    const int Hkv = s->Hkv, D = s->D;
    int32_t *cube_of = malloc(sizeof(int32_t) * S), *rank_of = malloc(sizeof(int32_t) * S);
    int32_t *size_of = malloc(sizeof(int32_t) * N);
    int64_t *start = malloc(sizeof(int64_t) * (N + 1));
    oracle_cube_map(s, cube_of, rank_of, size_of, start);
    for (size_t i = 0; i < (size_t)N * Hkv * D; ++i) kbar[i] = 0.0;
    for (int n = 0; n < S; ++n)
        for (int g = 0; g < Hkv; ++g)
            for (int d = 0; d < D; ++d)
                kbar[((size_t)cube_of[n] * Hkv + g) * D + d] += bf16_widen(K[((size_t)n * Hkv + g) * D + d]);
    for (int c = 0; c < N; ++c)
        for (int g = 0; g < Hkv; ++g)
            for (int d = 0; d < D; ++d)
                kbar[((size_t)c * Hkv + g) * D + d] /= (double)size_of[c];
    free(cube_of); free(rank_of); free(size_of); free(start);
}

/* ---------------------------------------------------------------------------
 * Relevance distribution of one query row over n candidate cubes (Eq. 1):
 * logits[j] = q . kbar_j / sqrt(D), probs = softmax(logits).
 * q: D fp64 values; kbar_rows: pointer to cube 0 of the row's KV head with
 * stride `stride` doubles between cubes.
 * ------------------------------------------------------------------------- */
void oracle_relevance(const double *q, const double *kbar_rows, int64_t stride, int n, int D,
                      double *logits, double *probs)
{
    if (n <= 0) return;
    const double scale = 1.0 / sqrt((double)D);
    for (int j = 0; j < n; ++j) {
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += q[d] * kbar_rows[(size_t)j * stride + d];
        logits[j] = dot * scale;
    }
    double m = logits[0];
    for (int j = 1; j < n; ++j) if (logits[j] > m) m = logits[j];
    double Z = 0.0;
    for (int j = 0; j < n; ++j) { probs[j] = exp(logits[j] - m); Z += probs[j]; }
    for (int j = 0; j < n; ++j) probs[j] /= Z;
}

typedef struct { double p; int j; } ranked;

static int ranked_cmp(const void *a, const void *b)
{
    const ranked *x = a, *y = b;
    if (x->p > y->p) return -1;
    if (x->p < y->p) return 1;
    return (x->j > y->j) - (x->j < y->j);   /* ties: lower cube index first */
}

/* ---------------------------------------------------------------------------
 * Nucleus (Top-p) rule on one distribution (Eq. 2).
 * probs[n] -> keep[n] in {0,1}; returns the number kept.
 * order_out (optional, n ints): candidate indices in ranked order.
 * cum_out (optional, n doubles): cumulative mass after each ranked element.
 * ------------------------------------------------------------------------- */
int oracle_top_p(const double *probs, int n, double p, uint8_t *keep, int32_t *order_out, double *cum_out)
{
    if (n <= 0) return 0;
    ranked *r = malloc(sizeof(ranked) * n);
    for (int j = 0; j < n; ++j) { r[j].p = probs[j]; r[j].j = j; keep[j] = 0; }
    qsort(r, n, sizeof(ranked), ranked_cmp);
    int kept = 0;
    double before = 0.0;
    for (int k = 0; k < n; ++k) {
        const int take = (p >= 1.0) ? 1 : (before < p);
        if (take) { keep[r[k].j] = 1; ++kept; }
        before += r[k].p;
        if (order_out) order_out[k] = r[k].j;
        if (cum_out) cum_out[k] = before;
    }
    free(r);
    return kept;
}

/* ---------------------------------------------------------------------------
 * Cube selection for a list of query rows (Eqs. 1-2 over preceding cubes).
 * Row id r = token * Hq + head.  rows == NULL means all S*Hq rows in order.
 * Outputs (indexed by position in the row list):
 *   sel_mask  uint32 [nrows][ceil(N/32)]  bit j of word j/32 set iff cube j in S
 *                                         (the own cube is never set)
 *   sel_count int32  [nrows]
 *   near_cut  uint8  [nrows] (optional)   1 iff the row sits within `eps` of
 *             the Top-p boundary: the kept mass exceeds p by < eps, or the mass
 *             before the last kept cube is within eps of p, or the logit gap
 *             between the last kept and first dropped cube (or between the last
 *             two kept cubes) is < eps.  Diagnostic used by parity tests to
 *             classify rows where a float32 implementation may legitimately
 *             differ; it does not influence the selection.
 * ------------------------------------------------------------------------- */
void oracle_cube_select(const oracle_shape *s, const uint16_t *Q, const double *kbar, double p,
                        const int64_t *rows, int64_t nrows,
                        uint32_t *sel_mask, int32_t *sel_count, uint8_t *near_cut, double eps)
{
    const int S = all_tokens(s), N = oracle_num_cubes(s), Nv = oracle_num_video_cubes(s);
    const int Np = oracle_num_lead_cubes(s);
    const int Hq = s->Hq, Hkv = s->Hkv, D = s->D, G = Hq / Hkv;
    const int words = ceil_div(N, 32);
    int32_t *cube_of = malloc(sizeof(int32_t) * S), *rank_of = malloc(sizeof(int32_t) * S);
    int32_t *size_of = malloc(sizeof(int32_t) * N);
    int64_t *start = malloc(sizeof(int64_t) * (N + 1));
    oracle_cube_map(s, cube_of, rank_of, size_of, start);

    #pragma omp parallel
    {
        double *q = malloc(sizeof(double) * D);
        double *logits = malloc(sizeof(double) * N), *probs = malloc(sizeof(double) * N);
        double *cum = malloc(sizeof(double) * N);
        uint8_t *keep = malloc(N);
        int32_t *order = malloc(sizeof(int32_t) * N);
        #pragma omp for schedule(dynamic, 64)
        for (int64_t x = 0; x < nrows; ++x) {
            const int64_t r = rows ? rows[x] : x;
            const int n = (int)(r / Hq), a = (int)(r % Hq), g = a / G;
            const int own = cube_of[n];
            /* candidates are the video cubes before the own cube: cubes Np .. Np+i-1 (a query in the trailing
             * text scores all video cubes, one in the leading text none).  The text cubes before the own cube
             * are always attended (token-wise attention to text) */
            const int first_trailing = Np + Nv;
            const int cand_end = own < first_trailing ? own : first_trailing;
            const int i = cand_end > Np ? cand_end - Np : 0;
            uint32_t *mrow = sel_mask + (size_t)x * words;
            for (int w = 0; w < words; ++w) mrow[w] = 0;
            sel_count[x] = 0;
            if (near_cut) near_cut[x] = 0;
            for (int j = 0; j < own; ++j)
                if (j < Np || j >= first_trailing) { mrow[j >> 5] |= (uint32_t)1 << (j & 31); sel_count[x] += 1; }
            if (i == 0) continue;
            for (int d = 0; d < D; ++d) q[d] = bf16_widen(Q[((size_t)n * Hq + a) * D + d]);
            oracle_relevance(q, kbar + ((size_t)Np * Hkv + g) * D, (int64_t)Hkv * D, i, D, logits, probs);
            const int kept = oracle_top_p(probs, i, p, keep, order, cum);
            for (int j = 0; j < i; ++j) if (keep[j]) mrow[(Np + j) >> 5] |= (uint32_t)1 << ((Np + j) & 31);
            sel_count[x] += kept;
            if (near_cut && p < 1.0 && p > 0.0) {
                int flag = 0;
                const double after = cum[kept - 1];
                const double before = kept >= 2 ? cum[kept - 2] : 0.0;
                if (after - p < eps || p - before < eps) flag = 1;
                if (kept < i && logits[order[kept - 1]] - logits[order[kept]] < eps) flag = 1;
                if (kept >= 2 && logits[order[kept - 2]] - logits[order[kept - 1]] < eps) flag = 1;
                near_cut[x] = (uint8_t)flag;
            }
        }
        free(q); free(logits); free(probs); free(cum); free(keep); free(order);
    }
    free(cube_of); free(rank_of); free(size_of); free(start);
}

/* ---------------------------------------------------------------------------
 * Fixed Top-K rule on one distribution (the baseline of the ablation "Effect of
 * Top-P Adaptive Selection", Sec. 4): rank by probability descending, ties by
 * ascending cube index, keep the first min(k, n).  Returns the number kept.
 * order_out (optional, n ints): candidate indices in ranked order.
 * ------------------------------------------------------------------------- */
int oracle_top_k(const double *probs, int n, int k, uint8_t *keep, int32_t *order_out)
{
    if (n <= 0) return 0;
    ranked *r = malloc(sizeof(ranked) * n);
    for (int j = 0; j < n; ++j) { r[j].p = probs[j]; r[j].j = j; keep[j] = 0; }
    qsort(r, n, sizeof(ranked), ranked_cmp);
    int kept = 0;
    for (int t = 0; t < n; ++t) {
        if (t < k) { keep[r[t].j] = 1; ++kept; }
        if (order_out) order_out[t] = r[t].j;
    }
    free(r);
    return kept;
}

/* ---------------------------------------------------------------------------
 * Top-K cube selection for a list of query rows: as oracle_cube_select with the
 * Top-K rule in place of Top-p.  The ranking uses the logits of Eq. 1 (softmax
 * is monotone, so this is the ranking by probability, free of underflow).
 * near_cut (optional): 1 iff the logit gap between the last kept and the first
 * dropped cube is < eps.
 * ------------------------------------------------------------------------- */
void oracle_cube_select_topk(const oracle_shape *s, const uint16_t *Q, const double *kbar, int k,
                             const int64_t *rows, int64_t nrows,
                             uint32_t *sel_mask, int32_t *sel_count, uint8_t *near_cut, double eps)
{
    const int S = all_tokens(s), N = oracle_num_cubes(s), Nv = oracle_num_video_cubes(s);
    const int Np = oracle_num_lead_cubes(s);
    const int Hq = s->Hq, Hkv = s->Hkv, D = s->D, G = Hq / Hkv;
    const int words = ceil_div(N, 32);
    int32_t *cube_of = malloc(sizeof(int32_t) * S), *rank_of = malloc(sizeof(int32_t) * S);
    int32_t *size_of = malloc(sizeof(int32_t) * N);
    int64_t *start = malloc(sizeof(int64_t) * (N + 1));
    oracle_cube_map(s, cube_of, rank_of, size_of, start);

    #pragma omp parallel
    {
        double *q = malloc(sizeof(double) * D);
        double *logits = malloc(sizeof(double) * N), *probs = malloc(sizeof(double) * N);
        uint8_t *keep = malloc(N);
        int32_t *order = malloc(sizeof(int32_t) * N);
        #pragma omp for schedule(dynamic, 64)
        for (int64_t x = 0; x < nrows; ++x) {
            const int64_t r = rows ? rows[x] : x;
            const int n = (int)(r / Hq), a = (int)(r % Hq), g = a / G;
            const int own = cube_of[n];
            /* candidates are the video cubes before the own cube: cubes Np .. Np+i-1 (a query in the trailing
             * text scores all video cubes, one in the leading text none).  The text cubes before the own cube
             * are always attended (token-wise attention to text) */
            const int first_trailing = Np + Nv;
            const int cand_end = own < first_trailing ? own : first_trailing;
            const int i = cand_end > Np ? cand_end - Np : 0;
            uint32_t *mrow = sel_mask + (size_t)x * words;
            for (int w = 0; w < words; ++w) mrow[w] = 0;
            sel_count[x] = 0;
            if (near_cut) near_cut[x] = 0;
            for (int j = 0; j < own; ++j)
                if (j < Np || j >= first_trailing) { mrow[j >> 5] |= (uint32_t)1 << (j & 31); sel_count[x] += 1; }
            if (i == 0) continue;
            for (int d = 0; d < D; ++d) q[d] = bf16_widen(Q[((size_t)n * Hq + a) * D + d]);
            oracle_relevance(q, kbar + ((size_t)Np * Hkv + g) * D, (int64_t)Hkv * D, i, D, logits, probs);
            /* rank the logits: the same order as the probabilities, and exact where exp() would underflow */
            const int kept = oracle_top_k(logits, i, k, keep, order);
            for (int j = 0; j < i; ++j) if (keep[j]) mrow[(Np + j) >> 5] |= (uint32_t)1 << ((Np + j) & 31);
            sel_count[x] += kept;
            if (near_cut && kept > 0 && kept < i && logits[order[kept - 1]] - logits[order[kept]] < eps)
                near_cut[x] = 1;
        }
        free(q); free(logits); free(probs); free(keep); free(order);
    }
    free(cube_of); free(rank_of); free(size_of); free(start);
}

/* ---------------------------------------------------------------------------
 * Sparse attention for a list of query rows (Eq. 3 and the own-cube rule of
 * Sec. 3.2): keys = all tokens of the cubes whose bit is set in the row's mask,
 * plus the tokens of the query's own cube with rank <= the query's rank.
 * Two passes over the key set: maximum logit, then the softmax sums.
 * Q bf16 [S][Hq][D], K,V bf16 [S][Hkv][D]; out fp64 [nrows][D];
 * n_keys (optional) int64 [nrows] = size of the attended key set.
 * ------------------------------------------------------------------------- */
static void sparse_attn_impl(const oracle_shape *s, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                             const int64_t *rows, int64_t nrows, const uint32_t *sel_mask,
                             double *out, int64_t *n_keys, int causal)
{
    const int S = all_tokens(s), N = oracle_num_cubes(s);
    const int Hq = s->Hq, Hkv = s->Hkv, D = s->D, G = Hq / Hkv;
    const int words = ceil_div(N, 32);
    const double scale = 1.0 / sqrt((double)D);
    int32_t *cube_of = malloc(sizeof(int32_t) * S), *rank_of = malloc(sizeof(int32_t) * S);
    int32_t *size_of = malloc(sizeof(int32_t) * N);
    int64_t *start = malloc(sizeof(int64_t) * (N + 1));
    oracle_cube_map(s, cube_of, rank_of, size_of, start);

    #pragma omp parallel
    {
        double *q = malloc(sizeof(double) * D);
        double *logit = malloc(sizeof(double) * S);
        int32_t *key = malloc(sizeof(int32_t) * S);
        #pragma omp for schedule(dynamic, 8)
        for (int64_t x = 0; x < nrows; ++x) {
            const int64_t r = rows ? rows[x] : x;
            const int n = (int)(r / Hq), a = (int)(r % Hq), g = a / G;
            const int i = cube_of[n];
            const uint32_t *mrow = sel_mask + (size_t)x * words;
            for (int d = 0; d < D; ++d) q[d] = bf16_widen(Q[((size_t)n * Hq + a) * D + d]);
            /* the attended key set, as a list of token indices */
            int nk = 0;
            for (int m = 0; m < S; ++m) {
                const int c = cube_of[m];
                const int in_selected = (c != i) && ((mrow[c >> 5] >> (c & 31)) & 1u);
                const int in_own = (c == i) && (!causal || rank_of[m] <= rank_of[n]);
                if (in_selected || in_own) key[nk++] = m;
            }
            double mx = -INFINITY;
            for (int k = 0; k < nk; ++k) {
                double dot = 0.0;
                const uint16_t *kr = K + ((size_t)key[k] * Hkv + g) * D;
                for (int d = 0; d < D; ++d) dot += q[d] * bf16_widen(kr[d]);
                logit[k] = dot * scale;
                if (logit[k] > mx) mx = logit[k];
            }
            double Z = 0.0;
            double *o = out + (size_t)x * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int k = 0; k < nk; ++k) {
                const double e = exp(logit[k] - mx);
                const uint16_t *vr = V + ((size_t)key[k] * Hkv + g) * D;
                Z += e;
                for (int d = 0; d < D; ++d) o[d] += e * bf16_widen(vr[d]);
            }
            for (int d = 0; d < D; ++d) o[d] /= Z;
            if (n_keys) n_keys[x] = nk;
        }
        free(q); free(logit); free(key);
    }
    free(cube_of); free(rank_of); free(size_of); free(start);
}

void oracle_sparse_attn(const oracle_shape *s, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                        const int64_t *rows, int64_t nrows, const uint32_t *sel_mask,
                        double *out, int64_t *n_keys)
{
    sparse_attn_impl(s, Q, K, V, rows, nrows, sel_mask, out, n_keys, 1);
}

/* Non-causal mode (causal = 0 of the interface; the paper's operator is causal): the selected cubes may lie on
 * either side of the own cube, and the own cube is attended in full. */
void oracle_sparse_attn_noncausal(const oracle_shape *s, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                                  const int64_t *rows, int64_t nrows, const uint32_t *sel_mask,
                                  double *out, int64_t *n_keys)
{
    sparse_attn_impl(s, Q, K, V, rows, nrows, sel_mask, out, n_keys, 0);
}

/* ---------------------------------------------------------------------------
 * Dense causal attention in cube-major order (the comparison point; supp.
 * "Detail of FLOPs Calculation"): a query attends every token whose cube-major
 * position is <= its own.  Coded separately from oracle_sparse_attn (positions,
 * no masks) so that "p -> 1 equals dense" tests two independent loops.
 * ------------------------------------------------------------------------- */
static void dense_attn_impl(const oracle_shape *s, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                            const int64_t *rows, int64_t nrows, double *out, int causal)
{
    const int S = all_tokens(s), N = oracle_num_cubes(s);
    const int Hq = s->Hq, Hkv = s->Hkv, D = s->D, G = Hq / Hkv;
    const double scale = 1.0 / sqrt((double)D);
    int32_t *cube_of = malloc(sizeof(int32_t) * S), *rank_of = malloc(sizeof(int32_t) * S);
    int32_t *size_of = malloc(sizeof(int32_t) * N);
    int64_t *start = malloc(sizeof(int64_t) * (N + 1));
    int64_t *pos = malloc(sizeof(int64_t) * S);
    oracle_cube_map(s, cube_of, rank_of, size_of, start);
    for (int n = 0; n < S; ++n) pos[n] = start[cube_of[n]] + rank_of[n];

    #pragma omp parallel
    {
        double *w = malloc(sizeof(double) * S);
        #pragma omp for schedule(dynamic, 8)
        for (int64_t x = 0; x < nrows; ++x) {
            const int64_t r = rows ? rows[x] : x;
            const int n = (int)(r / Hq), a = (int)(r % Hq), g = a / G;
            const uint16_t *qr = Q + ((size_t)n * Hq + a) * D;
            double mx = -INFINITY;
            for (int m = 0; m < S; ++m) {
                if (causal && pos[m] > pos[n]) { w[m] = -INFINITY; continue; }
                double dot = 0.0;
                const uint16_t *kr = K + ((size_t)m * Hkv + g) * D;
                for (int d = 0; d < D; ++d) dot += bf16_widen(qr[d]) * bf16_widen(kr[d]);
                w[m] = dot * scale;
                if (w[m] > mx) mx = w[m];
            }
            double Z = 0.0;
            for (int m = 0; m < S; ++m) { w[m] = (causal && pos[m] > pos[n]) ? 0.0 : exp(w[m] - mx); Z += w[m]; }
            double *o = out + (size_t)x * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int m = 0; m < S; ++m) {
                if (causal && pos[m] > pos[n]) continue;
                const uint16_t *vr = V + ((size_t)m * Hkv + g) * D;
                for (int d = 0; d < D; ++d) o[d] += w[m] * bf16_widen(vr[d]);
            }
            for (int d = 0; d < D; ++d) o[d] /= Z;
        }
        free(w);
    }
    free(cube_of); free(rank_of); free(size_of); free(start); free(pos);
}

void oracle_dense_attn(const oracle_shape *s, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                       const int64_t *rows, int64_t nrows, double *out)
{
    dense_attn_impl(s, Q, K, V, rows, nrows, out, 1);
}

/* Plain bidirectional attention over all tokens: what the non-causal mode computes when every cube is selected. */
void oracle_dense_attn_noncausal(const oracle_shape *s, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                                 const int64_t *rows, int64_t nrows, double *out)
{
    dense_attn_impl(s, Q, K, V, rows, nrows, out, 0);
}

/* ---------------------------------------------------------------------------
 * Cube selection in non-causal mode (causal = 0 of the interface; the paper's
 * operator is causal, Eq. 1 lists the cubes before the own one).  The
 * candidates of Eqs. 1-2 are ALL video cubes other than the row's own cube;
 * every text cube other than the own one is attended and its bit set.  Same
 * outputs and near_cut rule as oracle_cube_select.
 * ------------------------------------------------------------------------- */
void oracle_cube_select_noncausal(const oracle_shape *s, const uint16_t *Q, const double *kbar, double p,
                                  const int64_t *rows, int64_t nrows,
                                  uint32_t *sel_mask, int32_t *sel_count, uint8_t *near_cut, double eps)
{
    const int S = all_tokens(s), N = oracle_num_cubes(s), Nv = oracle_num_video_cubes(s);
    const int Np = oracle_num_lead_cubes(s);
    const int Hq = s->Hq, Hkv = s->Hkv, D = s->D, G = Hq / Hkv;
    const int words = ceil_div(N, 32);
    int32_t *cube_of = malloc(sizeof(int32_t) * S), *rank_of = malloc(sizeof(int32_t) * S);
    int32_t *size_of = malloc(sizeof(int32_t) * N);
    int64_t *start = malloc(sizeof(int64_t) * (N + 1));
    oracle_cube_map(s, cube_of, rank_of, size_of, start);

    #pragma omp parallel
    {
        double *q = malloc(sizeof(double) * D);
        double *rowsbuf = malloc(sizeof(double) * (size_t)N * D);  /* the candidates' mean keys, gathered */
        double *logits = malloc(sizeof(double) * N), *probs = malloc(sizeof(double) * N);
        double *cum = malloc(sizeof(double) * N);
        uint8_t *keep = malloc(N);
        int32_t *order = malloc(sizeof(int32_t) * N), *cand = malloc(sizeof(int32_t) * N);
        #pragma omp for schedule(dynamic, 64)
        for (int64_t x = 0; x < nrows; ++x) {
            const int64_t r = rows ? rows[x] : x;
            const int n = (int)(r / Hq), a = (int)(r % Hq), g = a / G;
            const int own = cube_of[n];
            uint32_t *mrow = sel_mask + (size_t)x * words;
            for (int w = 0; w < words; ++w) mrow[w] = 0;
            sel_count[x] = 0;
            if (near_cut) near_cut[x] = 0;
            int nc = 0;
            for (int j = 0; j < N; ++j) {
                if (j == own) continue;
                if (j < Np || j >= Np + Nv) { mrow[j >> 5] |= (uint32_t)1 << (j & 31); sel_count[x] += 1; }
                else cand[nc++] = j;
            }
            if (nc == 0) continue;
            for (int d = 0; d < D; ++d) q[d] = bf16_widen(Q[((size_t)n * Hq + a) * D + d]);
            for (int c = 0; c < nc; ++c)
                for (int d = 0; d < D; ++d) rowsbuf[(size_t)c * D + d] = kbar[((size_t)cand[c] * Hkv + g) * D + d];
            oracle_relevance(q, rowsbuf, (int64_t)D, nc, D, logits, probs);
            const int kept = oracle_top_p(probs, nc, p, keep, order, cum);
            for (int c = 0; c < nc; ++c) if (keep[c]) mrow[cand[c] >> 5] |= (uint32_t)1 << (cand[c] & 31);
            sel_count[x] += kept;
            if (near_cut && p < 1.0 && p > 0.0) {
                int flag = 0;
                const double after = cum[kept - 1];
                const double before = kept >= 2 ? cum[kept - 2] : 0.0;
                if (after - p < eps || p - before < eps) flag = 1;
                if (kept < nc && logits[order[kept - 1]] - logits[order[kept]] < eps) flag = 1;
                if (kept >= 2 && logits[order[kept - 2]] - logits[order[kept - 1]] < eps) flag = 1;
                near_cut[x] = (uint8_t)flag;
            }
        }
        free(q); free(rowsbuf); free(logits); free(probs); free(cum); free(keep); free(order); free(cand);
    }
    free(cube_of); free(rank_of); free(size_of); free(start);
}

