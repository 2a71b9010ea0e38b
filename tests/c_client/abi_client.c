/*
 * A plain C99 client of the library: nothing but adaspark.h and the HIP runtime API.  It runs the hot path
 * (mean keys, Top-p selection, sparse attention, dense attention) on a small seeded problem through the C ABI and
 * checks what comes back against a brute-force loop of its own:
 *   - Eq. 1: mean keys against a direct mean over each cube's tokens,
 *   - Eq. 2 invariants: top_p = 1 selects every preceding cube; at top_p = 0.6 the counts equal the set bits, no
 *     own or later cube is set, and the kept mass (recomputed here in double) reaches top_p and is minimal,
 *   - Eq. 3: the sparse entry on the produced selection and the dense entry against two-pass softmax attention in
 *     double over the attended tokens in cube-major causal order,
 *   - the compact list fed to adaspark_sparse_attn_csr gives the mask-fed output bit for bit.
 * Exit status 0 and "abi_client: OK" on success.  Built by the package's build step; run by tests/test_gpu_c_client.py.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adaspark.h"

#define CHECK_HIP(x)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__);     \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define CHECK_ADA(x)                                                                     \
    do {                                                                                 \
        int s_ = (x);                                                                    \
        if (s_ != ADASPARK_OK) {                                                         \
            fprintf(stderr, "%s at %s:%d\n", adaspark_status_string(s_), __FILE__, __LINE__); \
            return 3;                                                                    \
        }                                                                                \
    } while (0)
#define FAIL(...)                                                                        \
    do {                                                                                 \
        fprintf(stderr, "abi_client: FAILED: " __VA_ARGS__);                             \
        fprintf(stderr, "\n");                                                           \
        return 1;                                                                        \
    } while (0)

/* grid 6 x 8 x 10 tokens, cubes of 2 x 4 x 4 (the last column of cubes is clipped to width 2), 6 query heads on 2 KV heads */
enum { T = 6, H = 8, W = 10, CT = 2, CH = 4, CW = 4, HQ = 6, HKV = 2, D = 64, S = T * H * W, R = S * HQ, G = HQ / HKV };

static uint32_t lcg_state = 20260408u;
static float uniform_pm1(void)
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)((lcg_state >> 8) & 0xffffff) / 8388608.0f - 1.0f;
}
static uint16_t to_bf16(float x) /* round to nearest even */
{
    uint32_t u;
    memcpy(&u, &x, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static double from_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float x;
    memcpy(&x, &u, 4);
    return (double)x;
}

static int cube_of[S], rank_of[S], n_cubes;

static void build_cube_map(void)
{
    const int nh = (H + CH - 1) / CH, nw = (W + CW - 1) / CW;
    static int fill[64];
    n_cubes = ((T + CT - 1) / CT) * nh * nw;
    memset(fill, 0, sizeof fill);
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h)
            for (int w = 0; w < W; ++w) {
                const int n = (t * H + h) * W + w;
                cube_of[n] = ((t / CT) * nh + h / CH) * nw + w / CW;
            }
    /* rank: local raster order inside the cube = order of increasing n among the cube's tokens */
    for (int n = 0; n < S; ++n) rank_of[n] = fill[cube_of[n]]++;
}

/* does key token m precede (or equal) query token n in cube-major causal order? */
static int precedes(int m, int n)
{
    return cube_of[m] < cube_of[n] || (cube_of[m] == cube_of[n] && rank_of[m] <= rank_of[n]);
}

int main(void)
{
    int n_dev = 0;
    CHECK_HIP(hipGetDeviceCount(&n_dev));
    if (n_dev < 1) FAIL("no GPU");
    build_cube_map();
    const adaspark_shape shape = {T, H, W, CT, CH, CW, HQ, HKV, D, 0, 0};
    int32_t nc = 0;
    CHECK_ADA(adaspark_num_cubes(&shape, &nc));
    if (nc != n_cubes) FAIL("cube count %d, expected %d", (int)nc, n_cubes);
    const int words = (nc + 31) / 32;

    /* inputs */
    static uint16_t q[R * D], k[S * HKV * D], v[S * HKV * D];
    for (int x = 0; x < R * D; ++x) q[x] = to_bf16(2.0f * uniform_pm1());
    for (int x = 0; x < S * HKV * D; ++x) k[x] = to_bf16(2.0f * uniform_pm1() + 0.5f * (float)(cube_of[x / (HKV * D)] % 3));
    for (int x = 0; x < S * HKV * D; ++x) v[x] = to_bf16(uniform_pm1());

    void *dq, *dk, *dv, *dO, *dO2, *dws_sel, *dws_att;
    float *dkbar, *dlse;
    uint32_t *dmask;
    int32_t *dcount, *dcidx;
    int64_t *drptr;
    size_t ws_sel = 0, ws_att = 0, ws_dense = 0, ws_csr = 0;
    CHECK_ADA(adaspark_workspace_bytes(&shape, ADASPARK_CALL_CUBE_SELECT, &ws_sel));
    CHECK_ADA(adaspark_workspace_bytes(&shape, ADASPARK_CALL_SPARSE_ATTN, &ws_att));
    CHECK_ADA(adaspark_workspace_bytes(&shape, ADASPARK_CALL_DENSE_ATTN, &ws_dense));
    CHECK_ADA(adaspark_workspace_bytes(&shape, ADASPARK_CALL_SPARSE_ATTN_CSR, &ws_csr));
    if (ws_dense > ws_att) ws_att = ws_dense;
    if (ws_csr > ws_att) ws_att = ws_csr;
    const int64_t capacity = (int64_t)R * nc;
    CHECK_HIP(hipMalloc(&dq, sizeof q));
    CHECK_HIP(hipMalloc(&dk, sizeof k));
    CHECK_HIP(hipMalloc(&dv, sizeof v));
    CHECK_HIP(hipMalloc(&dO, sizeof q));
    CHECK_HIP(hipMalloc(&dO2, sizeof q));
    CHECK_HIP(hipMalloc((void **)&dkbar, (size_t)nc * HKV * D * 4));
    CHECK_HIP(hipMalloc((void **)&dlse, (size_t)R * 4));
    CHECK_HIP(hipMalloc((void **)&dmask, (size_t)R * words * 4));
    CHECK_HIP(hipMalloc((void **)&dcount, (size_t)R * 4));
    CHECK_HIP(hipMalloc((void **)&drptr, (size_t)(R + 1) * 8));
    CHECK_HIP(hipMalloc((void **)&dcidx, (size_t)capacity * 4));
    CHECK_HIP(hipMalloc(&dws_sel, ws_sel));
    CHECK_HIP(hipMalloc(&dws_att, ws_att));
    CHECK_HIP(hipMemcpy(dq, q, sizeof q, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dk, k, sizeof k, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dv, v, sizeof v, hipMemcpyHostToDevice));

    /* ---- Eq. 1 */
    CHECK_ADA(adaspark_cube_pool(&shape, dk, dkbar, NULL));
    static float kbar[64 * HKV * D];
    CHECK_HIP(hipMemcpy(kbar, dkbar, (size_t)nc * HKV * D * 4, hipMemcpyDeviceToHost));
    static double kbar_ref[64 * HKV * D];
    static int csize[64];
    memset(kbar_ref, 0, sizeof kbar_ref);
    memset(csize, 0, sizeof csize);
    for (int n = 0; n < S; ++n) {
        ++csize[cube_of[n]];
        for (int x = 0; x < HKV * D; ++x) kbar_ref[cube_of[n] * HKV * D + x] += from_bf16(k[n * HKV * D + x]);
    }
    for (int c = 0; c < nc; ++c)
        for (int x = 0; x < HKV * D; ++x) {
            const double want = kbar_ref[c * HKV * D + x] / csize[c];
            kbar_ref[c * HKV * D + x] = want;
            if (fabs((double)kbar[c * HKV * D + x] - want) > 1e-5) FAIL("mean key of cube %d off by %g", c, fabs(kbar[c * HKV * D + x] - want));
        }

    /* ---- Eq. 2, top_p = 1: every preceding cube */
    static uint32_t mask[R * 2];
    static int32_t count[R];
    CHECK_ADA(adaspark_cube_select(&shape, dq, dkbar, 1.0f, 1, dmask, dcount, NULL, NULL, 0, dws_sel, ws_sel, NULL));
    CHECK_HIP(hipMemcpy(mask, dmask, (size_t)R * words * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(count, dcount, (size_t)R * 4, hipMemcpyDeviceToHost));
    for (int r = 0; r < R; ++r) {
        const int i = cube_of[r / HQ];
        if (count[r] != i) FAIL("top_p = 1: row %d keeps %d of %d cubes", r, (int)count[r], i);
        for (int j = 0; j < nc; ++j)
            if ((int)((mask[r * words + (j >> 5)] >> (j & 31)) & 1u) != (j < i)) FAIL("top_p = 1: row %d, bit of cube %d", r, j);
    }

    /* ---- Eq. 2, top_p = 0.6, with the compact list */
    const float top_p = 0.6f;
    CHECK_ADA(adaspark_cube_select(&shape, dq, dkbar, top_p, 1, dmask, dcount, drptr, dcidx, capacity, dws_sel, ws_sel, NULL));
    CHECK_HIP(hipMemcpy(mask, dmask, (size_t)R * words * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(count, dcount, (size_t)R * 4, hipMemcpyDeviceToHost));
    size_t status_off = 0;
    int32_t status = 1;
    CHECK_ADA(adaspark_select_status_offset(&shape, &status_off));
    CHECK_HIP(hipMemcpy(&status, (char *)dws_sel + status_off, 4, hipMemcpyDeviceToHost));
    if (status != ADASPARK_OK) FAIL("status word %d", (int)status);
    int boundary_rows = 0;
    for (int r = 0; r < R; ++r) {
        const int n = r / HQ, a = r % HQ, i = cube_of[n], g = a / G;
        int bits = 0;
        double prob[64], z = 0.0, mx = -1e300, kept = 0.0, least = 1e300;
        for (int j = 0; j < nc; ++j) {
            const int b = (int)((mask[r * words + (j >> 5)] >> (j & 31)) & 1u);
            if (b && j >= i) FAIL("row %d keeps cube %d, not before its own (%d)", r, j, i);
            bits += b;
        }
        if (bits != count[r]) FAIL("row %d: count %d, set bits %d", r, (int)count[r], bits);
        if (i == 0) continue;
        for (int j = 0; j < i; ++j) {
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += from_bf16(q[r * D + d]) * kbar_ref[(j * HKV + g) * D + d];
            prob[j] = dot / sqrt((double)D);
            if (prob[j] > mx) mx = prob[j];
        }
        for (int j = 0; j < i; ++j) { prob[j] = exp(prob[j] - mx); z += prob[j]; }
        for (int j = 0; j < i; ++j)
            if ((mask[r * words + (j >> 5)] >> (j & 31)) & 1u) {
                kept += prob[j] / z;
                if (prob[j] / z < least) least = prob[j] / z;
            }
        /* the nucleus: mass reaches top_p, and would not without its least member (up to float32 resolution of the sums) */
        if (kept < top_p - 1e-5) FAIL("row %d keeps mass %g < %g", r, kept, (double)top_p);
        if (kept - least >= top_p + 1e-5) FAIL("row %d: the kept set is not minimal (%g without its least member)", r, kept - least);
        for (int j = 0; j < i; ++j) /* no cube left out that outweighs a kept one */
            if (!((mask[r * words + (j >> 5)] >> (j & 31)) & 1u) && prob[j] / z > least * (1.0 + 1e-5)) FAIL("row %d skips cube %d above a kept one", r, j);
        if (fabs(kept - top_p) < 1e-4 || fabs(kept - least - top_p) < 1e-4) ++boundary_rows;
    }

    /* ---- Eq. 3 on that selection, the same from the compact list, and the dense entry */
    static uint16_t o_sparse[R * D], o_csr[R * D], o_dense[R * D];
    static float lse[R];
    CHECK_ADA(adaspark_sparse_attn(&shape, dq, dk, dv, dmask, 1, dO, dlse, dws_att, ws_att, NULL));
    CHECK_HIP(hipMemcpy(o_sparse, dO, sizeof o_sparse, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(lse, dlse, sizeof lse, hipMemcpyDeviceToHost));
    CHECK_ADA(adaspark_sparse_attn_csr(&shape, dq, dk, dv, drptr, dcidx, 1, dO2, NULL, dws_att, ws_att, NULL));
    CHECK_HIP(hipMemcpy(o_csr, dO2, sizeof o_csr, hipMemcpyDeviceToHost));
    if (memcmp(o_sparse, o_csr, sizeof o_sparse) != 0) FAIL("list-fed and mask-fed attention differ");
    CHECK_ADA(adaspark_dense_attn(&shape, dq, dk, dv, 1, dO, NULL, dws_att, ws_att, NULL));
    CHECK_HIP(hipMemcpy(o_dense, dO, sizeof o_dense, hipMemcpyDeviceToHost));
    double worst_sparse = 0.0, worst_dense = 0.0, worst_lse = 0.0;
    static double sc[S], acc_s[D], acc_d[D];
    for (int r = 0; r < R; ++r) {
        const int n = r / HQ, a = r % HQ, i = cube_of[n], g = a / G;
        double mx_s = -1e300, mx_d = -1e300, z_s = 0.0, z_d = 0.0;
        for (int m = 0; m < S; ++m) {
            sc[m] = 0.0;
            if (!precedes(m, n)) continue;
            for (int d = 0; d < D; ++d) sc[m] += from_bf16(q[r * D + d]) * from_bf16(k[(m * HKV + g) * D + d]);
            sc[m] /= sqrt((double)D);
            const int j = cube_of[m];
            const int sel = j == i || ((mask[r * words + (j >> 5)] >> (j & 31)) & 1u);
            if (sc[m] > mx_d) mx_d = sc[m];
            if (sel && sc[m] > mx_s) mx_s = sc[m];
        }
        memset(acc_s, 0, sizeof acc_s);
        memset(acc_d, 0, sizeof acc_d);
        for (int m = 0; m < S; ++m) {
            if (!precedes(m, n)) continue;
            const int j = cube_of[m];
            const int sel = j == i || ((mask[r * words + (j >> 5)] >> (j & 31)) & 1u);
            const double pd = exp(sc[m] - mx_d), ps = sel ? exp(sc[m] - mx_s) : 0.0;
            z_d += pd;
            z_s += ps;
            for (int d = 0; d < D; ++d) {
                const double vv = from_bf16(v[(m * HKV + g) * D + d]);
                acc_d[d] += pd * vv;
                acc_s[d] += ps * vv;
            }
        }
        for (int d = 0; d < D; ++d) {
            const double es = fabs(from_bf16(o_sparse[r * D + d]) - acc_s[d] / z_s);
            const double ed = fabs(from_bf16(o_dense[r * D + d]) - acc_d[d] / z_d);
            if (es > worst_sparse) worst_sparse = es;
            if (ed > worst_dense) worst_dense = ed;
        }
        const double el = fabs((double)lse[r] - (mx_s + log(z_s)));
        if (el > worst_lse) worst_lse = el;
    }
    printf("abi_client: rows %d, cubes %d, rows at the nucleus boundary %d; max-abs error sparse %.3e dense %.3e lse %.3e\n", R,
           (int)nc, boundary_rows, worst_sparse, worst_dense, worst_lse);
    if (worst_sparse > 2e-2 || worst_dense > 2e-2) FAIL("attention output beyond 2e-2");
    if (worst_lse > 5e-2) FAIL("log-sum-exp beyond 5e-2");

    /* ---- error paths: nothing is launched, a status comes back */
    if (adaspark_cube_pool(&shape, NULL, dkbar, NULL) != ADASPARK_EINVAL) FAIL("null pointer accepted");
    if (adaspark_sparse_attn(&shape, dq, dk, dv, dmask, 1, dO, NULL, dws_att, 16, NULL) != ADASPARK_EWORKSPACE) FAIL("short workspace accepted");

    hipFree(dq); hipFree(dk); hipFree(dv); hipFree(dO); hipFree(dO2); hipFree(dkbar); hipFree(dlse); hipFree(dmask);
    hipFree(dcount); hipFree(drptr); hipFree(dcidx); hipFree(dws_sel); hipFree(dws_att);
    printf("abi_client: OK\n");
    return 0;
}
