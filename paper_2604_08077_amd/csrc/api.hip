// extern "C" boundary of the library: argument validation and kernel enqueueing only.
#include <mutex>

#include "geom.h"
#include "ffn.h"

using namespace adaspark;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(const adaspark_shape *s)
{
    if (s == nullptr) return ADASPARK_EINVAL;
    if (s->frames <= 0 || s->height <= 0 || s->width <= 0) return ADASPARK_EINVAL;
    if (s->cube_t <= 0 || s->cube_h <= 0 || s->cube_w <= 0) return ADASPARK_EINVAL;
    if (s->q_heads <= 0 || s->kv_heads <= 0 || s->head_dim <= 0) return ADASPARK_EINVAL;
    if (s->q_heads % s->kv_heads != 0) return ADASPARK_EINVAL;
    if (s->text_tokens < 0 || s->prefix_tokens < 0) return ADASPARK_EINVAL;
    const long long tokens = (long long)s->frames * s->height * s->width + s->text_tokens + s->prefix_tokens;
    if (tokens * s->q_heads >= (1ll << 31)) return ADASPARK_EUNSUPPORTED;
    if (s->head_dim != 64 && s->head_dim != 128) return ADASPARK_EUNSUPPORTED;
    const long long cube = (long long)s->cube_t * s->cube_h * s->cube_w;
    if (cube >= (1ll << 24)) return ADASPARK_EUNSUPPORTED;
    const long long nt = (s->frames + (long long)s->cube_t - 1) / s->cube_t, nh = (s->height + (long long)s->cube_h - 1) / s->cube_h,
                    nw = (s->width + (long long)s->cube_w - 1) / s->cube_w;
    if (nt * nh * nw + (s->text_tokens + cube - 1) / cube + (s->prefix_tokens + cube - 1) / cube > ADASPARK_MAX_CUBES)
        return ADASPARK_EUNSUPPORTED;
    return ADASPARK_OK;
}

int check_ffn(const adaspark_shape *s, const adaspark_ffn_dims *d)
{
    const int rc = check_shape(s);
    if (rc != ADASPARK_OK) return rc;
    if (d == nullptr || d->d_model <= 0 || d->d_ff <= 0) return ADASPARK_EINVAL;
    if (d->d_model % 256 != 0 || d->d_model > 16384 || d->d_ff % 128 != 0 || d->d_ff > 65536) return ADASPARK_EUNSUPPORTED;
    if ((long long)s->cube_t * s->cube_h * s->cube_w > FFN_MAX_CUBE_TOKENS) return ADASPARK_EUNSUPPORTED;
    const long long tokens = (long long)s->frames * s->height * s->width + s->text_tokens + s->prefix_tokens;
    if (tokens * d->d_model >= (1ll << 30)) return ADASPARK_EUNSUPPORTED;
    return ADASPARK_OK;
}

// adaspark_sparse_attn_csr: the mask rows rebuilt from the compact list lie behind the packed K/V copy
size_t csr_mask_bytes(const Geom &g) { return ((size_t)g.S * g.Hq * g.words * 4 + 255) / 256 * 256; }

int check_ptrs(std::initializer_list<const void *> ps)
{
    for (const void *p : ps)
        if (p == nullptr || !aligned16(p)) return ADASPARK_EINVAL;
    return ADASPARK_OK;
}

}  // namespace

// Scratch memory of adaspark_cube_select_noalloc: the selection kernels' workspace (the three-term bf16 split of the
// mean keys and the tile sums of the compact list's scan) as a device array of the library itself, so that callers
// who cannot allocate need not bring a workspace.  One copy per GPU, held until the process ends; every call on a
// GPU uses that GPU's copy.  Host code never uses the array's name as an address: the device address is asked for
// once per device (static_scratch) and that pointer is what the kernels get.
constexpr size_t STATIC_SCRATCH_BYTES = ADASPARK_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static std::mutex scratch_lock;
static void *scratch_ptr[STATIC_SCRATCH_MAX_DEVICES] = {};

// The calling thread's current device's copy of `scratch`; nullptr (and *err set) if the runtime refuses.
static void *static_scratch(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

extern "C" {

int adaspark_num_cubes(const adaspark_shape *shape, int32_t *n_cubes)
{
    if (n_cubes == nullptr) return ADASPARK_EINVAL;
    const int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    *n_cubes = make_geom(*shape).N;
    return ADASPARK_OK;
}

int adaspark_workspace_bytes(const adaspark_shape *shape, int which_call, size_t *bytes)
{
    if (bytes == nullptr) return ADASPARK_EINVAL;
    const int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    const Geom g = make_geom(*shape);
    switch (which_call) {
    case ADASPARK_CALL_CUBE_POOL: *bytes = 0; return ADASPARK_OK;
    case ADASPARK_CALL_CUBE_SELECT: *bytes = select_workspace_bytes(g); return ADASPARK_OK;
    case ADASPARK_CALL_SPARSE_ATTN:
    case ADASPARK_CALL_DENSE_ATTN: *bytes = attn_workspace_bytes(g); return ADASPARK_OK;
    case ADASPARK_CALL_ATTN_BWD: *bytes = attn_bwd_workspace_bytes(g); return ADASPARK_OK;
    case ADASPARK_CALL_CUBE_SELECT_SHARED: *bytes = select_shared_workspace_bytes(g); return ADASPARK_OK;
    case ADASPARK_CALL_SPARSE_ATTN_CSR:  // (256 more: the mask rows start on a 256-byte boundary of the address)
        *bytes = (attn_workspace_bytes(g) + 255) / 256 * 256 + 256 + csr_mask_bytes(g);
        return ADASPARK_OK;
    default: return ADASPARK_EINVAL;
    }
}

int adaspark_select_status_offset(const adaspark_shape *shape, size_t *offset)
{
    if (offset == nullptr) return ADASPARK_EINVAL;
    const int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    *offset = select_status_offset(make_geom(*shape));
    return ADASPARK_OK;
}

int adaspark_pairs_workspace_bytes(const adaspark_shape *shape, int64_t max_selected, size_t *bytes)
{
    const int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if (bytes == nullptr || max_selected < 0) return ADASPARK_EINVAL;
    const Geom g = make_geom(*shape);
    if (!pairs_supported(g)) return ADASPARK_EUNSUPPORTED;
    // the scratch part starts at the next 256-byte boundary after the minimum workspace
    *bytes = attn_workspace_bytes(g) + 256 + pairs_scratch_bytes(g, (long long)max_selected);
    return ADASPARK_OK;
}

const char *adaspark_status_string(int status)
{
    switch (status) {
    case ADASPARK_OK: return "ok";
    case ADASPARK_EINVAL: return "invalid argument";
    case ADASPARK_EUNSUPPORTED: return "unsupported configuration";
    case ADASPARK_EWORKSPACE: return "workspace missing or too small";
    case ADASPARK_EHIP: return "HIP launch failed";
    case ADASPARK_ECAPACITY: return "compact list capacity exceeded";
    default: return "unknown status";
    }
}

int adaspark_cube_pool(const adaspark_shape *shape, const void *K, float *kbar, void *stream)
{
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({K, kbar})) != ADASPARK_OK) return rc;
    const Geom g = make_geom(*shape);
    const hipError_t e = launch_cube_pool(g, static_cast<const uint16_t *>(K), kbar, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

// top_k < 0: Top-p with threshold top_p; otherwise fixed Top-K
static int cube_select(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int top_k, int causal,
                       uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx, int64_t capacity,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({Q, kbar, sel_mask, sel_count})) != ADASPARK_OK) return rc;
    if ((row_ptr == nullptr) != (cube_idx == nullptr)) return ADASPARK_EINVAL;
    if (row_ptr != nullptr && (!aligned16(row_ptr) || !aligned16(cube_idx) || capacity < 0)) return ADASPARK_EINVAL;
    Geom g = make_geom(*shape);
    g.causal = causal != 0;
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < select_workspace_bytes(g))
        return ADASPARK_EWORKSPACE;
    const hipError_t e =
        launch_cube_select(g, static_cast<const uint16_t *>(Q), kbar, top_p, top_k, sel_mask, sel_count, row_ptr,
                           cube_idx, capacity, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

int adaspark_cube_select(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int causal,
                         uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                         int64_t capacity, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!(top_p >= 0.f && top_p <= 1.f)) return ADASPARK_EINVAL;  // also rejects NaN
    return cube_select(shape, Q, kbar, top_p, -1, causal, sel_mask, sel_count, row_ptr, cube_idx, capacity, workspace,
                       workspace_bytes, stream);
}

int adaspark_cube_select_noalloc(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int causal,
                                 uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                                 int64_t capacity, void *stream)
{
    if (!(top_p >= 0.f && top_p <= 1.f)) return ADASPARK_EINVAL;
    const int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    // a workspace that does not fit the library's own array: said before anything is asked of the runtime
    if (select_workspace_bytes(make_geom(*shape)) > STATIC_SCRATCH_BYTES) return ADASPARK_EWORKSPACE;
    hipError_t err = hipSuccess;
    void *ws = static_scratch(&err);
    if (ws == nullptr) return ADASPARK_EHIP;
    return cube_select(shape, Q, kbar, top_p, -1, causal, sel_mask, sel_count, row_ptr, cube_idx, capacity, ws,
                       STATIC_SCRATCH_BYTES, stream);
}

int adaspark_cube_select_topk(const adaspark_shape *shape, const void *Q, const float *kbar, int32_t top_k, int causal,
                              uint32_t *sel_mask, int32_t *sel_count, int64_t *row_ptr, int32_t *cube_idx,
                              int64_t capacity, void *workspace, size_t workspace_bytes, void *stream)
{
    if (top_k < 0) return ADASPARK_EINVAL;
    return cube_select(shape, Q, kbar, 0.f, top_k, causal, sel_mask, sel_count, row_ptr, cube_idx, capacity, workspace,
                       workspace_bytes, stream);
}

int adaspark_cube_select_shared(const adaspark_shape *shape, const void *Q, const float *kbar, float top_p, int causal,
                                uint32_t *sel_mask, int32_t *sel_count, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    if (!(top_p >= 0.f && top_p <= 1.f)) return ADASPARK_EINVAL;  // also rejects NaN
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({Q, kbar, sel_mask, sel_count})) != ADASPARK_OK) return rc;
    Geom g = make_geom(*shape);
    g.causal = causal != 0;
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < select_shared_workspace_bytes(g))
        return ADASPARK_EWORKSPACE;
    const hipError_t e = launch_cube_select_shared(g, static_cast<const uint16_t *>(Q), kbar, top_p, sel_mask, sel_count,
                                                   workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

static int attn_check(const adaspark_shape *shape, const void *Q, const uint32_t *sel_mask, bool sparse, int causal,
                      void *O, float *lse)
{
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({Q, O})) != ADASPARK_OK) return rc;
    if (sparse && (sel_mask == nullptr || !aligned16(sel_mask))) return ADASPARK_EINVAL;
    if (lse != nullptr && !aligned16(lse)) return ADASPARK_EINVAL;
    (void)causal;  // both modes are implemented (non-causal: by the masked-walk / dense kernel only)
    return ADASPARK_OK;
}

static int workspace_check(const Geom &g, const void *workspace, size_t workspace_bytes)
{
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < attn_workspace_bytes(g))
        return ADASPARK_EWORKSPACE;
    return ADASPARK_OK;
}

int adaspark_kv_pack(const adaspark_shape *shape, const void *K, const void *V, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({K, V})) != ADASPARK_OK) return rc;
    const Geom g = make_geom(*shape);
    if ((rc = workspace_check(g, workspace, workspace_bytes)) != ADASPARK_OK) return rc;
    const hipError_t e = launch_kv_pack(g, static_cast<const uint16_t *>(K), static_cast<const uint16_t *>(V), workspace,
                                        true, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

// skip: bytes behind the minimum workspace (rounded up to 256) that are not scratch memory (the CSR entry keeps its
// mask rows there)
static int attn_packed(const adaspark_shape *shape, const void *Q, void *packed, size_t packed_bytes,
                       const uint32_t *sel_mask, bool sparse, int sparse_kernel, int causal, void *O, float *lse,
                       void *stream, size_t skip = 0)
{
    int rc = attn_check(shape, Q, sel_mask, sparse, causal, O, lse);
    if (rc != ADASPARK_OK) return rc;
    if (sparse_kernel != ADASPARK_SPARSE_AUTO && sparse_kernel != ADASPARK_SPARSE_COMPACT &&
        sparse_kernel != ADASPARK_SPARSE_MASKED && sparse_kernel != ADASPARK_SPARSE_PAIRS)
        return ADASPARK_EINVAL;
    if (!causal && sparse && (sparse_kernel == ADASPARK_SPARSE_COMPACT || sparse_kernel == ADASPARK_SPARSE_PAIRS))
        return ADASPARK_EUNSUPPORTED;  // those two kernels walk the cubes before the own one only
    Geom g = make_geom(*shape);
    g.causal = causal != 0;
    if ((rc = workspace_check(g, packed, packed_bytes)) != ADASPARK_OK) return rc;
    // whatever lies beyond the minimum workspace, from the next 256-byte boundary on, is scratch memory
    const uintptr_t begin = reinterpret_cast<uintptr_t>(packed);
    const uintptr_t sbegin = ((begin + attn_workspace_bytes(g) + 255) & ~static_cast<uintptr_t>(255)) + skip;
    void *scratch = nullptr;
    size_t scratch_bytes = 0;
    if (sparse && begin + packed_bytes > sbegin) {
        scratch = reinterpret_cast<void *>(sbegin);
        scratch_bytes = begin + packed_bytes - sbegin;
    }
    if (sparse && sparse_kernel == ADASPARK_SPARSE_PAIRS) {
        if (!pairs_supported(g)) return ADASPARK_EUNSUPPORTED;
        if (scratch_bytes < pairs_scratch_bytes(g, 0)) return ADASPARK_EWORKSPACE;
    }
    const hipError_t e = launch_attn(g, static_cast<const uint16_t *>(Q), packed, sparse ? sel_mask : nullptr, sparse_kernel,
                                     scratch, scratch_bytes, static_cast<uint16_t *>(O), lse,
                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

int adaspark_sparse_attn_packed(const adaspark_shape *shape, const void *Q, void *packed, size_t packed_bytes,
                                const uint32_t *sel_mask, int causal, void *O, float *lse, void *stream)
{
    return attn_packed(shape, Q, packed, packed_bytes, sel_mask, true, ADASPARK_SPARSE_AUTO, causal, O, lse, stream);
}

int adaspark_sparse_attn_packed_with(const adaspark_shape *shape, const void *Q, void *packed, size_t packed_bytes,
                                     const uint32_t *sel_mask, int causal, int sparse_kernel, void *O, float *lse,
                                     void *stream)
{
    return attn_packed(shape, Q, packed, packed_bytes, sel_mask, true, sparse_kernel, causal, O, lse, stream);
}

int adaspark_dense_attn_packed(const adaspark_shape *shape, const void *Q, const void *packed, size_t packed_bytes,
                               int causal, void *O, float *lse, void *stream)
{
    // the dense kernel only reads the workspace
    return attn_packed(shape, Q, const_cast<void *>(packed), packed_bytes, nullptr, false, ADASPARK_SPARSE_AUTO, causal, O,
                       lse, stream);
}

static int attn_full(const adaspark_shape *shape, const void *Q, const void *K, const void *V,
                     const uint32_t *sel_mask, bool sparse, int causal, void *O, float *lse, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    // validate everything before the first launch
    int rc = attn_check(shape, Q, sel_mask, sparse, causal, O, lse);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({K, V})) != ADASPARK_OK) return rc;
    if ((rc = workspace_check(make_geom(*shape), workspace, workspace_bytes)) != ADASPARK_OK) return rc;
    if ((rc = adaspark_kv_pack(shape, K, V, workspace, workspace_bytes, stream)) != ADASPARK_OK) return rc;
    return attn_packed(shape, Q, workspace, workspace_bytes, sel_mask, sparse, ADASPARK_SPARSE_AUTO, causal, O, lse, stream);
}

int adaspark_sparse_attn(const adaspark_shape *shape, const void *Q, const void *K, const void *V,
                         const uint32_t *sel_mask, int causal, void *O, float *lse, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    return attn_full(shape, Q, K, V, sel_mask, true, causal, O, lse, workspace, workspace_bytes, stream);
}

int adaspark_sparse_attn_csr(const adaspark_shape *shape, const void *Q, const void *K, const void *V,
                             const int64_t *row_ptr, const int32_t *cube_idx, int causal, void *O, float *lse,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({Q, K, V, O, row_ptr, cube_idx})) != ADASPARK_OK) return rc;
    if (lse != nullptr && !aligned16(lse)) return ADASPARK_EINVAL;
    const Geom g = make_geom(*shape);
    // the mask rows start at the first 256-byte boundary (of the address) behind the minimum workspace
    const uintptr_t begin = reinterpret_cast<uintptr_t>(workspace);
    const uintptr_t mbegin = (begin + attn_workspace_bytes(g) + 255) & ~static_cast<uintptr_t>(255);
    const size_t mbytes = csr_mask_bytes(g);
    if (workspace == nullptr || !aligned16(workspace) || begin + workspace_bytes < mbegin + mbytes)
        return ADASPARK_EWORKSPACE;
    uint32_t *mask = reinterpret_cast<uint32_t *>(mbegin);
    if ((rc = adaspark_kv_pack(shape, K, V, workspace, workspace_bytes, stream)) != ADASPARK_OK) return rc;
    launch_mask_from_csr(g, row_ptr, cube_idx, mask, static_cast<hipStream_t>(stream));
    if (hipGetLastError() != hipSuccess) return ADASPARK_EHIP;
    // (what lies behind the mask rows is scratch memory for the key-stationary kernel, as in the mask-fed entry)
    return attn_packed(shape, Q, workspace, workspace_bytes, mask, true, ADASPARK_SPARSE_AUTO, causal, O, lse, stream,
                       mbytes);
}

int adaspark_dense_attn(const adaspark_shape *shape, const void *Q, const void *K, const void *V, int causal, void *O,
                        float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    return attn_full(shape, Q, K, V, nullptr, false, causal, O, lse, workspace, workspace_bytes, stream);
}

int adaspark_sparse_attn_bwd(const adaspark_shape *shape, const void *Q, const void *K, const void *V, const void *O,
                             const float *lse, const void *dO, const uint32_t *sel_mask, int causal, void *dQ,
                             void *dK, void *dV, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({Q, K, V, O, lse, dO, dQ, dK, dV})) != ADASPARK_OK) return rc;
    if (sel_mask != nullptr && !aligned16(sel_mask)) return ADASPARK_EINVAL;
    if (!causal) return ADASPARK_EUNSUPPORTED;
    const Geom g = make_geom(*shape);
    if ((long long)g.S * g.Hq * g.words >= (1ll << 30)) return ADASPARK_EUNSUPPORTED;
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < attn_bwd_workspace_bytes(g))
        return ADASPARK_EWORKSPACE;
    const hipError_t e = launch_attn_bwd(g, static_cast<const uint16_t *>(Q), static_cast<const uint16_t *>(K),
                                         static_cast<const uint16_t *>(V), static_cast<const uint16_t *>(O), lse,
                                         static_cast<const uint16_t *>(dO), sel_mask, static_cast<uint16_t *>(dQ),
                                         static_cast<uint16_t *>(dK), static_cast<uint16_t *>(dV), workspace,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

int adaspark_ffn_workspace_bytes(const adaspark_shape *shape, const adaspark_ffn_dims *dims, size_t *bytes)
{
    const int rc = check_ffn(shape, dims);
    if (rc != ADASPARK_OK) return rc;
    if (bytes == nullptr) return ADASPARK_EINVAL;
    *bytes = ffn_workspace(make_geom(*shape), dims->d_model, dims->d_ff, nullptr).bytes;
    return ADASPARK_OK;
}

int adaspark_ffn_select(const adaspark_shape *shape, const adaspark_ffn_dims *dims, const void *X, float top_p,
                        float eps, uint8_t *keep, float *score, int32_t *keep_count, void *stream)
{
    int rc = check_ffn(shape, dims);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({X, keep})) != ADASPARK_OK) return rc;
    if ((score != nullptr && !aligned16(score)) || (keep_count != nullptr && !aligned16(keep_count))) return ADASPARK_EINVAL;
    if (!(top_p >= 0.0f && top_p <= 1.0f) || !(eps >= 0.0f) || eps > 3.0e38f) return ADASPARK_EINVAL;
    const hipError_t e = launch_ffn_select(make_geom(*shape), dims->d_model, static_cast<const uint16_t *>(X), top_p, eps,
                                           keep, score, keep_count, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

int adaspark_ffn_sparse(const adaspark_shape *shape, const adaspark_ffn_dims *dims, const void *X, const void *W_gate,
                        const void *W_up, const void *W_down, const uint8_t *keep, void *Y, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    int rc = check_ffn(shape, dims);
    if (rc != ADASPARK_OK) return rc;
    if ((rc = check_ptrs({X, W_gate, W_up, W_down, Y})) != ADASPARK_OK) return rc;
    if (keep != nullptr && !aligned16(keep)) return ADASPARK_EINVAL;
    const Geom g = make_geom(*shape);
    {   // Y must not overlap X at all: the mean compensation reads X rows of other tokens while Y is written
        const uintptr_t x0 = reinterpret_cast<uintptr_t>(X), y0 = reinterpret_cast<uintptr_t>(Y);
        const uintptr_t n = (uintptr_t)g.S * (uintptr_t)dims->d_model * 2u;
        if (x0 < y0 + n && y0 < x0 + n) return ADASPARK_EINVAL;
    }
    if (workspace == nullptr || !aligned16(workspace) ||
        workspace_bytes < ffn_workspace(g, dims->d_model, dims->d_ff, nullptr).bytes)
        return ADASPARK_EWORKSPACE;
    const hipError_t e = launch_ffn_sparse(g, dims->d_model, dims->d_ff, static_cast<const uint16_t *>(X),
                                           static_cast<const uint16_t *>(W_gate), static_cast<const uint16_t *>(W_up),
                                           static_cast<const uint16_t *>(W_down), keep, static_cast<uint16_t *>(Y), workspace,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ADASPARK_OK : ADASPARK_EHIP;
}

}  // extern "C"
