// C ABI of the device entry points: argument checks, workspace carving, kernel selection.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "common.h"
#include "kernels.h"

namespace {

constexpr int kKnownFlags = CF_FLAG_SCALAR_KERNELS | CF_FLAG_DKV_SINGLE_WRITER;

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_fwd(const cf_attn_fwd_params *p, const char *who, bool sizes_only)
{
    if (!p) return cf::fail(CF_EINVAL, "%s: params is NULL", who);
    if (p->dtype != CF_BF16 && p->dtype != CF_FP32)
        return cf::fail(CF_EUNSUPPORTED, "%s: dtype %d not supported", who, p->dtype);
    if (p->head_dim != 64 && p->head_dim != 128)
        return cf::fail(CF_EUNSUPPORTED, "%s: head_dim %d not supported (64 or 128)", who, p->head_dim);
    if (p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_q_heads % p->n_kv_heads != 0)
        return cf::fail(CF_EINVAL, "%s: n_q_heads %d must be a positive multiple of n_kv_heads %d", who,
                        p->n_q_heads, p->n_kv_heads);
    if (p->n_q_heads > 65535) return cf::fail(CF_EINVAL, "%s: n_q_heads %d > 65535", who, p->n_q_heads);
    if (p->n_tokens < 1 || p->n_segments < 1 || p->n_kv_tokens < p->n_tokens)
        return cf::fail(CF_EINVAL, "%s: need n_tokens >= 1, n_segments >= 1, n_kv_tokens >= n_tokens (got %d, %d, %d)",
                        who, p->n_tokens, p->n_segments, p->n_kv_tokens);
    if (p->n_segments > p->n_tokens)
        return cf::fail(CF_EINVAL, "%s: n_segments %d > n_tokens %d (empty segments are not allowed)", who,
                        p->n_segments, p->n_tokens);
    if (sizes_only) return CF_OK;
    if (p->flags & ~kKnownFlags) return cf::fail(CF_EINVAL, "%s: unknown flags 0x%x", who, p->flags);
    if (!p->cu_seqlens_q || !p->cu_seqlens_k || !p->q || !p->k || !p->v || !p->o || !p->lse)
        return cf::fail(CF_EINVAL, "%s: NULL device pointer", who);
    if (!(p->softmax_scale == p->softmax_scale))
        return cf::fail(CF_EINVAL, "%s: softmax_scale is NaN", who);
    const int64_t vec = p->dtype == CF_BF16 ? 8 : 4;  // elements per 16-byte access
    const int64_t D = p->head_dim;
    const int64_t strides[] = {p->q_stride_tok, p->q_stride_head, p->kv_stride_tok, p->kv_stride_head,
                               p->o_stride_tok, p->o_stride_head};
    for (int64_t s : strides)
        if (s < D || s % vec != 0)
            return cf::fail(CF_EINVAL, "%s: stride %lld must be >= head_dim and a multiple of %lld elements", who,
                            (long long)s, (long long)vec);
    if (!aligned(p->q, 16) || !aligned(p->k, 16) || !aligned(p->v, 16) || !aligned(p->o, 16) ||
        !aligned(p->lse, 4) || !aligned(p->cu_seqlens_q, 4) || !aligned(p->cu_seqlens_k, 4))
        return cf::fail(CF_EINVAL, "%s: q, k, v, o must be 16-byte aligned", who);
    // the optional tile table: between ceil(T / 128) and T / 128 + n_segments records of 32 bytes
    if ((p->q_tiles == nullptr) != (p->n_q_tiles == 0) || p->n_q_tiles < 0 || !aligned(p->q_tiles, 16))
        return cf::fail(CF_EINVAL, "%s: q_tiles / n_q_tiles = %d do not go together (NULL with 0, 16-byte aligned)", who,
                        p->n_q_tiles);
    if (p->q_tiles && (p->n_q_tiles < (p->n_tokens + 127) / 128 || p->n_q_tiles > p->n_tokens / 128 + p->n_segments))
        return cf::fail(CF_EINVAL, "%s: n_q_tiles = %d cannot be the tile count of %d tokens in %d segments", who,
                        p->n_q_tiles, p->n_tokens, p->n_segments);
    return CF_OK;
}

// Shapes the MFMA kernels cover (decides the workspace size, so it may only look at sizes, dtype, flags).
bool mfma_shape(const cf_attn_fwd_params &p)
{
    return p.dtype == CF_BF16 && p.head_dim == 128 && !(p.flags & CF_FLAG_SCALAR_KERNELS);
}
// The MFMA kernels take the row maximum before scaling, which needs a positive scale.
bool use_mfma(const cf_attn_fwd_params &p) { return mfma_shape(p) && p.softmax_scale > 0.f; }

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

int64_t delta_bytes(const cf_attn_fwd_params &p) { return round_up((int64_t)p.n_q_heads * p.n_tokens * 4, 256); }
// counters (256 bytes) + two arrays of 16-byte items
int64_t worklist_bytes(const cf_attn_fwd_params &p)
{
    return mfma_shape(p) ? 256 + cf::dkv_worklist_capacity(p) * 16 : 0;
}

int hip_fail(const char *who, hipError_t e)
{
    return cf::fail(CF_EHIP, "%s: %s", who, hipGetErrorString(e));
}

thread_local cf::ProfileHook g_hook;

}  // namespace

cf::ProfileHook cf::take_profile_hook()
{
    cf::ProfileHook h = g_hook;
    g_hook = cf::ProfileHook();
    return h;
}

extern "C" int cf_profile_next_call(void *start_event, void *stop_event)
{
    g_hook.start = start_event && stop_event ? static_cast<hipEvent_t>(start_event) : nullptr;
    g_hook.stop = start_event && stop_event ? static_cast<hipEvent_t>(stop_event) : nullptr;
    return CF_OK;
}

extern "C" int cf_attn_fwd(const cf_attn_fwd_params *p, void *hip_stream)
{
    if (int rc = check_fwd(p, "cf_attn_fwd", false)) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = use_mfma(*p) ? cf::launch_mfma_fwd(*p, s) : cf::launch_simple_fwd(*p, s);
    return e == hipSuccess ? CF_OK : hip_fail("cf_attn_fwd", e);
}

extern "C" int64_t cf_attn_bwd_workspace_bytes(const cf_attn_fwd_params *p)
{
    if (int rc = check_fwd(p, "cf_attn_bwd_workspace_bytes", true)) return rc;
    if (p->flags & ~kKnownFlags)
        return cf::fail(CF_EINVAL, "cf_attn_bwd_workspace_bytes: unknown flags 0x%x", p->flags);
    return delta_bytes(*p) + worklist_bytes(*p);
}

namespace {

// Argument checks of one backward call apart from its scratch memory.
int check_bwd_tensors(const cf_attn_bwd_params *b, const char *who)
{
    if (!b) return cf::fail(CF_EINVAL, "%s: params is NULL", who);
    if (int rc = check_fwd(&b->f, who, false)) return rc;
    const cf_attn_fwd_params &p = b->f;
    if (!b->d_o || !b->d_q || !b->d_k || !b->d_v)
        return cf::fail(CF_EINVAL, "%s: NULL device pointer", who);
    const int64_t vec = p.dtype == CF_BF16 ? 8 : 4, D = p.head_dim;
    const int64_t strides[] = {b->do_stride_tok, b->do_stride_head, b->dq_stride_tok, b->dq_stride_head};
    for (int64_t s : strides)
        if (s < D || s % vec != 0)
            return cf::fail(CF_EINVAL, "%s: stride %lld must be >= head_dim and a multiple of %lld elements", who,
                            (long long)s, (long long)vec);
    if (b->dkv_stride_tok < D || b->dkv_stride_head < D || b->dkv_stride_tok % 4 || b->dkv_stride_head % 4)
        return cf::fail(CF_EINVAL, "%s: d_k/d_v strides must be >= head_dim and multiples of 4 elements", who);
    if (!aligned(b->d_o, 16) || !aligned(b->d_q, 16) || !aligned(b->d_k, 16) || !aligned(b->d_v, 16))
        return cf::fail(CF_EINVAL, "%s: d_o, d_q, d_k, d_v must be 16-byte aligned", who);
    return CF_OK;
}

// Lays the backward's scratch (delta, then the dK/dV work list) out in `bytes` bytes of device memory at `base`.
int carve_workspace(const cf_attn_fwd_params &p, void *base, int64_t bytes, const char *who, const char *what,
                    cf::BwdWorkspace *ws)
{
    if (!base || !aligned(base, 256)) return cf::fail(CF_EINVAL, "%s: %s must be non-NULL and 256-byte aligned", who, what);
    const int64_t need = delta_bytes(p) + worklist_bytes(p);
    if (bytes < need)
        return cf::fail(CF_EINVAL, "%s: %s has %lld bytes, %lld needed", who, what, (long long)bytes, (long long)need);
    ws->delta = static_cast<float *>(base);
    ws->worklist = mfma_shape(p) ? reinterpret_cast<int *>(static_cast<char *>(base) + delta_bytes(p)) : nullptr;
    ws->worklist_items = mfma_shape(p) ? cf::dkv_worklist_capacity(p) : 0;
    return CF_OK;
}

// Argument checks of one backward call; on success fills the scratch layout inside the caller's workspace.
int check_bwd(const cf_attn_bwd_params *b, const char *who, cf::BwdWorkspace *ws)
{
    if (int rc = check_bwd_tensors(b, who)) return rc;
    return carve_workspace(b->f, b->workspace, b->workspace_bytes, who, "workspace", ws);
}

int bwd_one(const cf_attn_bwd_params *b, const cf::BwdWorkspace &ws, hipStream_t s, const char *who)
{
    hipError_t e = hipSuccess;
    if (use_mfma(b->f)) {
        e = cf::launch_mfma_bwd(*b, ws, s);          // its dQ kernel forms delta itself
    } else {
        e = cf::launch_delta(*b, ws, s);
        if (e != hipSuccess) return hip_fail(who, e);
        e = cf::launch_simple_bwd(*b, ws, s);
    }
    return e == hipSuccess ? CF_OK : hip_fail(who, e);
}

// Heaviest first: the order in which the workgroups of a fused launch are dealt (work ~ queries x keys).
template <typename GetFwd>
void heaviest_first(int *order, int n, GetFwd fwd)
{
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order, order + n, [&](int a, int b) {
        return (int64_t)fwd(a).n_tokens * fwd(a).n_kv_tokens > (int64_t)fwd(b).n_tokens * fwd(b).n_kv_tokens;
    });
}

}  // namespace

extern "C" int cf_attn_bwd(const cf_attn_bwd_params *b, void *hip_stream)
{
    cf::BwdWorkspace ws;
    if (int rc = check_bwd(b, "cf_attn_bwd", &ws)) return rc;
    return bwd_one(b, ws, static_cast<hipStream_t>(hip_stream), "cf_attn_bwd");
}

// ---- the backward for callers that cannot allocate -------------------------------------------------------------
// The scratch of cf_attn_bwd_static: one array per GPU, part of the loaded code object, alive until the process
// ends.  Host code never uses the array's name as an address: the device address is looked up once per device
// (hipGetSymbolAddress with that device current) and kept in g_static_scratch.
static __device__ __align__(256) unsigned char scratch[CF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_static_scratch[kMaxDevices];

// Device address of `scratch` on the current device.
int static_scratch(const char *who, void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(who, e);
    if (dev < 0 || dev >= kMaxDevices) return cf::fail(CF_EUNSUPPORTED, "%s: device ordinal %d out of range", who, dev);
    void *ptr = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // (two threads racing here both get the same address from the runtime)
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(who, e);
        if (!ptr) return cf::fail(CF_EHIP, "%s: hipGetSymbolAddress returned a NULL address", who);
        g_static_scratch[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return CF_OK;
}
}  // namespace

extern "C" int cf_attn_bwd_static(const cf_attn_bwd_params *b, void *hip_stream)
{
    const char *who = "cf_attn_bwd_static";
    if (int rc = check_bwd_tensors(b, who)) return rc;
    // the size check comes before any HIP call: an oversized chunk is refused on any host
    const int64_t need = delta_bytes(b->f) + worklist_bytes(b->f);
    if (need > (int64_t)CF_STATIC_SCRATCH_BYTES)
        return cf::fail(CF_EINVAL, "%s: this chunk needs %lld bytes of scratch, the static buffer holds %lld "
                        "(use cf_attn_bwd with a workspace)", who, (long long)need, (long long)CF_STATIC_SCRATCH_BYTES);
    void *base = nullptr;
    if (int rc = static_scratch(who, &base)) return rc;
    cf::BwdWorkspace ws;
    if (int rc = carve_workspace(b->f, base, CF_STATIC_SCRATCH_BYTES, who, "static scratch", &ws)) return rc;
    return bwd_one(b, ws, static_cast<hipStream_t>(hip_stream), who);
}

extern "C" int cf_attn_fwd_batch(const cf_attn_fwd_params *params, int32_t n, void *hip_stream)
{
    const char *who = "cf_attn_fwd_batch";
    (void)cf::take_profile_hook();      // the hook times single-chunk calls only: an armed one ends here, unused
    if (n < 0 || (n > 0 && !params)) return cf::fail(CF_EINVAL, "%s: bad argument", who);
    for (int32_t i = 0; i < n; ++i)
        if (int rc = check_fwd(&params[i], who, false)) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int32_t i = 0;
    while (i < n) {
        // a run of chunks the MFMA kernel covers with the same head counts becomes one launch
        int32_t j = i;
        while (j < n && j - i < cf::CF_FWD_BATCH_MAX && use_mfma(params[j]) && params[j].n_q_heads == params[i].n_q_heads &&
               params[j].n_kv_heads == params[i].n_kv_heads)
            ++j;
        hipError_t e;
        if (j - i >= 2) {
            int order[cf::CF_FWD_BATCH_MAX];
            heaviest_first(order, j - i, [&](int a) -> const cf_attn_fwd_params & { return params[i + a]; });
            const cf_attn_fwd_params *chunks[cf::CF_FWD_BATCH_MAX];
            for (int a = 0; a < j - i; ++a) chunks[a] = &params[i + order[a]];
            e = cf::launch_mfma_fwd_batch(chunks, j - i, s);
        } else {
            j = i + 1;
            e = use_mfma(params[i]) ? cf::launch_mfma_fwd(params[i], s) : cf::launch_simple_fwd(params[i], s);
        }
        if (e != hipSuccess) return hip_fail(who, e);
        i = j;
    }
    return CF_OK;
}

extern "C" int cf_attn_bwd_batch(const cf_attn_bwd_params *params, int32_t n, void *hip_stream)
{
    const char *who = "cf_attn_bwd_batch";
    (void)cf::take_profile_hook();      // the hook times single-chunk calls only: an armed one ends here, unused
    if (n < 0 || (n > 0 && !params)) return cf::fail(CF_EINVAL, "%s: bad argument", who);
    std::vector<cf::BwdWorkspace> ws;
    try {
        ws.resize((size_t)n);
    } catch (const std::bad_alloc &) {
        return cf::fail(CF_ENOMEM, "%s: out of host memory", who);
    }
    for (int32_t i = 0; i < n; ++i)
        if (int rc = check_bwd(&params[i], who, &ws[i])) return rc;
    // the chunks of one call run interleaved: their workspaces must not overlap
    for (int32_t i = 0; i < n; ++i)
        for (int32_t j = i + 1; j < n; ++j) {
            const char *a = static_cast<const char *>(params[i].workspace), *b = static_cast<const char *>(params[j].workspace);
            if (a < b + params[j].workspace_bytes && b < a + params[i].workspace_bytes)
                return cf::fail(CF_EINVAL, "%s: chunks %d and %d share workspace memory", who, i, j);
        }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int32_t i = 0;
    while (i < n) {
        int32_t j = i;
        while (j < n && j - i < cf::CF_BWD_BATCH_MAX && use_mfma(params[j].f) && params[j].f.n_q_heads == params[i].f.n_q_heads &&
               params[j].f.n_kv_heads == params[i].f.n_kv_heads)
            ++j;
        if (j - i >= 2) {
            int order[cf::CF_BWD_BATCH_MAX];
            heaviest_first(order, j - i, [&](int a) -> const cf_attn_fwd_params & { return params[i + a].f; });
            const cf_attn_bwd_params *chunks[cf::CF_BWD_BATCH_MAX];
            for (int a = 0; a < j - i; ++a) chunks[a] = &params[i + a];
            const hipError_t e = cf::launch_mfma_bwd_batch(chunks, &ws[i], order, j - i, s);
            if (e != hipSuccess) return hip_fail(who, e);
        } else {
            j = i + 1;
            if (int rc = bwd_one(&params[i], ws[i], s, who)) return rc;
        }
        i = j;
    }
    return CF_OK;
}
