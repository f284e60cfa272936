// C ABI entry points that touch the GPU: plan upload, the planned launches and the one-shot forms.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pv_plan.h"

namespace pv {
hipError_t launch_kv_append(const pv_plan *plan, const DeviceLists &dl, const void *k_new,
                            const void *v_new, const int32_t *page_table, void *k_pages,
                            void *v_pages, hipStream_t stream);
hipError_t launch_attn_narrow(const pv_plan *plan, const DeviceLists &dl, const void *q,
                              const void *k_pages, const void *v_pages,
                              const int32_t *page_table, float scale, void *out, float *ws_o,
                              float *ws_ml, hipStream_t stream);
hipError_t launch_attn_wide(const pv_plan *plan, const DeviceLists &dl, const void *q,
                            const void *k_pages, const void *v_pages, const int32_t *page_table,
                            float scale, void *out, float *ws_o, float *ws_ml,
                            hipStream_t stream);
hipError_t launch_attn_tile256(const pv_plan *plan, const DeviceLists &dl, const void *q,
                               const void *k_pages, const void *v_pages,
                               const int32_t *page_table, float scale, void *out, float *ws_o,
                               float *ws_ml, hipStream_t stream);
hipError_t launch_attn_combine(const pv_plan *plan, const DeviceLists &dl, const float *ws_o,
                               const float *ws_ml, void *out, hipStream_t stream);

hipError_t launch_rope_append(const pv_plan *plan, const DeviceLists &dl, int style,
                              const void *q_in, void *q_out, const void *k_new,
                              const void *v_new, const float *cos_sin, const int32_t *page_table,
                              void *k_pages, void *v_pages, hipStream_t stream);
hipError_t launch_pages_copy(bool gather, const pv_pool_desc *pool, const int32_t *page_ids,
                             int32_t n, void *k_pages, void *v_pages, void *staging,
                             hipStream_t stream);

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A planned launch needs the plan's lists on the current device: it never allocates or copies
// by itself.
static pv_status ensure_ready(const pv_plan *plan)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (!plan->uploaded) return PV_ERR_INVALID_ARG;  // pv_plan_upload / pv_plan_upload_to first
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return PV_ERR_HIP;
    if (dev != plan->device) return PV_ERR_INVALID_ARG;  // the lists live on another GPU
    return PV_OK;
}

// Brackets one kernel launch with the plan's events when timing is on.
struct KernelTimer {
    pv_plan *plan;
    int kind;
    hipStream_t stream;
    bool on;
    KernelTimer(pv_plan *p, int k, hipStream_t s, bool ran) : plan(p), kind(k), stream(s)
    {
        on = p->timing && ran;
        if (p->timing) p->event_used[k] = on;
        if (on) (void)hipEventRecord(static_cast<hipEvent_t>(p->events[2 * k]), s);
    }
    ~KernelTimer()
    {
        if (on) (void)hipEventRecord(static_cast<hipEvent_t>(plan->events[2 * kind + 1]), stream);
    }
};

}  // namespace pv

extern "C" {

pv_status pv_plan_enable_timing(pv_plan *plan, int32_t enable)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (enable) {
        for (void *&e : plan->events) {
            if (e) continue;
            hipEvent_t ev;
            if (hipEventCreate(&ev) != hipSuccess) return PV_ERR_HIP;
            e = ev;
        }
    }
    plan->timing = enable != 0;
    return PV_OK;
}

pv_status pv_plan_kernel_ms(pv_plan *plan, int32_t kind, float *ms)
{
    if (!plan || !ms || kind < 0 || kind > 4) return PV_ERR_INVALID_ARG;
    *ms = -1.f;
    if (!plan->events[0] || !plan->event_used[kind]) return PV_OK;
    hipEvent_t a = static_cast<hipEvent_t>(plan->events[2 * kind]);
    hipEvent_t b = static_cast<hipEvent_t>(plan->events[2 * kind + 1]);
    if (hipEventSynchronize(b) != hipSuccess) return PV_ERR_HIP;
    if (hipEventElapsedTime(ms, a, b) != hipSuccess) return PV_ERR_HIP;
    return PV_OK;
}

pv_status pv_plan_upload_to(pv_plan *plan, void *device_buf, size_t bytes, void *stream)
{
    if (!plan || !device_buf) return PV_ERR_INVALID_ARG;
    if (bytes < plan->image.size() || (reinterpret_cast<uintptr_t>(device_buf) & 255u) != 0)
        return PV_ERR_WORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return PV_ERR_HIP;
    if (hipMemcpyAsync(device_buf, plan->image.data(), plan->image.size(), hipMemcpyHostToDevice,
                       static_cast<hipStream_t>(stream)) != hipSuccess)
        return PV_ERR_HIP;
    if (plan->d_owned && plan->d_owned != device_buf) {
        (void)hipFree(plan->d_owned);
        plan->d_owned = nullptr;
    }
    plan->dev = pv::lists_at(plan, device_buf);
    plan->device = dev;
    plan->uploaded = true;
    return PV_OK;
}

pv_status pv_plan_upload(pv_plan *plan)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (plan->uploaded) return PV_OK;
    void *buf = nullptr;
    if (hipMalloc(&buf, plan->image.size()) != hipSuccess) return PV_ERR_HIP;
    pv_status s = pv_plan_upload_to(plan, buf, plan->image.size(), nullptr);
    if (s == PV_OK && hipStreamSynchronize(nullptr) != hipSuccess) s = PV_ERR_HIP;
    if (s != PV_OK) {
        (void)hipFree(buf);
        plan->uploaded = false;
        return s;
    }
    plan->d_owned = buf;
    return PV_OK;
}

void pv_plan_destroy(pv_plan *plan)
{
    if (!plan) return;
    if (plan->d_owned) (void)hipFree(plan->d_owned);
    for (void *e : plan->events)
        if (e) (void)hipEventDestroy(static_cast<hipEvent_t>(e));
    delete plan;
}

// The three attention kernels and the merge of split KV ranges, with the plan's lists at `dl`.
static pv_status attn_launch(pv_plan *plan, const pv::DeviceLists &dl, const void *q,
                             const void *k_pages, const void *v_pages, const int32_t *page_table,
                             float scale, void *out, float *ws_o, float *ws_ml, hipStream_t st)
{
    // the kernels touch disjoint rows of `out`; all run on the caller's stream
    {
        pv::KernelTimer t(plan, 4, st, !plan->tile256.empty());
        if (pv::launch_attn_tile256(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                    ws_ml, st) != hipSuccess)
            return PV_ERR_HIP;
    }
    {
        pv::KernelTimer t(plan, 1, st, !plan->wide.empty());
        if (pv::launch_attn_wide(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                 ws_ml, st) != hipSuccess)
            return PV_ERR_HIP;
    }
    {
        pv::KernelTimer t(plan, 0, st, !plan->narrow.empty());
        if (pv::launch_attn_narrow(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                   ws_ml, st) != hipSuccess)
            return PV_ERR_HIP;
    }
    {
        pv::KernelTimer t(plan, 2, st, !plan->combine.empty());
        if (pv::launch_attn_combine(plan, dl, ws_o, ws_ml, out, st) != hipSuccess)
            return PV_ERR_HIP;
    }
    return PV_OK;
}

static pv_status attn_args_ok(const pv_plan *plan, const void *q, const void *k_pages,
                              const void *v_pages, const int32_t *page_table, float scale,
                              const void *out)
{
    if (!q || !k_pages || !v_pages || !page_table || !out) return PV_ERR_INVALID_ARG;
    if (!pv::aligned16(q) || !pv::aligned16(k_pages) || !pv::aligned16(v_pages) ||
        !pv::aligned16(out))
        return PV_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return PV_ERR_INVALID_ARG;
    (void)plan;
    return PV_OK;
}

pv_status pv_kv_append_planned(pv_plan *plan, const void *k_new, const void *v_new,
                               const int32_t *page_table, void *k_pages, void *v_pages,
                               void *stream)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (plan->total_q == 0) return PV_OK;
    if (!k_new || !v_new || !page_table || !k_pages || !v_pages) return PV_ERR_INVALID_ARG;
    if (!pv::aligned16(k_new) || !pv::aligned16(v_new) || !pv::aligned16(k_pages) ||
        !pv::aligned16(v_pages))
        return PV_ERR_INVALID_ARG;
    pv_status s = pv::ensure_ready(plan);
    if (s != PV_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    {
        pv::KernelTimer t(plan, 3, st, true);
        e = pv::launch_kv_append(plan, plan->dev, k_new, v_new, page_table, k_pages, v_pages, st);
    }
    return e == hipSuccess ? PV_OK : PV_ERR_HIP;
}

pv_status pv_rope_kv_append_planned(pv_plan *plan, const void *q_in, void *q_out,
                                    const void *k_new, const void *v_new, const float *cos_sin,
                                    int32_t max_pos, int32_t style, const int32_t *page_table,
                                    void *k_pages, void *v_pages, void *stream)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (style != 0 && style != 1) return PV_ERR_INVALID_ARG;
    if ((q_in == nullptr) != (q_out == nullptr)) return PV_ERR_INVALID_ARG;
    if (plan->total_q == 0) return PV_OK;
    if (!k_new || !v_new || !cos_sin || !page_table || !k_pages || !v_pages)
        return PV_ERR_INVALID_ARG;
    if (!pv::aligned16(q_in) || !pv::aligned16(q_out) || !pv::aligned16(k_new) ||
        !pv::aligned16(v_new) || !pv::aligned16(cos_sin) || !pv::aligned16(k_pages) ||
        !pv::aligned16(v_pages))
        return PV_ERR_INVALID_ARG;
    for (int32_t r = 0; r < plan->num_reqs; ++r)
        if (plan->q_lens[r] > 0 && (int64_t)plan->ctx_lens[r] + plan->q_lens[r] > max_pos)
            return PV_ERR_OUT_OF_RANGE;
    pv_status s = pv::ensure_ready(plan);
    if (s != PV_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    {
        pv::KernelTimer t(plan, 3, st, true);
        e = pv::launch_rope_append(plan, plan->dev, style, q_in, q_out, k_new, v_new, cos_sin,
                                   page_table, k_pages, v_pages, st);
    }
    return e == hipSuccess ? PV_OK : PV_ERR_HIP;
}

pv_status pv_multi_token_paged_attn_planned(pv_plan *plan, const void *q, const void *k_pages,
                                            const void *v_pages, const int32_t *page_table,
                                            float scale, void *out, void *workspace,
                                            size_t workspace_bytes, void *stream)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (plan->total_q == 0) return PV_OK;
    pv_status s = attn_args_ok(plan, q, k_pages, v_pages, page_table, scale, out);
    if (s != PV_OK) return s;
    float *ws_o = nullptr, *ws_ml = nullptr;
    if (plan->workspace_bytes > 0) {
        if (!workspace || workspace_bytes < plan->workspace_bytes ||
            (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
            return PV_ERR_WORKSPACE;
        ws_o = static_cast<float *>(workspace);
        ws_ml = ws_o + (size_t)plan->partial_slots * plan->pool.head_dim;
    }
    s = pv::ensure_ready(plan);
    if (s != PV_OK) return s;
    return attn_launch(plan, plan->dev, q, k_pages, v_pages, page_table, scale, out, ws_o, ws_ml,
                       static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------------------------
// The launch that allocates nothing: everything the library itself would need device memory for
// (the plan's lists, the partial results of split KV ranges) lives in one static array.
// ---------------------------------------------------------------------------------------------
constexpr size_t kScratchBytes = PV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];  // per device: the address of that device's copy

// address of the current device's scratch array (looked up once per device, then kept)
static pv_status scratch_base(unsigned char **base)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return PV_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PV_ERR_UNSUPPORTED;
    void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PV_ERR_HIP;
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);  // same value from any thread
    }
    *base = static_cast<unsigned char *>(p);
    return PV_OK;
}

size_t pv_static_scratch_bytes(void) { return kScratchBytes; }

pv_status pv_multi_token_paged_attn_noalloc(pv_plan *plan, const void *q, const void *k_pages,
                                            const void *v_pages, const int32_t *page_table,
                                            float scale, void *out, void *stream)
{
    if (!plan) return PV_ERR_INVALID_ARG;
    if (plan->total_q == 0) return PV_OK;
    pv_status s = attn_args_ok(plan, q, k_pages, v_pages, page_table, scale, out);
    if (s != PV_OK) return s;
    const size_t lists = pv::align_up(plan->image.size(), 256);
    if (lists + plan->workspace_bytes > kScratchBytes) return PV_ERR_WORKSPACE;  // batch too large
    unsigned char *base = nullptr;
    s = scratch_base(&base);
    if (s != PV_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Nothing in the array has to start at zero: the lists are overwritten whole, and every
    // partial-result slot is written by the attention kernels before the merge reads it.
    if (hipMemcpyAsync(base, plan->image.data(), plan->image.size(), hipMemcpyHostToDevice, st) !=
        hipSuccess)
        return PV_ERR_HIP;
    float *ws_o = nullptr, *ws_ml = nullptr;
    if (plan->workspace_bytes > 0) {
        ws_o = reinterpret_cast<float *>(base + lists);
        ws_ml = ws_o + (size_t)plan->partial_slots * plan->pool.head_dim;
    }
    return attn_launch(plan, pv::lists_at(plan, base), q, k_pages, v_pages, page_table, scale, out,
                       ws_o, ws_ml, st);
}

static pv_status check_prefix(const int32_t *q_lens, const int32_t *q_start, int32_t num_reqs,
                              int32_t total_q)
{
    if (num_reqs < 0 || total_q < 0) return PV_ERR_INVALID_ARG;
    if (num_reqs > 0 && (!q_lens || !q_start)) return PV_ERR_INVALID_ARG;
    int64_t at = 0;
    for (int32_t r = 0; r < num_reqs; ++r) {
        if (q_lens[r] < 0 || q_start[r] != at) return PV_ERR_INVALID_ARG;
        at += q_lens[r];
    }
    return at == total_q ? PV_OK : PV_ERR_INVALID_ARG;
}

pv_status pv_kv_append(const pv_pool_desc *pool, const void *k_new, const void *v_new,
                       const int32_t *page_table, int32_t max_pages_per_req,
                       const int32_t *slot_offsets, const int32_t *q_lens, const int32_t *q_start,
                       int32_t num_reqs, int32_t total_q, void *k_pages, void *v_pages,
                       void *stream)
{
    pv_status s = check_prefix(q_lens, q_start, num_reqs, total_q);
    if (s != PV_OK) return s;
    if (!pool || pool->num_kv_heads <= 0) return PV_ERR_INVALID_ARG;
    pv_plan *plan = nullptr;
    // the append only needs positions, so any head grouping is fine: use G = 1
    s = pv_plan_create(pool, pool->num_kv_heads, slot_offsets, q_lens, num_reqs, max_pages_per_req,
                       &plan);
    if (s != PV_OK) return s;
    // this form has no buffer of the caller's to put the lists in: temporary device memory, and
    // a wait for the stream before it is freed
    if (plan->total_q > 0) s = pv_plan_upload(plan);
    if (s == PV_OK)
        s = pv_kv_append_planned(plan, k_new, v_new, page_table, k_pages, v_pages, stream);
    if (s == PV_OK && plan->total_q > 0 &&
        hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess)
        s = PV_ERR_HIP;
    pv_plan_destroy(plan);
    return s;
}

pv_status pv_multi_token_paged_attn(const pv_pool_desc *pool, int32_t num_q_heads, const void *q,
                                    const void *k_pages, const void *v_pages,
                                    const int32_t *page_table, int32_t max_pages_per_req,
                                    const int32_t *ctx_lens, const int32_t *q_lens,
                                    const int32_t *q_start, int32_t num_reqs, int32_t total_q,
                                    float scale, void *out, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    pv_status s = check_prefix(q_lens, q_start, num_reqs, total_q);
    if (s != PV_OK) return s;
    pv_plan *plan = nullptr;
    s = pv_plan_create(pool, num_q_heads, ctx_lens, q_lens, num_reqs, max_pages_per_req, &plan);
    if (s != PV_OK) return s;
    if (plan->total_q == 0) {
        pv_plan_destroy(plan);
        return PV_OK;
    }
    // The caller's workspace holds the partial results first and, behind them, the plan's lists
    // when it is large enough for both (pv_attn_workspace_bytes is): then nothing is allocated
    // and the library does not wait; the temporary plan, whose host image the copy of the lists
    // reads, is freed by a host function queued on the stream behind the launches.  Otherwise:
    // temporary device memory and a wait.
    const size_t ws_part = pv::align_up(plan->workspace_bytes, 256);
    const bool ws_ok = workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u) == 0;
    if (plan->workspace_bytes > 0 && (!ws_ok || workspace_bytes < plan->workspace_bytes)) {
        pv_plan_destroy(plan);
        return PV_ERR_WORKSPACE;
    }
    bool wait = false;
    if (ws_ok && workspace_bytes >= ws_part + plan->image.size()) {
        s = pv_plan_upload_to(plan, static_cast<unsigned char *>(workspace) + ws_part,
                              workspace_bytes - ws_part, stream);
    } else {
        s = pv_plan_upload(plan);
        wait = true;
    }
    if (s == PV_OK)
        s = pv_multi_token_paged_attn_planned(plan, q, k_pages, v_pages, page_table, scale, out,
                                              workspace, workspace_bytes, stream);
    if (s == PV_OK && !wait) {
        // the plan holds no device memory and no events here: freeing it is a plain delete,
        // which a host function may do (it must not call into the runtime)
        if (hipLaunchHostFunc(static_cast<hipStream_t>(stream),
                              [](void *p) { delete static_cast<pv_plan *>(p); },
                              plan) == hipSuccess)
            return PV_OK;
        wait = true;  // could not queue it: wait instead
    }
    if (s != PV_OK) wait = true;  // a copy that reads the plan's image may have been queued
    if (wait && hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess && s == PV_OK)
        s = PV_ERR_HIP;
    pv_plan_destroy(plan);
    return s;
}

static pv_status pages_copy(bool gather, const pv_pool_desc *pool, const int32_t *page_ids,
                            int32_t n, void *k_pages, void *v_pages, void *staging, void *stream)
{
    pv_status why;
    if (!pv::pool_desc_valid(pool, &why)) return why;
    if (n < 0) return PV_ERR_INVALID_ARG;
    if (n == 0) return PV_OK;
    if (!page_ids || !k_pages || !v_pages || !staging) return PV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(staging) & 15u) != 0) return PV_ERR_INVALID_ARG;
    hipError_t e = pv::launch_pages_copy(gather, pool, page_ids, n, k_pages, v_pages, staging,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PV_OK : PV_ERR_HIP;
}

pv_status pv_pages_gather(const pv_pool_desc *pool, const void *k_pages, const void *v_pages,
                          const int32_t *page_ids, int32_t n, void *staging, void *stream)
{
    return pages_copy(true, pool, page_ids, n, const_cast<void *>(k_pages),
                      const_cast<void *>(v_pages), staging, stream);
}

pv_status pv_pages_scatter(const pv_pool_desc *pool, const void *staging, const int32_t *page_ids,
                           int32_t n, void *k_pages, void *v_pages, void *stream)
{
    return pages_copy(false, pool, page_ids, n, k_pages, v_pages, const_cast<void *>(staging),
                      stream);
}

size_t pv_attn_workspace_bytes(const pv_pool_desc *pool, int32_t num_q_heads, int32_t num_reqs,
                               int32_t total_q, int32_t max_kv_len)
{
    if (!pv::pool_desc_valid(pool, nullptr) || num_q_heads <= 0 || num_reqs < 0 || total_q < 0 ||
        max_kv_len < 0)
        return 0;
    // Splitting only happens while a kernel has fewer items than the target and never makes a
    // part shorter than half the target share, so each kernel ends with fewer than
    // items + split_target parts of at most 16, kWideRows resp. kTileRows rows.  Independently, a row can be
    // in at most max_kv_len / min_split_keys + 1 parts.
    const pv::Tuning t = pv::default_tuning();
    const int64_t rows = (int64_t)total_q * num_q_heads +
                         (int64_t)num_reqs * pool->num_kv_heads * pv::kNarrowRows;
    const int64_t max_parts = (int64_t)max_kv_len / t.min_split_keys + 1;
    const int64_t by_rows = rows * max_parts;
    const int64_t by_items =
        2 * (int64_t)t.split_target * (pv::kNarrowRows + pv::kWideRows + pv::kTileRows);
    const int64_t slots = by_rows < by_items ? by_rows : by_items;
    // behind the partial results: room for the plan's lists (three int32 per request, 48 bytes
    // per work item and 40 per merge item and its chunks, 16 per append group, nine 256-byte
    // alignments), so that the one-shot call neither allocates nor waits
    const int64_t n_items = rows / pv::kNarrowRows + (int64_t)num_reqs * pool->num_kv_heads * 3 +
                            2 * (int64_t)t.split_target * 3;
    const int64_t lists = 12 * (int64_t)num_reqs + 48 * n_items + 40 * n_items / 2 +
                          8 * (slots / 8 + n_items) + 16 * ((int64_t)total_q + 2 * num_reqs) +
                          10 * 256;
    return pv::align_up((size_t)slots * (size_t)(pool->head_dim + 2) * sizeof(float), 256) +
           (size_t)lists;
}

}  // extern "C"
