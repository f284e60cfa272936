/*
 * pv.h - C ABI of libpv: multi-token attention over a paged KV cache, and the
 * KV append that feeds it, for one AMD MI355X (gfx950).
 *
 * The operation is the generalized PagedAttention of the Pensieve paper
 * (arXiv 2312.05516, Section 4.4 "Multi-token attention for non-contiguous
 * cache" and Section 4.4.1 "Unifying the prefill and generation phase"):
 * every request r of a batch brings n_r >= 0 new tokens (n_r = 1 is a
 * generation step, n_r > 1 a new prompt), its K/V rows are first stored into
 * the slots the page table assigns to them, and then each new token attends
 * causally to the request's c_r cached tokens plus the new tokens up to and
 * including itself (paper Eq. 2-3 with the causal rule of Section 4.4).
 *
 * Conventions
 *   - Every "device" pointer is GPU memory owned by the caller (allocate it
 *     with anything, e.g. PyTorch).  Every "host" pointer is ordinary CPU
 *     memory, read during the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Kernel launches are asynchronous on it unless stated otherwise.
 *   - Errors are return codes; nothing is thrown across the ABI.  Shapes,
 *     null pointers and unsupported combinations are checked on the host
 *     before anything is launched.  The *contents* of device index arrays are
 *     not checked by the launching calls; pv_plan_check_page_table() checks a
 *     host copy.
 *   - The library allocates device memory in two documented places only (pv_plan_upload; the
 *     one-shot forms when the workspace passed is too small for the lists).  Its only state
 *     outside plans is the static device array of pv_multi_token_paged_attn_noalloc and the
 *     address of that array on each GPU, looked up once.
 *   - A plan may be shared by the launches of many layers, but by one host thread at a time (a
 *     launch updates the plan's timing state).
 *   - Alignment: q, out, k_new, v_new, the pools and the rotary table are read and written with
 *     16-byte vector accesses: every such pointer must be 16-byte aligned (the launching calls
 *     return PV_ERR_INVALID_ARG otherwise); a workspace must be 256-byte aligned.
 *   - Supported: page_size 16; head_dim 64 or 128; dtype f16 or bf16;
 *     num_q_heads a multiple of num_kv_heads (consecutive query heads
 *     hq = hk*G .. hk*G+G-1 share KV head hk, G = num_q_heads/num_kv_heads).
 *     Anything else returns PV_ERR_UNSUPPORTED / PV_ERR_INVALID_ARG.
 *
 * Pool layout (one pool for K and one for V, 16-bit elements, P = page_size,
 * D = head_dim, Hkv = num_kv_heads).  Page-major, then KV head; inside one
 * (page, head) tile of P*D elements the data is grouped in runs of 8 along the
 * dimension the attention contracts over, which is what one MFMA lane consumes:
 *   K(page p, head h, slot s, dim d) at element (((p*Hkv+h)*(D/8) + d/8)*P + s)*8 + d%8
 *   V(page p, head h, slot s, dim d) at element (((p*Hkv+h)*(P/8) + s/8)*D + d)*8 + s%8
 * A logical token position t of request r lives in page
 * page_table[r*max_pages_per_req + t/P], slot t%P.  Slots past the end of a
 * request's last page may hold anything (including NaN); they are never used.
 *
 * Packed query / output layout: [total_q, num_q_heads, D], request r owns rows
 * q_start[r] .. q_start[r]+q_lens[r]-1 (paper Section 4.4.1: the tokens of all
 * requests are concatenated).  New K/V rows: [total_q, num_kv_heads, D].
 */
#ifndef PV_H_
#define PV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Size of the static device array behind pv_multi_token_paged_attn_noalloc (per GPU). */
#ifndef PV_STATIC_SCRATCH_BYTES
#define PV_STATIC_SCRATCH_BYTES (32u << 20)
#endif

typedef enum {
    PV_OK = 0,
    PV_ERR_INVALID_ARG = 1,  /* null pointer, negative size, inconsistent arrays */
    PV_ERR_UNSUPPORTED = 2,  /* page size / head dim / dtype outside the supported set */
    PV_ERR_OUT_OF_RANGE = 3, /* a length needs more pages than the table has, or a page index
                                is outside the pool, or sizes overflow 32-bit indexing */
    PV_ERR_WORKSPACE = 4,    /* workspace missing or too small */
    PV_ERR_HIP = 5           /* a HIP runtime call failed (no device, launch failure, ...) */
} pv_status;

typedef enum { PV_F16 = 0, PV_BF16 = 1 } pv_dtype;

typedef struct {
    int32_t num_pages;    /* pages in the pool */
    int32_t page_size;    /* tokens per page; must be 16 */
    int32_t num_kv_heads; /* Hkv */
    int32_t head_dim;     /* D: 64 or 128 */
    int32_t dtype;        /* pv_dtype of q, k, v and out */
} pv_pool_desc;

/* Opaque: the per-batch auxiliary data built once on the CPU and reused by every layer. */
typedef struct pv_plan pv_plan;

/* Human-readable name of a status code (static storage). */
const char *pv_status_string(pv_status s);

/* Bytes of ONE pool (K or V) for this description; 0 if the description is invalid. */
size_t pv_pool_bytes(const pv_pool_desc *pool);

/* Element offsets inside a pool, as documented above (host helpers for callers that fill or
 * inspect a pool themselves).  Return -1 on an invalid description or index. */
int64_t pv_pool_k_offset(const pv_pool_desc *pool, int32_t page, int32_t head, int32_t slot,
                         int32_t d);
int64_t pv_pool_v_offset(const pv_pool_desc *pool, int32_t page, int32_t head, int32_t slot,
                         int32_t d);

/*
 * Auxiliary arrays of a batch (paper Section 6.4: cumulative sequence lengths and the like are
 * computed once on the CPU and shared by all layers; Section 4.4.1: the batch carries a record of
 * which rows of the concatenated tokens belong to which request).
 *
 * pv_plan_create is pure host code: it validates the lengths, computes
 * q_start = exclusive prefix sum of q_lens, and splits the work of the batch into the work
 * items the kernels consume (longest first).  ctx_lens[r] counts the tokens already cached
 * for request r, NOT including its q_lens[r] new ones; both are host arrays of num_reqs
 * entries.  q_lens[r] == 0 is legal (the request produces nothing); num_reqs == 0 is legal.
 * Every request must fit its page-table row: ceil((ctx+q)/page_size) <= max_pages_per_req,
 * else PV_ERR_OUT_OF_RANGE.  On success *plan owns host memory only, until pv_plan_destroy.
 */
pv_status pv_plan_create(const pv_pool_desc *pool, int32_t num_q_heads,
                         const int32_t *ctx_lens /* host [num_reqs] */,
                         const int32_t *q_lens /* host [num_reqs] */, int32_t num_reqs,
                         int32_t max_pages_per_req, pv_plan **plan);

/* Frees the plan (and the device memory pv_plan_upload allocated, if it was used).  The caller
 * must make sure no launch that uses the plan is still running.  NULL is ignored. */
void pv_plan_destroy(pv_plan *plan);

/*
 * The kernels read the plan's lists (work items, prefix sums, append groups) from device memory.
 * A *_planned launch never allocates or copies: the lists must have been put on the current
 * device first, by one of the two calls below, else the launch returns PV_ERR_INVALID_ARG.
 *
 * pv_plan_upload_to: the caller owns the memory.  Copies pv_plan_device_bytes(plan) bytes into
 * device_buf (256-byte aligned, at least that large, else PV_ERR_WORKSPACE) with one asynchronous
 * copy on `stream`, allocates nothing and does not wait; launches on the same stream may follow
 * at once.  The buffer must stay untouched until the last launch that uses the plan has finished,
 * and the plan (the copy reads its host memory) must not be destroyed before `stream` has passed
 * the copy.
 *
 * pv_plan_upload: convenience.  Allocates device memory that the plan then owns (freed by
 * pv_plan_destroy), copies, and waits for the copy.  Idempotent.
 */
size_t pv_plan_device_bytes(const pv_plan *plan);
pv_status pv_plan_upload_to(pv_plan *plan, void *device_buf, size_t bytes, void *stream);
pv_status pv_plan_upload(pv_plan *plan);
/* 1 if the plan holds device memory of its own (pv_plan_upload was used), 0 if not, -1 for NULL. */
int32_t pv_plan_owns_device_memory(const pv_plan *plan);

/* Total number of new tokens (rows of q / out / k_new / v_new). */
int32_t pv_plan_total_q(const pv_plan *plan);
/* Host pointer to q_start[num_reqs], valid until pv_plan_destroy. */
const int32_t *pv_plan_q_start(const pv_plan *plan);
/* Bytes of workspace the attention launch of this plan needs (0 if none; the pointer passed
 * must be 256-byte aligned). */
size_t pv_plan_workspace_bytes(const pv_plan *plan);

/* Work-item introspection (for tests and reports).  kind: 0 = items of the bandwidth-oriented
 * kernel (at most 16 query rows per item), 1 = items of the matrix-core kernel (at most 128
 * rows), 2 = split-KV combine items, 3 = items of the 256-row matrix-core kernel (exactly 256
 * rows; the full 256-row tiles of units with at least 256 rows and 8192 keys, head size 128).
 * pv_plan_work_item fills eight int32 fields:
 *   req, kv_head, row_begin, row_count, kv_begin, kv_end, split_index, split_count
 * where a "row" is a (new token, query head of the group) pair, row = token*G + g.  Which kernel
 * a (request, KV head) unit goes to is the plan's decision: more than 32 rows always means the
 * matrix-core kernel (items of at most 128 rows); smaller units join it when the batch has such
 * work and the small units are not a large amount of work themselves (one attention launch
 * instead of two), otherwise they are cut into items of the bandwidth-oriented kernel. */
int32_t pv_plan_num_work_items(const pv_plan *plan, int32_t kind);
pv_status pv_plan_work_item(const pv_plan *plan, int32_t kind, int32_t index, int32_t out[8]);

/* Host-side check of a page table against the plan (host copy of the table, row stride
 * max_pages_per_req): every page a request needs must be in [0, num_pages); and, if
 * check_append_unique != 0, no two new tokens may land in the same (page, slot).  Pages may be
 * shared between requests for reading (paper Section 4.3.4, sub-requests). */
pv_status pv_plan_check_page_table(const pv_plan *plan, const int32_t *page_table /* host */,
                                   int32_t check_append_unique);

/*
 * KV append (paper Section 4.4.1: newly generated KV-tokens are stored in their allocated slots
 * before attention).  For request r and new token j < q_lens[r], the row
 * k_new[q_start[r]+j, h, :] is stored at logical position ctx_lens[r]+j of that request, for
 * every KV head h; likewise v_new.  Pure 16-bit moves: the pool image is bit-exact and slots
 * that are not addressed keep their contents.  Destinations must be distinct.
 *   k_new, v_new : device [total_q, Hkv, D]
 *   page_table   : device int32 [num_reqs, max_pages_per_req]
 *   k_pages, v_pages : device pools (pv_pool_bytes each)
 */
pv_status pv_kv_append_planned(pv_plan *plan, const void *k_new, const void *v_new,
                               const int32_t *page_table, void *k_pages, void *v_pages,
                               void *stream);

/*
 * Multi-token paged attention (paper Section 4.4, Eq. 2-3).  For request r, query head hq
 * (KV head hk = hq / G) and new token i < q_lens[r]:
 *   s_t = scale * <q[q_start[r]+i, hq, :], K_r[t, hk, :]>     for t = 0 .. ctx_lens[r]+i
 *   out[q_start[r]+i, hq, :] = sum_t softmax(s)_t * V_r[t, hk, :]
 * with K_r, V_r read through the page table.  `scale` multiplies the scores (the paper's
 * divisor is its reciprocal; 1/sqrt(D) is customary) and may be any finite number, negative
 * and zero included; NaN or infinity returns PV_ERR_INVALID_ARG.  Scores, softmax and the
 * weighted sum are accumulated in fp32; out is rounded to the 16-bit dtype.  For
 * |scale*log2(e)| <= 0.25 the 256-row kernel applies the scale to the queries (rounded back to
 * 16 bits) instead of the scores, a perturbation of the size of the rounding the probabilities
 * get; larger scales are applied to the scores in fp32 by every kernel.  Must run after the append of
 * the same batch on the same stream.
 *   q, out     : device [total_q, Hq, D]
 * Launches at most four kernels (the two matrix-core attention kernels, bandwidth-oriented
 * attention, merge of split KV ranges), all on `stream`; which of them a batch needs is decided
 * by the plan.  Asynchronous, no allocation.
 *   workspace  : device, >= pv_plan_workspace_bytes(plan) bytes, 256-byte aligned; may be NULL
 *                when that is 0.  Its contents are scratch (partial results of split KV
 *                ranges); two launches that overlap in time need different workspaces.
 */
pv_status pv_multi_token_paged_attn_planned(pv_plan *plan, const void *q, const void *k_pages,
                                            const void *v_pages, const int32_t *page_table,
                                            float scale, void *out, void *workspace,
                                            size_t workspace_bytes, void *stream);

/*
 * The same attention launch for callers that cannot allocate device memory or be handed any by
 * something that does: code under HIP graph capture set-up, tight serving loops, harnesses that
 * forbid allocation.  Behaves like pv_multi_token_paged_attn_planned, except that the plan need
 * not have been uploaded and no workspace is passed: the plan's lists and the partial results of
 * split KV ranges go into a static device array of PV_STATIC_SCRATCH_BYTES (32 MiB) that every
 * GPU the library runs on holds until the process ends.  The call copies the lists there with one
 * asynchronous copy on `stream` and launches; it calls no allocating routine and does not wait.
 * PV_ERR_WORKSPACE if the batch needs more than the array holds (pv_plan_device_bytes rounded up
 * to 256 + pv_plan_workspace_bytes > pv_static_scratch_bytes()): use the planned call then.
 * All calls on one GPU share that GPU's array: two calls whose execution may overlap (different
 * streams, or the same plan replayed while an earlier launch still runs) race on it.  Nothing in
 * the array needs clearing between calls.  The plan must not be destroyed before `stream` has
 * passed the call (the copy reads its host memory).
 */
size_t pv_static_scratch_bytes(void);
pv_status pv_multi_token_paged_attn_noalloc(pv_plan *plan, const void *q, const void *k_pages,
                                            const void *v_pages, const int32_t *page_table,
                                            float scale, void *out, void *stream);

/*
 * Per-kernel timing for reports.  After pv_plan_enable_timing(plan, 1) every planned launch also
 * records a pair of HIP events around each kernel it launches (on the launch stream; the events
 * belong to the plan).  pv_plan_kernel_ms waits for the end event of that kernel in the plan's most
 * recent launch and returns its duration in milliseconds; *ms = -1 if that kernel did not run.
 * kind: 0 = bandwidth-oriented attention kernel, 1 = matrix-core attention kernel,
 *       2 = split-KV combine, 3 = KV append, 4 = 256-row matrix-core attention kernel.
 */
pv_status pv_plan_enable_timing(pv_plan *plan, int32_t enable);
pv_status pv_plan_kernel_ms(pv_plan *plan, int32_t kind, float *ms);

/*
 * One-shot forms with explicit arrays: convenient, not meant for the per-layer hot loop (use a
 * plan there).  They build a temporary plan from the HOST length arrays (read during the call),
 * launch, and free the plan.  q_start must be the exclusive prefix sum of q_lens and total_q their
 * sum, else PV_ERR_INVALID_ARG.  slot_offsets[r] is the logical position of request r's first
 * new token (normally ctx_lens[r]).
 *   pv_multi_token_paged_attn: when `workspace` (256-byte aligned) holds at least
 *     pv_attn_workspace_bytes(...) bytes, the temporary plan's lists go behind the partial results
 *     in it: nothing is allocated, the lists are copied with hipMemcpyAsync on `stream`, the
 *     library does not synchronise, and the temporary plan is freed by a host function queued on
 *     `stream` behind the launches (what the runtime does for a copy out of pageable host memory
 *     is its own business; it may wait for that one copy).  With a smaller workspace that still
 *     covers the partial results, the lists go to temporary device memory and the call waits for
 *     the stream before freeing it.
 *   pv_kv_append has no buffer argument: temporary device memory, and it waits for the stream.
 */
pv_status pv_kv_append(const pv_pool_desc *pool, const void *k_new, const void *v_new,
                       const int32_t *page_table /* device */, int32_t max_pages_per_req,
                       const int32_t *slot_offsets /* host */, const int32_t *q_lens /* host */,
                       const int32_t *q_start /* host */, int32_t num_reqs, int32_t total_q,
                       void *k_pages, void *v_pages, void *stream);

pv_status pv_multi_token_paged_attn(const pv_pool_desc *pool, int32_t num_q_heads, const void *q,
                                    const void *k_pages, const void *v_pages,
                                    const int32_t *page_table /* device */,
                                    int32_t max_pages_per_req, const int32_t *ctx_lens /* host */,
                                    const int32_t *q_lens /* host */,
                                    const int32_t *q_start /* host */, int32_t num_reqs,
                                    int32_t total_q, float scale, void *out, void *workspace,
                                    size_t workspace_bytes, void *stream);

/*
 * Page gather / scatter for tier swapping (paper Section 4.3.2: KV-tokens are copied out to a CPU
 * cache ahead of time; Section 4.3.3: they are copied back layer by layer, and a layer's attention
 * starts once its KV-tokens have landed).  Whole pages move between the pools and a staging buffer:
 * for the i-th listed page the staging buffer holds that page's K image (num_kv_heads*16*D
 * elements, exactly as in the pool) followed by its V image, i.e. 2*pv_pool_bytes/num_pages bytes
 * per page.  Pure copies (bit-exact); pages that are not listed are not touched.
 *   page_ids : device int32 [n]; every id must be in [0, num_pages) and, for the scatter, distinct
 *              (not checked by these calls)
 *   staging  : device memory, or pinned host memory the GPU can address (e.g. hipHostMalloc): then
 *              the copy crosses PCIe inside the kernel; 16-byte aligned
 * Asynchronous on `stream`; record an event after a scatter and make the attention stream wait for
 * it to get the paper's per-layer gating.
 */
pv_status pv_pages_gather(const pv_pool_desc *pool, const void *k_pages, const void *v_pages,
                          const int32_t *page_ids /* device */, int32_t n, void *staging,
                          void *stream);
pv_status pv_pages_scatter(const pv_pool_desc *pool, const void *staging,
                           const int32_t *page_ids /* device */, int32_t n, void *k_pages,
                           void *v_pages, void *stream);

/*
 * Rotary position embedding fused with the KV append: the producer step in front of the hot path
 * for the Llama 2 models of the paper (Section 6.1 names rotary embedding among their features;
 * Section 4.4.1: the linear layers produce Q/K/V, the new K/V are stored, attention follows).
 * The paper does not print the transform; it is the published RoFormer one.  For request r and
 * new token j < q_lens[r] at logical position t = ctx_lens[r] + j, pair i of every head (of k_new
 * and of q_in) is rotated by the angle t * theta_i:
 *     out_a = a cos - b sin,   out_b = b cos + a sin,
 *   style 0 (interleaved): (a, b) = elements (2i, 2i+1);  style 1 (half split): (i, i + D/2).
 * The rotated K rows and the unchanged V rows are stored as by pv_kv_append_planned; the rotated
 * Q rows go to q_out (may be q_in itself).  Arithmetic in fp32, rounded to the 16-bit type
 * (nearest even); V is moved bit for bit; slots that are not addressed keep their contents.
 *   q_in, q_out : device [total_q, Hq, D]; both NULL = K/V only
 *   k_new, v_new: device [total_q, Hkv, D]
 *   cos_sin     : device float [max_pos, D]: for position t, D/2 cosines then D/2 sines of
 *                 t * theta_i (pv_rope_table fills a host copy with theta_i = base^(-2i/D))
 *   max_pos     : rows of the table; PV_ERR_OUT_OF_RANGE unless every ctx_lens[r] + q_lens[r]
 *                 <= max_pos
 * One launch on `stream`, asynchronous, no allocation.
 */
pv_status pv_rope_kv_append_planned(pv_plan *plan, const void *q_in, void *q_out,
                                    const void *k_new, const void *v_new, const float *cos_sin,
                                    int32_t max_pos, int32_t style, const int32_t *page_table,
                                    void *k_pages, void *v_pages, void *stream);

/* Host: table[t*D + i] = cos(t * base^(-2i/D)), table[t*D + D/2 + i] = sin(same), t < max_pos,
 * i < D/2, evaluated in double precision and rounded to float.  PV_ERR_INVALID_ARG unless
 * base > 0, head_dim is even and positive, max_pos >= 0 and table is not NULL. */
pv_status pv_rope_table(double base, int32_t head_dim, int32_t max_pos, float *table /* host */);

/*
 * Recomputation-cost model of the eviction policy (paper Section 4.3.1).  Pure host code.
 * Cost(l) = Cost_attention(l) + c_other is the cost of recomputing one 32-token chunk whose
 * attention spans l context tokens; Cost_attention is profiled at a few context sizes (the paper
 * uses powers of two; `bench.py --cost-profile` measures it with this library's kernel) and
 * interpolated linearly in between, the first / last segment being extended outside the range.
 *   ctx_points : host, strictly ascending context sizes [n];  attn_cost : host [n]
 * pv_cost_model returns Cost(l) (c_other alone when n == 0, attn_cost[0] + c_other when n == 1);
 * NaN on a null pointer with n > 0.
 * pv_retention_order writes the chunk indices in eviction order, i.e. ascending retention value
 * V = cost[i] / idle_time[i] (idle_time = time since the chunk's conversation was last active,
 * > 0; ties keep the lower index first).  PV_ERR_INVALID_ARG on null pointers or idle_time <= 0.
 */
double pv_cost_model(const int32_t *ctx_points, const double *attn_cost, int32_t n, double c_other,
                     int32_t l);
pv_status pv_retention_order(const double *cost, const double *idle_time, int32_t n,
                             int32_t *order_out);

/* Upper bound of what the one-shot attention call can need for such a batch: partial results of
 * split KV ranges plus the lists of its temporary plan. */
size_t pv_attn_workspace_bytes(const pv_pool_desc *pool, int32_t num_q_heads, int32_t num_reqs,
                               int32_t total_q, int32_t max_kv_len);

#ifdef __cplusplus
}
#endif
#endif /* PV_H_ */
