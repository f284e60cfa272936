/*
 * CPU oracle for multi-token paged attention and KV append.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
 * library is checked against.  It shares no code, header, table or helper with
 * the HIP path and nothing in the product may call it.
 *
 * What it computes (paper, Section 2.1 Eq. 2-3 and Section 4.4 / 4.4.1):
 *   1. append:  the new K/V rows of each request are stored into the slots the
 *      page table assigns to logical positions ctx .. ctx+n-1 (store first,
 *      attend afterwards, Section 4.4.1);
 *   2. rebuild: each request's K and V are read back through the page table
 *      into contiguous [L, D] arrays ("logically contiguous, physically at
 *      random locations", Fig. single-vs-multi-token attention);
 *   3. attend:  per query head, A = Q K^T * scale, a new token i sees logical
 *      positions 0 .. ctx+i (causal rule of Section 4.4), O = softmax(A) V
 *      (Eq. 2-3); query heads are grouped consecutively onto KV heads
 *      (Section 6.1, grouped-query attention).
 * All arithmetic is done in the requested real type (double by default, float
 * on request); the 16-bit inputs are widened exactly; nothing is tiled, fused
 * or reordered.
 *
 * Pool layout (one pool for K, one for V; 16-bit elements; P = page_size = 16,
 * D = head_dim, Hkv = num_kv_heads).  Both pools are page-major, then KV head,
 * and inside one (page, head) tile the elements are grouped in runs of 8 along
 * the dimension that attention contracts over:
 *   K(page p, head h, slot s, dim d) at (((p*Hkv + h)*(D/8) + d/8)*P + s)*8 + d%8
 *   V(page p, head h, slot s, dim d) at (((p*Hkv + h)*(P/8) + s/8)*D + d)*8 + s%8
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t num_pages;
    int32_t page_size;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t dtype; /* 0 = IEEE binary16, 1 = bfloat16 */
} pvo_pool_desc;

enum { PVO_OK = 0, PVO_BAD_ARG = 1, PVO_BAD_PAGE = 2, PVO_NO_MEM = 3 };

/* ---- exact widening of the 16-bit formats ---- */
static float pvo_half_to_float(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h >> 15) & 1u;
    const uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
    const uint32_t mant = (uint32_t)h & 0x3FFu;
    float v;
    if (expo == 0) {
        v = ldexpf((float)mant, -24); /* subnormal or zero */
    } else if (expo == 31) {
        v = mant ? NAN : INFINITY;
    } else {
        v = ldexpf((float)(mant | 0x400u), (int)expo - 25);
    }
    return sign ? -v : v;
}

static float pvo_bf16_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static double pvo_widen(uint16_t x, int dtype)
{
    return (double)(dtype == 0 ? pvo_half_to_float(x) : pvo_bf16_to_float(x));
}

double pvo_widen16(uint16_t x, int32_t dtype) { return pvo_widen(x, dtype); }

/* ---- pool addressing ---- */
int64_t pvo_k_index(const pvo_pool_desc *p, int64_t page, int64_t head, int64_t slot, int64_t d)
{
    const int64_t P = p->page_size, D = p->head_dim, H = p->num_kv_heads;
    return (((page * H + head) * (D / 8) + d / 8) * P + slot) * 8 + d % 8;
}

int64_t pvo_v_index(const pvo_pool_desc *p, int64_t page, int64_t head, int64_t slot, int64_t d)
{
    const int64_t P = p->page_size, D = p->head_dim, H = p->num_kv_heads;
    return (((page * H + head) * (P / 8) + slot / 8) * D + d) * 8 + slot % 8;
}

static int pvo_desc_ok(const pvo_pool_desc *p)
{
    return p && p->num_pages > 0 && p->page_size > 0 && p->page_size % 8 == 0 &&
           p->num_kv_heads > 0 && p->head_dim > 0 && p->head_dim % 8 == 0 &&
           (p->dtype == 0 || p->dtype == 1);
}

/* ---- step 1: append (pure 16-bit copies) ---- */
int pvo_kv_append(const pvo_pool_desc *p, const uint16_t *k_new, const uint16_t *v_new,
                  const int32_t *page_table, int32_t max_pages, const int32_t *slot_offsets,
                  const int32_t *q_lens, const int32_t *q_start, int32_t num_reqs,
                  uint16_t *k_pages, uint16_t *v_pages)
{
    if (!pvo_desc_ok(p)) return PVO_BAD_ARG;
    const int64_t P = p->page_size, D = p->head_dim, H = p->num_kv_heads;
    for (int32_t r = 0; r < num_reqs; ++r) {
        for (int32_t j = 0; j < q_lens[r]; ++j) {
            const int64_t t = (int64_t)slot_offsets[r] + j; /* logical position */
            const int64_t lp = t / P, slot = t % P;
            if (lp >= max_pages) return PVO_BAD_PAGE;
            const int64_t page = page_table[(int64_t)r * max_pages + lp];
            if (page < 0 || page >= p->num_pages) return PVO_BAD_PAGE;
            const int64_t row = (int64_t)q_start[r] + j;
            for (int64_t h = 0; h < H; ++h)
                for (int64_t d = 0; d < D; ++d) {
                    k_pages[pvo_k_index(p, page, h, slot, d)] = k_new[(row * H + h) * D + d];
                    v_pages[pvo_v_index(p, page, h, slot, d)] = v_new[(row * H + h) * D + d];
                }
        }
    }
    return PVO_OK;
}

/* ---- step 2: rebuild one request's contiguous K and V for one KV head ---- */
int pvo_gather_kv(const pvo_pool_desc *p, const uint16_t *k_pages, const uint16_t *v_pages,
                  const int32_t *page_row, int32_t max_pages, int32_t len, int32_t head,
                  double *k_out, double *v_out)
{
    if (!pvo_desc_ok(p)) return PVO_BAD_ARG;
    const int64_t P = p->page_size, D = p->head_dim;
    for (int64_t t = 0; t < len; ++t) {
        const int64_t lp = t / P, slot = t % P;
        if (lp >= max_pages) return PVO_BAD_PAGE;
        const int64_t page = page_row[lp];
        if (page < 0 || page >= p->num_pages) return PVO_BAD_PAGE;
        for (int64_t d = 0; d < D; ++d) {
            k_out[t * D + d] = pvo_widen(k_pages[pvo_k_index(p, page, head, slot, d)], p->dtype);
            v_out[t * D + d] = pvo_widen(v_pages[pvo_v_index(p, page, head, slot, d)], p->dtype);
        }
    }
    return PVO_OK;
}

/* ---- step 3: attend, instantiated for double and float ---- */
#define PVO_REAL double
#define PVO_EXP exp
#define PVO_NAME pvo_attend_unit_f64
#include "pv_oracle_attend.inc"
#undef PVO_REAL
#undef PVO_EXP
#undef PVO_NAME

#define PVO_REAL float
#define PVO_EXP expf
#define PVO_NAME pvo_attend_unit_f32
#include "pv_oracle_attend.inc"
#undef PVO_REAL
#undef PVO_EXP
#undef PVO_NAME

/*
 * Whole batch.  out is [total_q, Hq, D] doubles; only rows of the selected
 * units are written.  unit_mask is NULL (all units) or [R * Hkv] bytes, nonzero
 * = compute that (request, KV head).  precision: 0 = double, 1 = float.
 * probs (optional) receives the probability rows of (probs_req, probs_head):
 * [q_lens[probs_req], ctx+n] doubles, zero where masked.
 * Returns PVO_OK or an error; *threads_used gets the OpenMP team size.
 */
int pvo_attn(const pvo_pool_desc *p, int32_t num_q_heads, const uint16_t *q,
             const uint16_t *k_pages, const uint16_t *v_pages, const int32_t *page_table,
             int32_t max_pages, const int32_t *ctx_lens, const int32_t *q_lens,
             const int32_t *q_start, int32_t num_reqs, double scale, const uint8_t *unit_mask,
             int32_t precision, int32_t num_threads, double *out, int32_t probs_req,
             int32_t probs_head, double *probs, int32_t *threads_used)
{
    if (!pvo_desc_ok(p) || num_q_heads <= 0 || num_q_heads % p->num_kv_heads != 0)
        return PVO_BAD_ARG;
    const int64_t D = p->head_dim, Hkv = p->num_kv_heads, Hq = num_q_heads;
    const int64_t G = Hq / Hkv;
    const int64_t units = (int64_t)num_reqs * Hkv;
    int status = PVO_OK;
    int team = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        team = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1)
        for (int64_t u = 0; u < units; ++u) {
            const int64_t r = u / Hkv, hk = u % Hkv;
            if (unit_mask && !unit_mask[u]) continue;
            const int64_t n = q_lens[r], c = ctx_lens[r], L = c + n;
            if (n <= 0) continue;
            double *kbuf = (double *)malloc(sizeof(double) * (size_t)(L * D));
            double *vbuf = (double *)malloc(sizeof(double) * (size_t)(L * D));
            if (!kbuf || !vbuf) {
#pragma omp critical
                status = PVO_NO_MEM;
                free(kbuf);
                free(vbuf);
                continue;
            }
            int rc = pvo_gather_kv(p, k_pages, v_pages, page_table + r * max_pages, max_pages,
                                   (int32_t)L, (int32_t)hk, kbuf, vbuf);
            if (rc != PVO_OK) {
#pragma omp critical
                status = rc;
            } else {
                for (int64_t g = 0; g < G; ++g) {
                    const int64_t hq = hk * G + g; /* consecutive query heads share a KV head */
                    double *pr = (probs && r == probs_req && hq == probs_head) ? probs : NULL;
                    const uint16_t *qrow = q + ((int64_t)q_start[r] * Hq + hq) * D;
                    double *orow = out + ((int64_t)q_start[r] * Hq + hq) * D;
                    if (precision == 0)
                        rc = pvo_attend_unit_f64(qrow, Hq * D, kbuf, vbuf, n, c, D, scale,
                                                 p->dtype, orow, Hq * D, pr);
                    else
                        rc = pvo_attend_unit_f32(qrow, Hq * D, kbuf, vbuf, n, c, D, scale,
                                                 p->dtype, orow, Hq * D, pr);
                    if (rc != PVO_OK) {
#pragma omp critical
                        status = rc;
                    }
                }
            }
            free(kbuf);
            free(vbuf);
        }
    }
    if (threads_used) *threads_used = team;
    return status;
}

/*
 * Tier swapping (paper Section 4.3.2 "ahead-of-time swapping" and 4.3.3 "pipelined KV-cache
 * recovery"): KV-tokens leave the GPU pool for a CPU cache and come back in whole pages.  The
 * staging buffer holds, for the i-th listed page, that page's K image followed by its V image
 * (each num_kv_heads * page_size * head_dim 16-bit elements, exactly as they lie in the pools).
 * Pure copies.
 */
int pvo_pages_gather(const pvo_pool_desc *p, const uint16_t *k_pages, const uint16_t *v_pages,
                     const int32_t *page_ids, int32_t n, uint16_t *staging)
{
    if (!pvo_desc_ok(p) || n < 0) return PVO_BAD_ARG;
    const int64_t page_elems = (int64_t)p->num_kv_heads * p->page_size * p->head_dim;
    for (int32_t i = 0; i < n; ++i) {
        const int64_t page = page_ids[i];
        if (page < 0 || page >= p->num_pages) return PVO_BAD_PAGE;
        for (int64_t e = 0; e < page_elems; ++e) {
            staging[(2 * (int64_t)i) * page_elems + e] = k_pages[page * page_elems + e];
            staging[(2 * (int64_t)i + 1) * page_elems + e] = v_pages[page * page_elems + e];
        }
    }
    return PVO_OK;
}

int pvo_pages_scatter(const pvo_pool_desc *p, const uint16_t *staging, const int32_t *page_ids,
                      int32_t n, uint16_t *k_pages, uint16_t *v_pages)
{
    if (!pvo_desc_ok(p) || n < 0) return PVO_BAD_ARG;
    const int64_t page_elems = (int64_t)p->num_kv_heads * p->page_size * p->head_dim;
    for (int32_t i = 0; i < n; ++i) {
        const int64_t page = page_ids[i];
        if (page < 0 || page >= p->num_pages) return PVO_BAD_PAGE;
        for (int64_t e = 0; e < page_elems; ++e) {
            k_pages[page * page_elems + e] = staging[(2 * (int64_t)i) * page_elems + e];
            v_pages[page * page_elems + e] = staging[(2 * (int64_t)i + 1) * page_elems + e];
        }
    }
    return PVO_OK;
}

/*
 * Recomputation-cost model of the eviction policy (paper Section 4.3.1).  The cost of recomputing
 * a 32-token chunk whose attention spans a context of l tokens is Cost(l) = Cost_attention(l) + c,
 * with Cost_attention profiled at a few context sizes (powers of two) and interpolated in between
 * (linearly here; beyond the profiled range the nearest segment is extended); the retention value
 * of a chunk is V = Cost(l) / T with T the time since its conversation was last active, and chunks
 * are evicted in ascending order of V.
 */
double pvo_cost(const int32_t *ctx_points, const double *attn_cost, int32_t n, double c_other,
                int32_t l)
{
    if (n <= 0) return c_other;
    if (n == 1) return attn_cost[0] + c_other;
    int32_t k = 0; /* segment [k, k+1] used for l */
    while (k + 2 < n && l > ctx_points[k + 1]) ++k;
    const double x0 = ctx_points[k], x1 = ctx_points[k + 1];
    const double y0 = attn_cost[k], y1 = attn_cost[k + 1];
    return y0 + (y1 - y0) * ((double)l - x0) / (x1 - x0) + c_other;
}

/* order_out = chunk indices by ascending V = cost / idle_time (ties: lower index first). */
int pvo_retention_order(const double *cost, const double *idle_time, int32_t n, int32_t *order_out)
{
    if (n < 0) return PVO_BAD_ARG;
    for (int32_t i = 0; i < n; ++i) {
        if (!(idle_time[i] > 0.0)) return PVO_BAD_ARG;
        order_out[i] = i;
    }
    for (int32_t i = 1; i < n; ++i) { /* insertion sort: plain and stable */
        const int32_t cur = order_out[i];
        const double v = cost[cur] / idle_time[cur];
        int32_t j = i - 1;
        while (j >= 0 && cost[order_out[j]] / idle_time[order_out[j]] > v) {
            order_out[j + 1] = order_out[j];
            --j;
        }
        order_out[j + 1] = cur;
    }
    return PVO_OK;
}

/*
 * Rotary position embedding in front of the append: the producer of the new K rows (and of the
 * Q rows) in the Llama 2 models the paper serves (Section 6.1 names rotary embedding as one of
 * their features; Section 4.4.1 has the new K/V stored after the linear layers produce them).
 * The paper does not print the transform; it is the published RoFormer one: the head dimension
 * is split into D/2 pairs, pair i of a token at logical position t is rotated by the angle
 * t * theta_i with theta_i = base^(-2i/D).  Two pairings are in use and both are provided:
 *   style 0 (interleaved): pair i = elements (2i, 2i+1);
 *   style 1 (half split):  pair i = elements (i, i + D/2).
 *   out_a = a cos - b sin,   out_b = b cos + a sin.
 * The angles come from a table the caller passes in (float, [max_pos][D]: D/2 cosines then D/2
 * sines per position), so that the arithmetic checked here is the rotation itself; the table
 * generator below is the definition written out in double precision.
 */
int pvo_rope_table(double base, int32_t D, int32_t max_pos, float *table)
{
    if (!(base > 0.0) || D <= 0 || D % 2 != 0 || max_pos < 0 || !table) return PVO_BAD_ARG;
    for (int64_t t = 0; t < max_pos; ++t)
        for (int32_t i = 0; i < D / 2; ++i) {
            const double theta = pow(base, -2.0 * (double)i / (double)D);
            table[t * D + i] = (float)cos((double)t * theta);
            table[t * D + D / 2 + i] = (float)sin((double)t * theta);
        }
    return PVO_OK;
}

/* x: [rows, heads, D] 16-bit; pos: [rows]; out: [rows, heads, D] doubles, not rounded. */
int pvo_rope(const uint16_t *x, int64_t rows, int32_t heads, int32_t D, const int32_t *pos,
             const float *table, int32_t max_pos, int32_t style, int32_t dtype, double *out)
{
    if (rows < 0 || heads <= 0 || D <= 0 || D % 2 != 0 || (style != 0 && style != 1) ||
        (dtype != 0 && dtype != 1))
        return PVO_BAD_ARG;
    for (int64_t r = 0; r < rows; ++r) {
        if (pos[r] < 0 || pos[r] >= max_pos) return PVO_BAD_ARG;
        const float *cs = table + (int64_t)pos[r] * D;
        for (int32_t h = 0; h < heads; ++h) {
            const uint16_t *src = x + (r * heads + h) * D;
            double *dst = out + (r * heads + h) * D;
            for (int32_t i = 0; i < D / 2; ++i) {
                const int32_t ia = style == 0 ? 2 * i : i;
                const int32_t ib = style == 0 ? 2 * i + 1 : i + D / 2;
                const double a = pvo_widen(src[ia], dtype), b = pvo_widen(src[ib], dtype);
                const double c = (double)cs[i], s = (double)cs[D / 2 + i];
                dst[ia] = a * c - b * s;
                dst[ib] = b * c + a * s;
            }
        }
    }
    return PVO_OK;
}

/*
 * Round a double to the nearest value of a 16-bit format, ties to even (the rounding the
 * paper's 16-bit storage implies), and return its bit pattern.  p = significand bits including
 * the hidden one (11 / 8), emin = exponent of the smallest normal (-14 / -126), emax = exponent
 * of the largest finite value (15 / 127).
 */
static uint16_t pvo_round16_one(double v, int dtype)
{
    const int p = dtype == 0 ? 11 : 8, emin = dtype == 0 ? -14 : -126, emax = dtype == 0 ? 15 : 127;
    const int ebits = dtype == 0 ? 5 : 8, bias = dtype == 0 ? 15 : 127;
    const uint16_t sign = (uint16_t)(signbit(v) ? 0x8000u : 0u);
    const uint16_t inf = (uint16_t)(((1u << ebits) - 1u) << (p - 1));
    if (isnan(v)) return (uint16_t)(sign | inf | (1u << (p - 2)));
    double a = fabs(v);
    if (isinf(a)) return (uint16_t)(sign | inf);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e); /* a = f * 2^e, f in [0.5, 1)  ->  floor(log2 a) = e - 1 */
    int ex = e - 1;
    if (ex < emin) ex = emin; /* subnormal range shares the quantum of the smallest normal */
    const double quantum = ldexp(1.0, ex - (p - 1));
    double n = nearbyint(a / quantum); /* exact division; default rounding mode = ties to even */
    if (n >= ldexp(1.0, p)) { /* rounded up into the next binade */
        n /= 2.0;
        ex += 1;
    }
    if (ex > emax) return (uint16_t)(sign | inf);
    const uint32_t ni = (uint32_t)n;
    if (ni < (1u << (p - 1))) return (uint16_t)(sign | ni); /* subnormal (ex == emin) */
    return (uint16_t)(sign | ((uint32_t)(ex + bias) << (p - 1)) | (ni - (1u << (p - 1))));
}

int pvo_round16(const double *v, int64_t n, int32_t dtype, uint16_t *out)
{
    if (n < 0 || (dtype != 0 && dtype != 1)) return PVO_BAD_ARG;
    for (int64_t i = 0; i < n; ++i) out[i] = pvo_round16_one(v[i], dtype);
    return PVO_OK;
}
