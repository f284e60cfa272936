// Bandwidth-oriented attention kernel: work items of at most 16 query rows (generation steps,
// and the G query heads that share a KV head in grouped-query attention).
//
// Computes, for the rows of one item, paper Eq. 2-3 with the causal rule of Section 4.4 over the
// KV range of the item, reading K and V through the page table.  This is the "single-token"
// special case of Section 4.4.1 generalised to up to 16 rows so that a GQA group reads its K/V
// once.
//
// Mapping to gfx950.  One workgroup = 4 wavefronts = one item.  The wavefronts take the 32-key
// blocks (two pages) of the item's KV range round-robin; nothing is shared between them, so K and
// V go straight from HBM into registers in the lane order the matrix cores consume (the pool
// stores runs of 8 elements along the contracted dimension, 16 bytes = one lane's operand), with
// streaming (non-temporal) loads, since every byte is used once, and with the next block's loads in
// flight while the current one is processed.  Scores are produced
// transposed, S^T = K Q^T (16 keys x 16 rows per v_mfma_f32_16x16x32), so that every lane owns one
// query row: the softmax needs no cross-lane traffic beyond two exchanges for the running
// maximum, and the probabilities are already laid out as the B operand of O^T += V^T P^T.  The
// four partial (max, sum, O) triples are merged through LDS at the end.
#include "pv_device.h"

namespace pv {

template <typename T, int D>
struct NarrowFrag {
    u32x4 k[2][D / 32];  // [16-key tile][k-step]
    u32x4 v[D / 16];     // [16-wide block of d]
};

template <typename T, int D>
__global__ __launch_bounds__(256, 2) void attn_narrow_kernel(
    const WorkItem *__restrict__ items, const uint16_t *__restrict__ q,
    const uint16_t *__restrict__ k_pages, const uint16_t *__restrict__ v_pages,
    const int32_t *__restrict__ page_table, int32_t max_pages, int32_t num_q_heads,
    int32_t num_kv_heads, int32_t group, float scale_log2e, uint16_t *__restrict__ out,
    float *__restrict__ ws_o, float *__restrict__ ws_ml)
{
    constexpr int NW = 4;
    constexpr int KS = D / 32;
    constexpr int NB = D / 16;
    constexpr int OSTRIDE = D + 4;
    typedef typename T::vec8 vec8;
    __shared__ float sm_o[NW][16][OSTRIDE];
    __shared__ float sm_m[NW][16];
    __shared__ float sm_l[NW][16];

    const WorkItem it = items[blockIdx.x];
    const int lane = lane_id();
    const int w = wave_id();
    const int q16 = lane & 15;
    const int g = lane >> 4;

    const int row = it.row_begin + q16;
    const bool valid = q16 < it.row_count;
    const int tok = valid ? row / group : 0;
    const int hq = it.kv_head * group + (valid ? row % group : 0);
    // one past the last key this row may see (rows beyond the item are fed zeros, any limit works)
    const int vis_end = valid ? it.ctx + tok + 1 : it.kv_end;
    // every valid row sees all keys below this
    const int unmasked_end = it.ctx + it.row_begin / group + 1;

    vec8 qf[KS];
    {
        const uint16_t *qrow = q + ((int64_t)(it.q_row0 + tok) * num_q_heads + hq) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (valid) raw = load16(qrow + 32 * ks + 8 * g);
            qf[ks] = as_vec8<T>(raw);
        }
    }

    // lane-constant element offsets inside a (page, head) tile
    const int64_t tile_elems = 16 * D;
    int ksel[2], koff[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int key = 8 * (q16 >> 2) + 4 * t + (q16 & 3);  // key of S^T row q16 in tile t
        ksel[t] = key >> 4;
        koff[t] = (g * 16 + (key & 15)) * 8;  // + ks * 4 * 16 * 8
    }
    const int vsel = g >> 1;
    const int voff = ((g & 1) * D + q16) * 8;  // + blk * 16 * 8

    const int32_t *pt = page_table + (int64_t)it.req * max_pages;
    const int last_pg = (it.kv_end - 1) >> 4;
    const int pg0 = it.kv_begin >> 4;
    const int nblocks = (it.kv_end - it.kv_begin + 31) >> 5;

    auto load_block = [&](NarrowFrag<T, D> &f, int b) {
        const int pg = pg0 + 2 * b;
        const int64_t p0 = pt[pg];
        const int64_t p1 = pt[pg + 1 <= last_pg ? pg + 1 : last_pg];
        const int64_t base0 = (p0 * num_kv_heads + it.kv_head) * tile_elems;
        const int64_t base1 = (p1 * num_kv_heads + it.kv_head) * tile_elems;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint16_t *kb = k_pages + (ksel[t] ? base1 : base0) + koff[t];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) f.k[t][ks] = load16_stream(kb + ks * (4 * 16 * 8));
        }
        const uint16_t *vb = v_pages + (vsel ? base1 : base0) + voff;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) f.v[blk] = load16_stream(vb + blk * (16 * 8));
    };

    f32x4 o[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) o[blk] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;  // running maximum of the scaled scores (log2 domain)
    float l_run = 0.f;        // this lane's share of the running sum

    auto compute_block = [&](NarrowFrag<T, D> &f, int b) {
        const int kb0 = it.kv_begin + 32 * b;
        f32x4 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) s[t] = T::mfma16(as_vec8<T>(f.k[t][ks]), qf[ks], s[t]);
        }
        float x[8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) x[4 * t + bb] = s[t][bb] * scale_log2e;
        if (kb0 + 32 > unmasked_end) {  // block reaches the causal boundary or the end
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = kb0 + 8 * g + j;
                if (key >= vis_end) x[j] = -INFINITY;
            }
        }
        if (kb0 + 32 > it.kv_end) {  // slots past the end may hold anything: zero those V values
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int key = kb0 + 8 * g + 2 * jj;
                    uint32_t word = f.v[blk][jj];
                    if (key >= it.kv_end) word &= 0xFFFF0000u;
                    if (key + 1 >= it.kv_end) word &= 0x0000FFFFu;
                    f.v[blk][jj] = word;
                }
            }
        }
        float mx = x[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) mx = fmaxf(mx, x[j]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_safe);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = fast_exp2(x[j] - m_safe);
            psum += x[j];
        }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) o[blk] *= alpha;
        }
        u32x4 praw;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) praw[jj] = T::pack2(x[2 * jj], x[2 * jj + 1]);
        const vec8 pf = as_vec8<T>(praw);
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) o[blk] = T::mfma16(as_vec8<T>(f.v[blk]), pf, o[blk]);
    };

    {
        NarrowFrag<T, D> fa, fb;
        int b = w;
        if (b < nblocks) load_block(fa, b);
        while (b < nblocks) {
            int nxt = b + NW;
            if (nxt < nblocks) load_block(fb, nxt);
            compute_block(fa, b);
            b = nxt;
            if (b >= nblocks) break;
            nxt = b + NW;
            if (nxt < nblocks) load_block(fa, nxt);
            compute_block(fb, b);
            b = nxt;
        }
    }

    // ---- merge the four wavefronts ----
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (g == 0) {
        sm_m[w][q16] = m_run;
        sm_l[w][q16] = l_tot;
    }
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
        *reinterpret_cast<f32x4 *>(&sm_o[w][q16][16 * blk + 4 * g]) = o[blk];
    __syncthreads();

    constexpr int PER = D / 16;  // output elements per thread
    const int r16 = (int)threadIdx.x >> 4;
    const int d0 = ((int)threadIdx.x & 15) * PER;
    if (r16 >= it.row_count) return;
    float mw[NW], wgt[NW];
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        mw[i] = sm_m[i][r16];
        M = fmaxf(M, mw[i]);
    }
    const float M_safe = M == -INFINITY ? 0.f : M;
    float L = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        wgt[i] = fast_exp2(mw[i] - M_safe);
        L += wgt[i] * sm_l[i][r16];
    }
    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        float a = 0.f;
#pragma unroll
        for (int i = 0; i < NW; ++i) a += wgt[i] * sm_o[i][r16][d0 + e];
        acc[e] = a;
    }
    const int orow = it.row_begin + r16;
    if (it.split_count == 1) {
        const float inv = 1.f / L;
        const int otok = orow / group;
        const int ohq = it.kv_head * group + orow % group;
        uint16_t *dst = out + ((int64_t)(it.q_row0 + otok) * num_q_heads + ohq) * D + d0;
        uint32_t packed[PER / 2];
#pragma unroll
        for (int e = 0; e < PER / 2; ++e)
            packed[e] = T::pack2(acc[2 * e] * inv, acc[2 * e + 1] * inv);
        if constexpr (PER == 8) {
            *reinterpret_cast<u32x4 *>(dst) = u32x4{packed[0], packed[1], packed[2], packed[3]};
        } else {
            *reinterpret_cast<u32x2 *>(dst) = u32x2{packed[0], packed[1]};
        }
    } else {
        const int64_t slot = (int64_t)it.partial_base + r16;
        float *po = ws_o + slot * D + d0;
#pragma unroll
        for (int e = 0; e < PER; e += 4)
            *reinterpret_cast<f32x4 *>(po + e) = f32x4{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
        if (((int)threadIdx.x & 15) == 0) {
            ws_ml[2 * slot] = M;
            ws_ml[2 * slot + 1] = L;
        }
    }
}

// Merge of split-KV partial results: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One workgroup = 8 rows of one split item (32 threads per row, D/32 output elements each).
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(
    const CombineChunk *__restrict__ chunks, const CombineItem *__restrict__ items,
    const float *__restrict__ ws_o, const float *__restrict__ ws_ml, int32_t num_q_heads,
    int32_t group, uint16_t *__restrict__ out)
{
    constexpr int PER = D / 32;
    const CombineChunk ch = chunks[blockIdx.x];
    const CombineItem it = items[ch.item];
    const int r = ch.row0 + ((int)threadIdx.x >> 5);
    if (r >= it.row_count) return;
    const int d0 = ((int)threadIdx.x & 31) * PER;
    float M = -INFINITY;
    for (int s = 0; s < it.split_count; ++s) {
        const int64_t slot = (int64_t)it.partial_base + (int64_t)s * it.row_count + r;
        M = fmaxf(M, ws_ml[2 * slot]);
    }
    const float M_safe = M == -INFINITY ? 0.f : M;
    float L = 0.f;
    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;
    for (int s = 0; s < it.split_count; ++s) {
        const int64_t slot = (int64_t)it.partial_base + (int64_t)s * it.row_count + r;
        const float wgt = fast_exp2(ws_ml[2 * slot] - M_safe);
        L += wgt * ws_ml[2 * slot + 1];
        const float *po = ws_o + slot * D + d0;
#pragma unroll
        for (int e = 0; e < PER; ++e) acc[e] += wgt * po[e];
    }
    const float inv = 1.f / L;
    const int orow = it.row_begin + r;
    const int otok = orow / group;
    const int ohq = it.kv_head * group + orow % group;
    uint16_t *dst = out + ((int64_t)(it.q_row0 + otok) * num_q_heads + ohq) * D + d0;
    if constexpr (PER == 4) {
        *reinterpret_cast<u32x2 *>(dst) =
            u32x2{T::pack2(acc[0] * inv, acc[1] * inv), T::pack2(acc[2] * inv, acc[3] * inv)};
    } else {
        *reinterpret_cast<uint32_t *>(dst) = T::pack2(acc[0] * inv, acc[1] * inv);
    }
}

template <typename T, int D>
static hipError_t launch_narrow_t(const pv_plan *plan, const DeviceLists &dl, const void *q, const void *k_pages,
                                  const void *v_pages, const int32_t *page_table, float scale,
                                  void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    const int n = (int)plan->narrow.size();
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL((attn_narrow_kernel<T, D>), dim3(n), dim3(256), 0, stream, dl.narrow,
                       (const uint16_t *)q, (const uint16_t *)k_pages, (const uint16_t *)v_pages,
                       page_table, plan->max_pages_per_req, plan->num_q_heads,
                       plan->pool.num_kv_heads, plan->group, scale * kLog2e, (uint16_t *)out, ws_o,
                       ws_ml);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_combine_t(const pv_plan *plan, const DeviceLists &dl, const float *ws_o, const float *ws_ml,
                                   void *out, hipStream_t stream)
{
    const int n = (int)plan->combine_chunks.size();
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL((attn_combine_kernel<T, D>), dim3(n), dim3(256), 0, stream,
                       dl.combine_chunks, dl.combine, ws_o, ws_ml, plan->num_q_heads,
                       plan->group, (uint16_t *)out);
    return hipGetLastError();
}

hipError_t launch_attn_narrow(const pv_plan *plan, const DeviceLists &dl, const void *q, const void *k_pages,
                              const void *v_pages, const int32_t *page_table, float scale,
                              void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    const bool h = plan->pool.dtype == PV_F16;
    if (plan->pool.head_dim == 128)
        return h ? launch_narrow_t<F16, 128>(plan, dl, q, k_pages, v_pages, page_table, scale, out,
                                             ws_o, ws_ml, stream)
                 : launch_narrow_t<BF16, 128>(plan, dl, q, k_pages, v_pages, page_table, scale, out,
                                              ws_o, ws_ml, stream);
    return h ? launch_narrow_t<F16, 64>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                        ws_ml, stream)
             : launch_narrow_t<BF16, 64>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                         ws_ml, stream);
}

hipError_t launch_attn_combine(const pv_plan *plan, const DeviceLists &dl, const float *ws_o, const float *ws_ml,
                               void *out, hipStream_t stream)
{
    const bool h = plan->pool.dtype == PV_F16;
    if (plan->pool.head_dim == 128)
        return h ? launch_combine_t<F16, 128>(plan, dl, ws_o, ws_ml, out, stream)
                 : launch_combine_t<BF16, 128>(plan, dl, ws_o, ws_ml, out, stream);
    return h ? launch_combine_t<F16, 64>(plan, dl, ws_o, ws_ml, out, stream)
             : launch_combine_t<BF16, 64>(plan, dl, ws_o, ws_ml, out, stream);
}

}  // namespace pv
