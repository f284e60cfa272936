// Rotary position embedding fused with the KV append: the producer step in front of the hot path
// for the Llama 2 models of the paper (Section 6.1 lists rotary embedding among their features;
// Section 4.4.1: the linear layers produce each token's Q/K/V, the new K/V are stored in their
// slots, then attention runs).  One launch rotates the new K rows and stores them in the pool,
// stores the new V rows, and rotates the Q rows, instead of a rotary pass over Q and K followed by
// the append.
//
// The transform is the published RoFormer one: pair i of a head, for a token at logical position
// t, is rotated by t * theta_i.  cos / sin come from a table [max_pos][D] (D/2 cosines, then D/2
// sines) that the caller computes once (pv_rope_table).  Pairing: style 0 = elements (2i, 2i+1),
// style 1 = elements (i, i + D/2).  The rotation is evaluated in fp32 and rounded to the 16-bit
// type (nearest even); V is moved bit for bit.
//
// Grid: (append groups, Hkv + Hq) with D threads.  y < Hkv: KV head y (K rotated + scattered, V
// scattered as in kv_append_kernel); y >= Hkv: query head y - Hkv of the group's tokens.
#include "pv_device.h"

namespace pv {

template <typename T>
__device__ __forceinline__ void unpack8(u32x4 raw, float (&x)[8])
{
    const typename T::vec8 v = as_vec8<T>(raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)v[e];
}

template <typename T>
__device__ __forceinline__ u32x4 pack8(const float (&x)[8])
{
    return u32x4{T::pack2(x[0], x[1]), T::pack2(x[2], x[3]), T::pack2(x[4], x[5]),
                 T::pack2(x[6], x[7])};
}

template <typename T, int D, int STYLE>
__global__ __launch_bounds__(D) void rope_append_kernel(
    const AppendGroup *__restrict__ groups, const uint16_t *q_in,
    uint16_t *q_out /* may be q_in */, const uint16_t *__restrict__ k_new,
    const uint16_t *__restrict__ v_new, const float *__restrict__ cos_sin,
    const int32_t *__restrict__ page_table, int32_t max_pages, int32_t num_q_heads,
    int32_t num_kv_heads, uint16_t *__restrict__ k_pages, uint16_t *__restrict__ v_pages)
{
    constexpr int CH = D / 8;
    const AppendGroup g = groups[blockIdx.x];
    const int y = (int)blockIdx.y;
    const int t = (int)threadIdx.x;
    const bool is_q = y >= num_kv_heads;
    const int head = is_q ? y - num_kv_heads : y;
    const int64_t row_stride = (int64_t)(is_q ? num_q_heads : num_kv_heads) * D;
    const uint16_t *src = (is_q ? q_in : k_new) + (int64_t)g.q_row * row_stride + (int64_t)head * D;

    int64_t tile = 0;
    int slot0 = 0;
    if (!is_q) {
        const int64_t page = page_table[(int64_t)g.req * max_pages + (g.t_begin >> 4)];
        slot0 = g.t_begin & 15;
        tile = (page * num_kv_heads + head) * (int64_t)(16 * D);
    }
    // destination of the 16-byte chunk c8 of token j
    auto store_chunk = [&](int j, int c8, u32x4 val) {
        if (is_q)
            *reinterpret_cast<u32x4 *>(q_out + (int64_t)(g.q_row + j) * row_stride +
                                       (int64_t)head * D + 8 * c8) = val;
        else
            *reinterpret_cast<u32x4 *>(k_pages + tile + (c8 * 16 + slot0 + j) * 8) = val;
    };

    if constexpr (STYLE == 0) {
        // one thread per (token j, chunk c8): 4 pairs inside the chunk
        const int j = t / CH, c8 = t % CH;
        if (j < g.count) {
            const float *cs = cos_sin + (int64_t)(g.t_begin + j) * D;
            const f32x4 c = *reinterpret_cast<const f32x4 *>(cs + 4 * c8);
            const f32x4 s = *reinterpret_cast<const f32x4 *>(cs + D / 2 + 4 * c8);
            float x[8], o[8];
            unpack8<T>(load16(src + j * row_stride + 8 * c8), x);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                o[2 * p] = x[2 * p] * c[p] - x[2 * p + 1] * s[p];
                o[2 * p + 1] = x[2 * p + 1] * c[p] + x[2 * p] * s[p];
            }
            store_chunk(j, c8, pack8<T>(o));
        }
    } else {
        // one thread per (token j, chunk c8 of the first half): its partner chunk is c8 + CH/2
        const int j = t / (CH / 2), c8 = t % (CH / 2);
        if (t < 8 * (CH / 2) && j < g.count) {
            const float *cs = cos_sin + (int64_t)(g.t_begin + j) * D;
            float xa[8], xb[8], oa[8], ob[8];
            unpack8<T>(load16(src + j * row_stride + 8 * c8), xa);
            unpack8<T>(load16(src + j * row_stride + 8 * c8 + D / 2), xb);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const f32x4 c = *reinterpret_cast<const f32x4 *>(cs + 8 * c8 + 4 * half);
                const f32x4 s = *reinterpret_cast<const f32x4 *>(cs + D / 2 + 8 * c8 + 4 * half);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * half + e;
                    oa[i] = xa[i] * c[e] - xb[i] * s[e];
                    ob[i] = xb[i] * c[e] + xa[i] * s[e];
                }
            }
            store_chunk(j, c8, pack8<T>(oa));
            store_chunk(j, c8 + CH / 2, pack8<T>(ob));
        }
    }

    if (!is_q) {
        // V: thread -> head dimension d = t, moved bit for bit
        const uint16_t *vsrc = v_new + (int64_t)g.q_row * row_stride + (int64_t)head * D;
        scatter_v_group<D>(vsrc, row_stride, g.count, slot0, t, v_pages + tile);
    }
}

template <typename T, int D>
static hipError_t launch_rope_t(const pv_plan *plan, const DeviceLists &dl, int style, const void *q_in, void *q_out,
                                const void *k_new, const void *v_new, const float *cos_sin,
                                const int32_t *page_table, void *k_pages, void *v_pages,
                                hipStream_t stream)
{
    const unsigned heads = (unsigned)plan->pool.num_kv_heads + (q_in ? (unsigned)plan->num_q_heads : 0u);
    const dim3 grid((unsigned)plan->append_groups.size(), heads);
    if (style == 0)
        hipLaunchKernelGGL((rope_append_kernel<T, D, 0>), grid, dim3(D), 0, stream,
                           dl.append_groups, (const uint16_t *)q_in, (uint16_t *)q_out,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, cos_sin, page_table,
                           plan->max_pages_per_req, plan->num_q_heads, plan->pool.num_kv_heads,
                           (uint16_t *)k_pages, (uint16_t *)v_pages);
    else
        hipLaunchKernelGGL((rope_append_kernel<T, D, 1>), grid, dim3(D), 0, stream,
                           dl.append_groups, (const uint16_t *)q_in, (uint16_t *)q_out,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, cos_sin, page_table,
                           plan->max_pages_per_req, plan->num_q_heads, plan->pool.num_kv_heads,
                           (uint16_t *)k_pages, (uint16_t *)v_pages);
    return hipGetLastError();
}

hipError_t launch_rope_append(const pv_plan *plan, const DeviceLists &dl, int style, const void *q_in, void *q_out,
                              const void *k_new, const void *v_new, const float *cos_sin,
                              const int32_t *page_table, void *k_pages, void *v_pages,
                              hipStream_t stream)
{
    if (plan->append_groups.empty()) return hipSuccess;
    const bool f = plan->pool.dtype == PV_F16;
    if (plan->pool.head_dim == 128)
        return f ? launch_rope_t<F16, 128>(plan, dl, style, q_in, q_out, k_new, v_new, cos_sin,
                                           page_table, k_pages, v_pages, stream)
                 : launch_rope_t<BF16, 128>(plan, dl, style, q_in, q_out, k_new, v_new, cos_sin,
                                            page_table, k_pages, v_pages, stream);
    return f ? launch_rope_t<F16, 64>(plan, dl, style, q_in, q_out, k_new, v_new, cos_sin, page_table,
                                      k_pages, v_pages, stream)
             : launch_rope_t<BF16, 64>(plan, dl, style, q_in, q_out, k_new, v_new, cos_sin, page_table,
                                       k_pages, v_pages, stream);
}

}  // namespace pv
