// Matrix-core attention kernel: work items of up to 128 query rows (new-prompt tokens, times the
// query heads of a GQA group) that share one KV head's K/V stream.
//
// Computes paper Eq. 2-3 with the causal rule of Section 4.4 for the rows of one item over the
// item's KV range, reading K and V through the page table: the "two matrix-matrix
// multiplications" with fused mask of Section 4.4, fused flash-style so that the score matrix is
// never materialised.
//
// Mapping to gfx950.  One workgroup = 4 wavefronts = one item; wavefront w owns rows 32w..32w+31.
// The K/V page tiles of a 32-key block (two pages) are copied from HBM into LDS once per workgroup
// (16 bytes per lane, fully coalesced: a (page, head) tile is contiguous in the pool) and every
// wavefront reads its matrix-core operands from there, so the tile is shared by all 128 rows.  The
// pool keeps runs of 8 elements along the contracted dimension together, so a plain linear copy
// already puts the operands where 16 consecutive lanes read 256 consecutive bytes (no bank
// conflicts, no padding, no transposes).  Scores are produced transposed, S^T = K Q^T
// (v_mfma_f32_32x32x16), so each lane owns one query row (softmax without cross-lane traffic except
// one exchange for the maximum) and the probabilities are already the B operand of
// O^T += V^T P^T.  The next block's global loads are in flight while the current one is computed;
// LDS is double-buffered with one barrier per block.
#include "pv_device.h"

namespace pv {

template <typename T, int D>
__global__ __launch_bounds__(256, 2) void attn_wide_kernel(
    const WorkItem *__restrict__ items, const uint16_t *__restrict__ q,
    const uint16_t *__restrict__ k_pages, const uint16_t *__restrict__ v_pages,
    const int32_t *__restrict__ page_table, int32_t max_pages, int32_t num_q_heads,
    int32_t num_kv_heads, int32_t group, float scale_log2e, uint16_t *__restrict__ out,
    float *__restrict__ ws_o, float *__restrict__ ws_ml)
{
    constexpr int KS = D / 16;                // k-steps of S^T = K Q^T
    constexpr int NB = D / 32;                // 32-wide blocks of d in O^T
    constexpr int TILE_BYTES = 16 * D * 2;    // one (page, head) tile
    constexpr int HALF_BYTES = 2 * TILE_BYTES;  // K (or V) part of a stage: two pages
    constexpr int PASSES = HALF_BYTES / 4096;   // 16-byte loads per thread for K (same for V)
    typedef typename T::vec8 vec8;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2][2 * HALF_BYTES];

    const WorkItem it = items[blockIdx.x];
    const int tid = (int)threadIdx.x;
    const int lane = lane_id();
    const int w = wave_id();
    const int q32 = lane & 31;
    const int h = lane >> 5;

    const int row = it.row_begin + 32 * w + q32;
    const bool valid = 32 * w + q32 < it.row_count;
    const int tok = valid ? row / group : 0;
    const int hq = it.kv_head * group + (valid ? row % group : 0);
    const int vis_end = valid ? it.ctx + tok + 1 : it.kv_end;
    // wavefront-uniform limits: below unmasked_end nothing is masked for this wavefront's rows;
    // at or beyond wave_end nothing is visible to them
    const int wave_rows = it.row_count - 32 * w;  // may be <= 0
    const int unmasked_end = it.ctx + (it.row_begin + 32 * w) / group + 1;
    int wave_end = 0;
    if (wave_rows > 0) {
        const int last = it.row_begin + 32 * w + (wave_rows < 32 ? wave_rows : 32) - 1;
        wave_end = it.ctx + last / group + 1;
        if (wave_end > it.kv_end) wave_end = it.kv_end;
    }

    vec8 qf[KS];
    {
        const uint16_t *qrow = q + ((int64_t)(it.q_row0 + tok) * num_q_heads + hq) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (valid) raw = load16(qrow + 16 * ks + 8 * h);
            qf[ks] = as_vec8<T>(raw);
        }
    }

    // LDS byte offsets of this lane's operands inside a stage
    const int key = (q32 & 0x13) | ((q32 & 4) << 1) | ((q32 & 8) >> 1);  // bits 2 and 3 swapped
    const int k_lds = (key >> 4) * TILE_BYTES + (h * 16 + (key & 15)) * 16;  // + ks * 512
    const int v_lds = HALF_BYTES + (h * D + q32) * 16;  // + page * TILE_BYTES + blk * 512

    const int32_t *pt = page_table + (int64_t)it.req * max_pages;
    const int last_pg = (it.kv_end - 1) >> 4;
    const int pg0 = it.kv_begin >> 4;
    const int nblocks = (it.kv_end - it.kv_begin + 31) >> 5;
    const int64_t head_off = (int64_t)it.kv_head * (16 * D);
    const int64_t page_stride = (int64_t)num_kv_heads * (16 * D);

    u32x4 stage_k[PASSES], stage_v[PASSES];
    auto global_load = [&](int b) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int off = p * 4096 + tid * 16;       // byte offset inside the K (or V) half
            const int pg_in = off / TILE_BYTES;         // 0 or 1
            int pg = pg0 + 2 * b + pg_in;
            pg = pg <= last_pg ? pg : last_pg;
            const int64_t elem = (int64_t)pt[pg] * page_stride + head_off + (off % TILE_BYTES) / 2;
            stage_k[p] = load16(k_pages + elem);
            stage_v[p] = load16(v_pages + elem);
        }
    };
    auto lds_store = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int off = p * 4096 + tid * 16;
            *reinterpret_cast<u32x4 *>(&smem[buf][off]) = stage_k[p];
            *reinterpret_cast<u32x4 *>(&smem[buf][HALF_BYTES + off]) = stage_v[p];
        }
    };

    f32x16 o[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[blk][v] = 0.f;
    float m_run = -INFINITY;
    float l_run = 0.f;

    auto compute_block = [&](int buf, int b) {
        const int kb0 = it.kv_begin + 32 * b;
        const unsigned char *sb = smem[buf];
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 kf = *reinterpret_cast<const u32x4 *>(sb + k_lds + ks * 512);
            s = T::mfma32(as_vec8<T>(kf), qf[ks], s);
        }
        float x[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) x[v] = s[v] * scale_log2e;
        if (kb0 + 32 > unmasked_end) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                // register v = 8*page + 4*a0 + b  <->  key kb0 + 16*page + 8*h + 4*a0 + b
                const int kk = kb0 + 16 * (v >> 3) + 8 * h + (v & 7);
                if (kk >= vis_end) x[v] = -INFINITY;
            }
        }
        float mx = x[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, x[v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_safe);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            x[v] = fast_exp2(x[v] - m_safe);
            psum += x[v];
        }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) o[blk] *= alpha;
        }
        const bool tail = kb0 + 32 > it.kv_end;  // slots past the end may hold anything
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            u32x4 praw;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                praw[jj] = T::pack2(x[8 * pg + 2 * jj], x[8 * pg + 2 * jj + 1]);
            const vec8 pf = as_vec8<T>(praw);
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                u32x4 vf = *reinterpret_cast<const u32x4 *>(sb + v_lds + pg * TILE_BYTES + blk * 512);
                if (tail) {
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int kk = kb0 + 16 * pg + 8 * h + 2 * jj;
                        uint32_t word = vf[jj];
                        if (kk >= it.kv_end) word &= 0xFFFF0000u;
                        if (kk + 1 >= it.kv_end) word &= 0x0000FFFFu;
                        vf[jj] = word;
                    }
                }
                o[blk] = T::mfma32(as_vec8<T>(vf), pf, o[blk]);
            }
        }
    };

    global_load(0);
    lds_store(0);
    __syncthreads();
    for (int b = 0; b < nblocks; ++b) {
        const bool more = b + 1 < nblocks;
        if (more) global_load(b + 1);
        if (it.kv_begin + 32 * b < wave_end) compute_block(b & 1, b);
        if (more) lds_store((b + 1) & 1);
        __syncthreads();
    }

    // ---- finish: every lane owns one row; the two half-waves hold partial sums ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!valid) return;
    if (it.split_count == 1) {
        const float inv = 1.f / l_tot;
        uint16_t *dst = out + ((int64_t)(it.q_row0 + tok) * num_q_heads + hq) * D;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int d = 32 * blk + 8 * a + 4 * h;
                *reinterpret_cast<u32x2 *>(dst + d) =
                    u32x2{T::pack2(o[blk][4 * a] * inv, o[blk][4 * a + 1] * inv),
                          T::pack2(o[blk][4 * a + 2] * inv, o[blk][4 * a + 3] * inv)};
            }
    } else {
        const int64_t slot = (int64_t)it.partial_base + 32 * w + q32;
        float *po = ws_o + slot * D;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int d = 32 * blk + 8 * a + 4 * h;
                *reinterpret_cast<f32x4 *>(po + d) = f32x4{o[blk][4 * a], o[blk][4 * a + 1],
                                                           o[blk][4 * a + 2], o[blk][4 * a + 3]};
            }
        if (h == 0) {
            ws_ml[2 * slot] = m_run;
            ws_ml[2 * slot + 1] = l_tot;
        }
    }
}

template <typename T, int D>
static hipError_t launch_wide_t(const pv_plan *plan, const void *q, const void *k_pages,
                                const void *v_pages, const int32_t *page_table, float scale,
                                void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    const int n = (int)plan->wide.size();
    hipLaunchKernelGGL((attn_wide_kernel<T, D>), dim3(n), dim3(256), 0, stream, plan->d_wide,
                       (const uint16_t *)q, (const uint16_t *)k_pages, (const uint16_t *)v_pages,
                       page_table, plan->max_pages_per_req, plan->num_q_heads,
                       plan->pool.num_kv_heads, plan->group, scale * kLog2e, (uint16_t *)out, ws_o,
                       ws_ml);
    return hipGetLastError();
}

hipError_t launch_attn_wide(const pv_plan *plan, const void *q, const void *k_pages,
                            const void *v_pages, const int32_t *page_table, float scale, void *out,
                            float *ws_o, float *ws_ml, hipStream_t stream)
{
    if (plan->wide.empty()) return hipSuccess;
    const bool f = plan->pool.dtype == PV_F16;
    if (plan->pool.head_dim == 128)
        return f ? launch_wide_t<F16, 128>(plan, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                           ws_ml, stream)
                 : launch_wide_t<BF16, 128>(plan, q, k_pages, v_pages, page_table, scale, out,
                                            ws_o, ws_ml, stream);
    return f ? launch_wide_t<F16, 64>(plan, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                      ws_ml, stream)
             : launch_wide_t<BF16, 64>(plan, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                       ws_ml, stream);
}

}  // namespace pv
