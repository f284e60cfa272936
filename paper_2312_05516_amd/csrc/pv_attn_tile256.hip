// Matrix-core attention kernel for long multi-token work: items of exactly 256 query rows (new
// tokens times the query heads of a GQA group) that share one KV head's K/V stream.
//
// Computes paper Eq. 2-3 with the causal rule of Section 4.4 for the rows of one item over the
// item's KV range, reading K and V through the page table (the pair of fused matrix products of
// Section 4.4, never materialising the scores).  Same operand layouts and transposed-score scheme
// as attn_wide_kernel; what differs is how the work is laid over a compute unit, chosen for the
// case that dominates long histories (hundreds of 32-key blocks per item):
//
//  * One workgroup per CU, 4 wavefronts, one per SIMD with the whole register file (512 registers
//    per lane).  A wavefront owns 64 rows as two 32-row sub-tiles that share every K and V operand
//    it reads from LDS, so each LDS byte feeds two matrix-core instructions (half the LDS reads per
//    flop) and a K/V tile fetched from L2 serves 256 rows (half the L2 -> LDS traffic per flop of
//    the 128-row kernel).  On this chip long matrix-core kernels run against the power limit, so
//    data movement saved is clock frequency gained.
//  * Software pipeline inside the wavefront: iteration b issues, in one basic block, the score
//    product of block b+1 (16 matrix-core instructions), the exponentials of block b (vector ALU)
//    and the value product of block b (16 more), so the matrix cores and the vector ALU of the SIMD
//    overlap without relying on other wavefronts.  The rare running-maximum update (lazy, as in
//    attn_wide_kernel) is a branch at the end of the iteration and works on block b+1's scores.
//  * K/V page tiles go HBM/L2 -> LDS directly (global_load_lds) into a ring of 8 stages, six blocks
//    ahead; one s_barrier per block.  K operands of block b+2 are requested before the barrier at
//    the end of iteration b, so they are in registers when iteration b+1 starts.
//
// Blocks that touch the causal boundary or the end of the sequence run in a second, masked loop
// with the same barrier protocol, so the wavefronts of a workgroup stay in step.
#include <type_traits>

#include "pv_device.h"

namespace pv {

template <typename T>
__global__ __launch_bounds__(256, 1) void attn_tile256_kernel(
    const WorkItem *__restrict__ items, const uint16_t *__restrict__ q,
    const uint16_t *__restrict__ k_pages, const uint16_t *__restrict__ v_pages,
    const int32_t *__restrict__ page_table, int32_t max_pages, int32_t num_q_heads,
    int32_t num_kv_heads, int32_t group, float scale_log2e, uint32_t q_sign,
    uint16_t *__restrict__ out, float *__restrict__ ws_o, float *__restrict__ ws_ml)
{
    constexpr int D = 128;
    constexpr int SUB = 2;                      // 32-row sub-tiles per wavefront
    constexpr int BK = 32;                      // keys per block
    constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T
    constexpr int NB = D / 32;                  // 32-wide blocks of d in O^T
    constexpr int TILE_BYTES = 16 * D * 2;      // one (page, head) tile
    constexpr int HALF_BYTES = 2 * TILE_BYTES;  // K (or V) part of a stage: two pages
    constexpr int STAGE_BYTES = 2 * HALF_BYTES;
    constexpr int STAGES = 8;
    constexpr int PF = 6;                       // blocks the copies run ahead of their use
    constexpr int LOADS = STAGE_BYTES / 1024 / 4;  // 1 KiB copies per wavefront per block
    typedef typename T::vec8 vec8;
    __shared__ __attribute__((aligned(16))) unsigned char smem[STAGES][STAGE_BYTES];

    const WorkItem it = items[blockIdx.x];
    const int lane = lane_id();
    const int w = wave_id();
    const int q32 = lane & 31;
    const int h = lane >> 5;

    // every row of the item exists (the plan only makes full 256-row items for this kernel)
    int tok[SUB], hq[SUB], vis_end[SUB];
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
        const int row = it.row_begin + 32 * (SUB * w + u) + q32;
        tok[u] = row / group;
        hq[u] = it.kv_head * group + row % group;
        vis_end[u] = it.ctx + tok[u] + 1;
    }
    // wavefront-uniform limits: below unmasked_end nothing is masked for this wavefront's rows
    // (and no slot is past the end); at or beyond wave_end nothing is visible to them
    const int first_row = it.row_begin + 32 * SUB * w;
    int unmasked_end = it.ctx + first_row / group + 1;
    if (unmasked_end > it.kv_end) unmasked_end = it.kv_end;
    int wave_end = it.ctx + (first_row + 32 * SUB - 1) / group + 1;
    if (wave_end > it.kv_end) wave_end = it.kv_end;

    vec8 qf[SUB][KS];
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
        const uint16_t *qrow = q + ((int64_t)(it.q_row0 + tok[u]) * num_q_heads + hq[u]) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = load16(qrow + 16 * ks + 8 * h);
            raw ^= q_sign;  // a negative scale is applied as |scale| on negated queries
            qf[u][ks] = as_vec8<T>(raw);
        }
    }

    // LDS byte offsets of this lane's operands inside a stage (see attn_wide_kernel): S^T row i of
    // the K operand is fed with key pi(i) (bits 2 and 3 of i swapped), so that the accumulator
    // registers of S^T, in order, are the 8 consecutive keys the P^T operand needs.
    const int key = (q32 & 0x13) | ((q32 & 4) << 1) | ((q32 & 8) >> 1);
    const int k_lds = (key >> 4) * TILE_BYTES + (h * 16 + (key & 15)) * 16;  // + ks * 512
    const int v_lds = HALF_BYTES + (h * D + q32) * 16;  // + page * TILE_BYTES + blk * 512

    const int32_t *pt = page_table + (int64_t)it.req * max_pages;
    const int last_pg = (it.kv_end - 1) >> 4;
    const int pg0 = it.kv_begin >> 4;
    const int nblocks = (it.kv_end - it.kv_begin + BK - 1) / BK;
    const int64_t head_off = (int64_t)it.kv_head * (16 * D);
    const int64_t page_stride = (int64_t)num_kv_heads * (16 * D);
    const uint32_t lane_bytes = (uint32_t)lane * 16u;

    // page ids of a block (two pages; a page past the end is never used, so any valid id will do)
    auto page_ids = [&](int b, int &id0, int &id1) {
        const int pg = pg0 + 2 * b;
        id0 = pt[pg <= last_pg ? pg : last_pg];
        id1 = pt[pg + 1 <= last_pg ? pg + 1 : last_pg];
    };
    // asynchronous copy of block b into stage b % STAGES: the stage is 16 pieces of 1 KiB (K page
    // 0, K page 1, V page 0, V page 1, four pieces each); wavefront w moves pieces w, w+4, w+8, w+12
    auto dma_block = [&](int b, int id0, int id1) {
        unsigned char *stage = smem[b % STAGES];
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int off = (w + 4 * i) * 1024;  // wavefront-uniform offset inside the stage
            const bool is_v = off >= HALF_BYTES;
            const int hoff = off % HALF_BYTES;
            const int page = hoff / TILE_BYTES ? id1 : id0;
            const int64_t elem = (int64_t)page * page_stride + head_off + (hoff % TILE_BYTES) / 2;
            lds_dma16((is_v ? v_pages : k_pages) + elem, lane_bytes, stage + off);
        }
    };

    f32x16 o[SUB][NB];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[u][blk][v] = 0.f;
    float m_run[SUB], l_run[SUB], mc[SUB];
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
        m_run[u] = -INFINITY;  // reference maximum of the RAW scores (before scaling)
        l_run[u] = 0.f;        // this lane's share of the running sum
        mc[u] = 0.f;           // m_run in the exp2 domain (0 while there is no reference yet)
    }

    u32x4 kf[KS];  // K operands of the block whose scores are computed next
    auto read_k = [&](int b) {
        const unsigned char *sb = smem[b % STAGES];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            kf[ks] = *reinterpret_cast<const u32x4 *>(sb + k_lds + ks * 512);
    };
    // S^T of the block whose K operands are in kf, both sub-tiles (they share the operands)
    auto scores = [&](f32x16 (&sn)[SUB]) {
#pragma unroll
        for (int u = 0; u < SUB; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) sn[u][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int u = 0; u < SUB; ++u) sn[u] = T::mfma32(as_vec8<T>(kf[ks]), qf[u][ks], sn[u]);
    };
    // register v = 8*page + j of S^T  <->  key kb0 + 16*page + 8*h + j
    auto key_of = [&](int kb0, int v) { return kb0 + 16 * (v >> 3) + 8 * h + (v & 7); };

    // Lazy reference maximum (exact, softmax is shift-invariant): it only moves when a score of
    // the coming block exceeds it by more than 2^kLazyLog2 in the scaled domain, so rescaling the
    // accumulators is rare.  Works on the scores of the block that the NEXT softmax will consume.
    auto update_reference = [&](const f32x16 (&sn)[SUB], int kb0, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        float mx[SUB];
        bool grow = false;
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            mx[u] = -INFINITY;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float x = sn[u][v];
                if constexpr (MASKED)
                    if (key_of(kb0, v) >= vis_end[u]) x = -INFINITY;
                mx[u] = fmaxf(mx[u], x);
            }
            grow = grow || m_run[u] == -INFINITY || (mx[u] - m_run[u]) * scale_log2e > kLazyLog2;
        }
        if (__any(grow)) {
#pragma unroll
            for (int u = 0; u < SUB; ++u) {
                const float mxx = fmaxf(mx[u], __shfl_xor(mx[u], 32));
                const float m_new = (m_run[u] == -INFINITY ||
                                     (mxx - m_run[u]) * scale_log2e > kLazyLog2)
                                        ? mxx
                                        : m_run[u];
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                const float alpha =
                    m_run[u] == -INFINITY ? 0.f : fast_exp2((m_run[u] - m_safe) * scale_log2e);
                mc[u] = m_safe * scale_log2e;
                m_run[u] = m_new;
                l_run[u] *= alpha;
                if (__any(alpha != 1.f)) {
#pragma unroll
                    for (int blk = 0; blk < NB; ++blk) o[u][blk] *= alpha;
                }
            }
        }
    };

    // exponentials of block b (scores in s) and O^T += V^T P^T for both sub-tiles
    auto softmax_pv = [&](const f32x16 (&s)[SUB], const unsigned char *sb, int kb0,
                          auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        u32x4 praw[SUB][2];
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            float psum = 0.f;
#pragma unroll
            for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int v = 8 * pg + 2 * jj;
                    float p0 = fast_exp2(__builtin_fmaf(s[u][v], scale_log2e, -mc[u]));
                    float p1 = fast_exp2(__builtin_fmaf(s[u][v + 1], scale_log2e, -mc[u]));
                    if constexpr (MASKED) {
                        p0 = key_of(kb0, v) < vis_end[u] ? p0 : 0.f;
                        p1 = key_of(kb0, v + 1) < vis_end[u] ? p1 : 0.f;
                    }
                    praw[u][pg][jj] = T::pack2(p0, p1);
                    psum = T::add_pair(praw[u][pg][jj], psum);  // sums what the matrix core sees
                }
            l_run[u] += psum;
        }
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                u32x4 vf = *reinterpret_cast<const u32x4 *>(sb + v_lds + pg * TILE_BYTES + blk * 512);
                if constexpr (MASKED) {  // slots past the end may hold anything: zero those values
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int kk = kb0 + 16 * pg + 8 * h + 2 * jj;
                        uint32_t word = vf[jj];
                        if (kk >= it.kv_end) word &= 0xFFFF0000u;
                        if (kk + 1 >= it.kv_end) word &= 0x0000FFFFu;
                        vf[jj] = word;
                    }
                }
#pragma unroll
                for (int u = 0; u < SUB; ++u)
                    o[u][blk] = T::mfma32(as_vec8<T>(vf), as_vec8<T>(praw[u][pg]), o[u][blk]);
            }
    };

    // end of iteration b: the copies of block b+3 (issued three iterations ago) must have landed
    // before the barrier publishes them; younger copies may stay in flight.  This wavefront's LDS
    // reads of block b have been consumed by then, so after the barrier stage b % STAGES may be
    // refilled (it is, two iterations later).
    auto publish = [&](int b) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        if (b + PF < nblocks)
            __builtin_amdgcn_s_waitcnt(waitcnt_imm((PF - 3) * LOADS, 15));
        else
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // ---- prologue: copies of blocks 0..PF-1 on their way, blocks 0..2 landed and published ----
    int id0, id1;
    for (int b = 0; b < PF && b < nblocks; ++b) {
        page_ids(b, id0, id1);
        dma_block(b, id0, id1);
    }
    page_ids(PF, id0, id1);
    asm volatile("" ::: "memory");
    if (nblocks > PF)
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((PF - 3) * LOADS, 15));
    else
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    f32x16 s[SUB], sn[SUB];
    read_k(0);
    scores(s);
    update_reference(s, it.kv_begin, std::true_type{});
    read_k(1);  // a stage without a block holds stale data: those scores are never used

    // blocks 0 .. nfast are unmasked for every row of this wavefront
    int nfast = (unmasked_end - it.kv_begin) / BK - 1;
    if (nfast > nblocks - 1) nfast = nblocks - 1;
    if (nfast < 0) nfast = 0;

    int b = 0;
    // ---- pipelined loop over unmasked blocks that have an unmasked successor ----
    for (; b < nfast; ++b) {
        if (b + PF < nblocks) dma_block(b + PF, id0, id1);
        page_ids(b + PF + 1, id0, id1);
        const int kb0 = it.kv_begin + BK * b;
        scores(sn);                                                  // block b+1
        softmax_pv(s, smem[b % STAGES], kb0, std::false_type{});     // block b
        read_k(b + 2);
        update_reference(sn, kb0 + BK, std::false_type{});
#pragma unroll
        for (int u = 0; u < SUB; ++u) s[u] = sn[u];
        publish(b);
    }
    // ---- masked loop: blocks at the causal boundary / the end of the sequence ----
    for (; b < nblocks; ++b) {
        if (b + PF < nblocks) dma_block(b + PF, id0, id1);
        page_ids(b + PF + 1, id0, id1);
        const int kb0 = it.kv_begin + BK * b;
        if (kb0 < wave_end) softmax_pv(s, smem[b % STAGES], kb0, std::true_type{});
        if (b + 1 < nblocks && kb0 + BK < wave_end) {
            scores(s);
            update_reference(s, kb0 + BK, std::true_type{});
        }
        read_k(b + 2);
        publish(b);
    }

    // ---- finish: every lane owns one row per sub-tile; the two half-waves hold partial sums ----
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
        const float l_tot = l_run[u] + __shfl_xor(l_run[u], 32);
        if (it.split_count == 1) {
            const float inv = 1.f / l_tot;
            uint16_t *dst = out + ((int64_t)(it.q_row0 + tok[u]) * num_q_heads + hq[u]) * D;
#pragma unroll
            for (int blk = 0; blk < NB; ++blk)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int d = 32 * blk + 8 * a + 4 * h;
                    *reinterpret_cast<u32x2 *>(dst + d) = u32x2{
                        T::pack2(o[u][blk][4 * a] * inv, o[u][blk][4 * a + 1] * inv),
                        T::pack2(o[u][blk][4 * a + 2] * inv, o[u][blk][4 * a + 3] * inv)};
                }
        } else {
            const int64_t slot = (int64_t)it.partial_base + 32 * (SUB * w + u) + q32;
            float *po = ws_o + slot * D;
#pragma unroll
            for (int blk = 0; blk < NB; ++blk)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int d = 32 * blk + 8 * a + 4 * h;
                    *reinterpret_cast<f32x4 *>(po + d) =
                        f32x4{o[u][blk][4 * a], o[u][blk][4 * a + 1], o[u][blk][4 * a + 2],
                              o[u][blk][4 * a + 3]};
                }
            if (h == 0) {
                // the merge works in the log2 domain of the scaled scores
                ws_ml[2 * slot] = m_run[u] == -INFINITY ? -INFINITY : m_run[u] * scale_log2e;
                ws_ml[2 * slot + 1] = l_tot;
            }
        }
    }
}

template <typename T>
static hipError_t launch_tile256_t(const pv_plan *plan, const void *q, const void *k_pages,
                                   const void *v_pages, const int32_t *page_table, float scale,
                                   void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    const int n = (int)plan->tile256.size();
    const float c = (scale < 0.f ? -scale : scale) * kLog2e;
    const uint32_t q_sign = scale < 0.f ? 0x80008000u : 0u;
    hipLaunchKernelGGL((attn_tile256_kernel<T>), dim3(n), dim3(256), 0, stream, plan->d_tile256,
                       (const uint16_t *)q, (const uint16_t *)k_pages, (const uint16_t *)v_pages,
                       page_table, plan->max_pages_per_req, plan->num_q_heads,
                       plan->pool.num_kv_heads, plan->group, c, q_sign, (uint16_t *)out, ws_o,
                       ws_ml);
    return hipGetLastError();
}

hipError_t launch_attn_tile256(const pv_plan *plan, const void *q, const void *k_pages,
                               const void *v_pages, const int32_t *page_table, float scale,
                               void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    if (plan->tile256.empty()) return hipSuccess;
    if (plan->pool.head_dim != 128) return hipErrorInvalidValue;  // the plan never does this
    return plan->pool.dtype == PV_F16
               ? launch_tile256_t<F16>(plan, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                       ws_ml, stream)
               : launch_tile256_t<BF16>(plan, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                        ws_ml, stream);
}

}  // namespace pv
