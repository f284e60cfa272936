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
//  * With one wavefront per SIMD nothing else hides a stall, and every instruction of any kind
//    costs that wavefront four to five issue cycles (measured), of which about 27 are free next
//    to a 32-cycle matrix-core instruction.  So the steady-state iteration is a hand-laid
//    schedule of 32 slots, one matrix-core instruction each, software-pipelined: slot by slot it
//    issues the score product of block b+1, the exponentials of block b and the value product of
//    block b (see fast_step).  The instruction count per slot is what is tuned:
//      - for the usual small scales the queries are pre-multiplied by scale*log2(e) once (rounded
//        to the 16-bit type; see PRE below) and the score product starts from minus the row's
//        reference maximum instead of zero, so a probability is one exp2 of a matrix-core result;
//      - row sums are plain additions of the exponentials, spread over the slots of the value
//        product (a v_dot2 on the packed probabilities would halve their number, but a dot
//        instruction waits for the matrix pipe to drain);
//      - addresses of the asynchronous copies are two scalar multiplies and four 64-bit adds.
//  * K/V page tiles go HBM/L2 -> LDS directly (global_load_lds) into a ring of 8 stages, six blocks
//    ahead; one s_barrier per block.  K operands of block b+2 are requested before the barrier at
//    the end of iteration b, so they are in registers when iteration b+1 starts.
//
// Blocks that touch the causal boundary or the end of the sequence run in a second, masked loop
// with the same barrier protocol, so the wavefronts of a workgroup stay in step.
//
// PRE (template flag, chosen per launch): the queries are multiplied by scale*log2(e) and rounded
// back to 16 bits when they are loaded.  That rounding moves a score by at most 2^-9 (bf16) or
// 2^-12 (fp16) of sum_d |q_d k_d| * scale*log2(e), the size of the rounding the probabilities get
// anyway before the second product; the launch uses it only while |scale*log2(e)| <= 0.25 (1/sqrt(D)
// for D >= 34), and the exact fp32 scaling otherwise.
#include <type_traits>

#include "pv_device.h"

namespace pv {

template <typename T, bool PRE>
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
    static_assert(LOADS == 4, "piece layout below assumes four pieces per wavefront");
    __shared__ __attribute__((aligned(16))) unsigned char smem[STAGES][STAGE_BYTES];
    // the item's page ids, two per block: read back through LDS, whose results return in order
    // with the operand reads (a scalar load in the loop would make every wait for an operand a
    // wait for that load too)
    __shared__ __attribute__((aligned(8))) int32_t page_lds[kTileMaxPages];

    const WorkItem it = items[blockIdx.x];
    const int lane = lane_id();
    const int w = wave_id();
    const int q32 = lane & 31;
    const int h = lane >> 5;
    // what multiplies a matrix-core score to get the exponent: with PRE the scores come out scaled
    const float cfac = PRE ? 1.f : scale_log2e;

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

    u32x4 qf[SUB][KS];  // live in accumulation registers: only the matrix cores read them
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
        const uint16_t *qrow = q + ((int64_t)(it.q_row0 + tok[u]) * num_q_heads + hq[u]) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 raw = load16(qrow + 16 * ks + 8 * h);
            if constexpr (PRE) {
                // q * scale*log2(e), rounded to the 16-bit type (the sign of the scale included)
                const typename T::vec8 v = as_vec8<T>(raw);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    raw[e] = T::pack2((float)v[2 * e] * scale_log2e,
                                      (float)v[2 * e + 1] * scale_log2e);
            } else {
                raw ^= q_sign;  // a negative scale is applied as |scale| on negated queries
            }
            qf[u][ks] = raw;
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
    const uint32_t lane_bytes = (uint32_t)lane * 16u;

    // page ids of a block (two pages; a page past the end is never used, so any valid id will do)
    for (int i = (int)threadIdx.x; i < 2 * nblocks && i < kTileMaxPages; i += 256)
        page_lds[i] = pt[pg0 + i <= last_pg ? pg0 + i : last_pg];
    __syncthreads();
    // in two steps, so that the pipelined loop can put other work between the LDS read and the
    // first use of its result
    auto page_ids_request = [&](int b) {
        const int bb = b < nblocks ? b : nblocks - 1;  // ids past the last block are never used
        return *reinterpret_cast<const u32x2 *>(&page_lds[2 * bb]);
    };
    auto page_ids_take = [&](u32x2 ids, int &id0, int &id1) {
        id0 = __builtin_amdgcn_readfirstlane((int)ids[0]);
        id1 = __builtin_amdgcn_readfirstlane((int)ids[1]);
    };
    auto page_ids = [&](int b, int &id0, int &id1) { page_ids_take(page_ids_request(b), id0, id1); };
    // Asynchronous copy of block b into stage b % STAGES.  The stage is 16 pieces of 1 KiB: K page
    // 0, K page 1, V page 0, V page 1, four pieces each; wavefront w moves piece w of each, i.e. the
    // bytes [w KiB, w KiB + 1 KiB) of the (page, head) tile: source = pool + page id * page bytes
    // + a per-wavefront constant (one 32x32 -> 64 bit multiply per page, one 64-bit add per piece).
    const uint32_t page_bytes = (uint32_t)num_kv_heads * TILE_BYTES;
    const uint64_t wave_off = (uint64_t)it.kv_head * TILE_BYTES + (uint32_t)w * 1024u;
    const unsigned char *k_src = reinterpret_cast<const unsigned char *>(k_pages) + wave_off;
    const unsigned char *v_src = reinterpret_cast<const unsigned char *>(v_pages) + wave_off;
    auto dma_piece = [&](int b, int id0, int id1, int i) {
        unsigned char *dst = smem[b % STAGES] + (w + 4 * i) * 1024;
        const uint64_t page_off = (uint64_t)(uint32_t)((i & 1) ? id1 : id0) * page_bytes;
        lds_dma16(((i & 2) ? v_src : k_src) + page_off, lane_bytes, dst);
    };
    auto dma_block = [&](int b, int id0, int id1) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) dma_piece(b, id0, id1, i);
    };

    f32x16 o[SUB][NB];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[u][blk][v] = 0.f;
    // Softmax state per sub-tile.  Scores are raw matrix-core results; x = score * cfac is the
    // exponent in the exp2 domain.  Lazy reference maximum (exact, softmax is shift-invariant): it
    // only moves when a score of the coming block exceeds it by more than 2^kLazyLog2 in the exp2
    // domain (thr = reference + that margin in score units; -inf while there is no reference), so
    // rescaling the accumulators is rare.
    float m_run[SUB], l_run[SUB], mc[SUB], thr[SUB];
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
        m_run[u] = -INFINITY;  // reference maximum of the scores
        l_run[u] = 0.f;        // this lane's share of the running sum
        mc[u] = 0.f;           // m_run in the exp2 domain (0 while there is no reference yet)
        thr[u] = -INFINITY;
    }
    const float lazy_margin = kLazyLog2 / cfac;  // +inf for a zero scale: set once, kept

    u32x4 kf[KS];  // K operands of the block whose scores are computed next
    auto read_k = [&](int b) {
        const unsigned char *sb = smem[b % STAGES];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            kf[ks] = *reinterpret_cast<const u32x4 *>(sb + k_lds + ks * 512);
    };
    // S^T of the block whose K operands are in kf, both sub-tiles (they share the operands), for
    // the prologue and the masked loop.  Every use of the Q operands in this kernel is a pinned
    // instruction with the operand in an accumulation register (see mfma32_first), so that the
    // register allocator keeps all of Q there for good.  Outside the hand-laid schedule of the pipelined loop the
    // compiler may still move an operand into place right in front of the statement, hence the
    // guarded form here, and the wait for the results before anything reads them.
    auto scores = [&](f32x16 (&sn)[SUB]) {
#pragma unroll
        for (int u = 0; u < SUB; ++u) T::mfma32_first_guarded(sn[u], kf[0], qf[u][0]);
#pragma unroll
        for (int ks = 1; ks < KS; ++ks)
#pragma unroll
            for (int u = 0; u < SUB; ++u) T::mfma32_next_guarded(sn[u], kf[ks], qf[u][ks]);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // register v = 8*page + j of S^T  <->  key kb0 + 16*page + 8*h + j
    auto key_of = [&](int kb0, int v) { return kb0 + 16 * (v >> 3) + 8 * h + (v & 7); };

    // moves the reference of every row whose block maximum mx (score units) exceeds its threshold
    auto raise_reference = [&](const float (&mx)[SUB]) {
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            const float mxx = fmaxf(mx[u], __shfl_xor(mx[u], 32));
            const float m_new = mxx > thr[u] ? mxx : m_run[u];
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha =
                m_run[u] == -INFINITY ? 0.f : fast_exp2((m_run[u] - m_safe) * cfac);
            mc[u] = m_safe * cfac;
            m_run[u] = m_new;
            thr[u] = m_new == -INFINITY ? -INFINITY : m_new + lazy_margin;
            l_run[u] *= alpha;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int blk = 0; blk < NB; ++blk) o[u][blk] *= alpha;
            }
        }
    };
    // works on the scores of the block that the NEXT softmax will consume
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
            grow = grow || mx[u] > thr[u];
        }
        if (__any(grow)) raise_reference(mx);
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
                    float p0 = fast_exp2(__builtin_fmaf(s[u][v], cfac, -mc[u]));
                    float p1 = fast_exp2(__builtin_fmaf(s[u][v + 1], cfac, -mc[u]));
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
    // refilled (it is, two iterations later).  `more` = a copy was issued in this iteration.
    auto publish = [&](bool more) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        if (more)
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
    publish(nblocks > PF);

    f32x16 s[SUB], sn[SUB];
    read_k(0);
    scores(s);
    update_reference(s, it.kv_begin, std::true_type{});
    read_k(1);  // a stage without a block holds stale data: those scores are never used

    // One pipelined iteration: block b's exponents (PRE) or scores are in `cur`; leaves those of
    // block b+1 in `nxt`.  With PRE an "exponent" is score - reference, ready for exp2: the score
    // product starts from cinit = -reference instead of zero.  The instruction order is laid out
    // by hand in 32 slots, one matrix-core instruction each, fenced so that the compiler keeps it:
    //   slots  0-15  score product of block b+1 (k-step slot/2, sub-tile slot%2), and the
    //                exponentials of block b as a pipeline over its 16 score pairs (scale-and-shift
    //                unless PRE, exp2 one slot later, pack to 16 bits one slot after that);
    //   slots 16-31  value product of block b (V operand (slot-16)/2, sub-tile slot%2; every P
    //                operand is complete when its instruction issues), the V operands requested
    //                six slots ahead of their use; in between the copy of block b+PF (its four
    //                pieces spread over slots 16-20 and 29-32), the
    //                page ids of the next copy (requested in slot 21, taken in slot 31), from slot 20 on the maximum of block b+1's results
    //                (its last score instruction issued in slot 15, see mfma32_first); K operands
    //                are requested six slots ahead of their use as well, those of the next
    //                iteration's first three k-steps in slots 26-30;
    //                the 32 additions of the row sums fill what room the slots 16-31 have left;
    //   then the test for a reference update, and the barrier.
    f32x16 cinit[SUB];
    float thr_rel[SUB];  // PRE: threshold for block maxima that are relative to the reference
    auto fast_step = [&](int b, const f32x16 (&cur)[SUB], f32x16 (&nxt)[SUB]) {
        const unsigned char *sb = smem[b % STAGES];
        const unsigned char *sk1 = smem[(b + 1) % STAGES];
        const unsigned char *sk = smem[(b + 2) % STAGES];
        u32x4 vf[2][NB];
        u32x4 praw[SUB][2];
        float xs[SUB * 8][2], es[SUB * 8][2];
        float mx[SUB];
        float psum[SUB] = {0.f, 0.f};
        uint64_t dma_off[2];
        const unsigned char *dma_src[LOADS];
        u32x2 next_ids;
        // how many of the 32 row-sum additions each of the slots 16-31 takes: as many as fit
        // beside what the slot already carries
        constexpr int kSumAdds[16] = {0, 3, 1, 3, 0, 0, 2, 3, 2, 3, 2, 3, 3, 3, 1, 3};
#pragma unroll
        for (int slot = 0; slot < 32; ++slot) {
            // --- the slot's matrix-core instruction
            if (slot < 16) {
                const int ks = slot / 2, u = slot % 2;
                if (ks == 0) {
                    if constexpr (PRE)
                        T::mfma32_from(nxt[u], kf[0], qf[u][0], cinit[u]);
                    else
                        T::mfma32_first(nxt[u], kf[0], qf[u][0]);
                } else {
                    T::mfma32_next(nxt[u], kf[ks], qf[u][ks]);
                }
            } else {
                // V operand i = 4*page + blk feeds both sub-tiles back to back, so it is live
                // for a few slots only
                const int i = (slot - 16) / 2, u = (slot - 16) % 2;
                const int pg = i / 4, blk = i % 4;
                o[u][blk] = T::mfma32(as_vec8<T>(vf[pg][blk]), as_vec8<T>(praw[u][pg]), o[u][blk]);
            }
            // the matrix-core instruction opens its slot: what follows runs beside it (left to
            // itself the compiler puts every other slot's exponentials in front of it, and two
            // slots' worth of them between two matrix-core instructions do not fit beside one)
            __builtin_amdgcn_sched_barrier(0);
            // --- LDS reads: V operand i of this block six slots ahead of its first use (they
            //     take over the registers of K operands already consumed), later the K operands
            //     of block b+2
            if (slot >= 10 && slot < 26 && slot % 2 == 0) {
                const int i = (slot - 10) / 2;
                vf[i / 4][i % 4] = *reinterpret_cast<const u32x4 *>(
                    sb + v_lds + (i / 4) * TILE_BYTES + (i % 4) * 512);
            }
            // K operand ks of block b+1 is used in slots 2*ks, 2*ks+1: operands 3-7 are requested
            // six slots ahead, operands 0-2 of block b+2 at the end (slots 26, 28, 30)
            if (slot <= 8 && slot % 2 == 0)
                kf[3 + slot / 2] =
                    *reinterpret_cast<const u32x4 *>(sk1 + k_lds + (3 + slot / 2) * 512);
            if (slot >= 26 && slot % 2 == 0)
                kf[(slot - 26) / 2] =
                    *reinterpret_cast<const u32x4 *>(sk + k_lds + ((slot - 26) / 2) * 512);
            // --- exponentials: pair j = 8*u + 4*page + jj holds results 2*(j%8), 2*(j%8)+1 of u
            if constexpr (PRE) {
                if (slot < 16) {
                    const int u = slot / 8, v = 2 * (slot % 8);
                    es[slot][0] = fast_exp2(cur[u][v]);
                    es[slot][1] = fast_exp2(cur[u][v + 1]);
                }
                if (slot >= 1 && slot < 17) {
                    const int j = slot - 1;
                    praw[j / 8][(j % 8) / 4][j % 4] = T::pack2(es[j][0], es[j][1]);
                }
            } else {
                if (slot < 16) {
                    const int u = slot / 8, v = 2 * (slot % 8);
                    xs[slot][0] = __builtin_fmaf(cur[u][v], cfac, -mc[u]);
                    xs[slot][1] = __builtin_fmaf(cur[u][v + 1], cfac, -mc[u]);
                }
                if (slot >= 1 && slot < 17) {
                    es[slot - 1][0] = fast_exp2(xs[slot - 1][0]);
                    es[slot - 1][1] = fast_exp2(xs[slot - 1][1]);
                }
                if (slot >= 2 && slot < 18) {
                    const int j = slot - 2;
                    praw[j / 8][(j % 8) / 4][j % 4] = T::pack2(es[j][0], es[j][1]);
                }
            }
            // --- copy of block b+PF (of the last block again once b + PF >= nblocks: page_ids
            // clamps the block number), one piece a slot
            // (the scalar address arithmetic of a piece goes one slot ahead of its copy, into
            // slots that have no operand read, so that no slot carries more than about five
            // instructions next to its matrix-core instruction)
            if (slot == 16) {
                dma_off[0] = (uint64_t)(uint32_t)id0 * page_bytes;
                dma_off[1] = (uint64_t)(uint32_t)id1 * page_bytes;
            }
            if (slot == 17 || slot == 19 || slot == 29 || slot == 31) {
                const int i = slot < 20 ? (slot - 17) / 2 : 2 + (slot - 29) / 2;
                dma_src[i] = ((i & 2) ? v_src : k_src) + dma_off[i & 1];
            }
            if (slot == 18 || slot == 20 || slot == 30) {
                const int i = slot < 21 ? (slot - 18) / 2 : 2;
                lds_dma16(dma_src[i], lane_bytes, smem[(b + PF) % STAGES] + (w + 4 * i) * 1024);
            }
            if (slot == 21) next_ids = page_ids_request(b + PF + 1);
            if (slot == 31) page_ids_take(next_ids, id0, id1);
            // --- maximum of block b+1's results, two registers per slot and sub-tile
            if (slot >= 20 && slot < 28) {
                const int i = slot - 20;
#pragma unroll
                for (int u = 0; u < SUB; ++u)
                    mx[u] = max3_raw(i == 0 ? nxt[u][0] : mx[u], nxt[u][2 * i], nxt[u][2 * i + 1]);
            }
            // --- row sums: plain additions of the exponentials (before their rounding to 16
            // bits), spread over the slots of the value product
            if (slot >= 16) {
                int first = 0;
#pragma unroll
                for (int t = 16; t < slot; ++t) first += kSumAdds[t - 16];
#pragma unroll
                for (int a = 0; a < kSumAdds[slot - 16]; ++a) {
                    const int k = first + a;
                    psum[k / 16] += es[k / 2][k % 2];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_dma16(dma_src[3], lane_bytes, smem[(b + PF) % STAGES] + (w + 4 * 3) * 1024);
#pragma unroll
        for (int u = 0; u < SUB; ++u) l_run[u] += psum[u];
        if constexpr (PRE) {
            if (__any(mx[0] > thr_rel[0] || mx[1] > thr_rel[1])) {
                float mx_abs[SUB], mc_old[SUB];
#pragma unroll
                for (int u = 0; u < SUB; ++u) {
                    mc_old[u] = mc[u];
                    mx_abs[u] = mx[u] + mc[u];  // cfac = 1: scores and exponents share a unit
                }
                raise_reference(mx_abs);
#pragma unroll
                for (int u = 0; u < SUB; ++u) {
                    const float shift = mc_old[u] - mc[u];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        nxt[u][v] += shift;  // block b+1's exponents follow the new reference
                        cinit[u][v] += shift;  // = -mc[u], updated in place (no register move)
                    }
                    thr_rel[u] = thr[u] - mc[u];
                }
                asm volatile("s_nop 1" ::: "memory");  // cinit feeds a pinned instruction soon
            }
        } else {
            if (__any(mx[0] > thr[0] || mx[1] > thr[1])) raise_reference(mx);
        }
        publish(true);
    };

    // blocks 0 .. nfast are unmasked for every row of this wavefront.  Near the end of the item a
    // pipelined iteration has no further block to copy: it fetches the last block once more, into
    // a stage nobody reads again, so that the count of copies in flight stays what the waits assume
    int nfast = (unmasked_end - it.kv_begin) / BK - 1;
    if (nfast < 0) nfast = 0;
    nfast &= ~1;  // pairs: the results ping-pong between two register sets without copies

    int b = 0;
    // ---- pipelined loop over unmasked blocks that have an unmasked successor ----
    if (nfast > 0) {
        if constexpr (PRE) {
            // scores -> exponents for the block in flight, and the starting value of the next ones
#pragma unroll
            for (int u = 0; u < SUB; ++u) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    s[u][v] -= mc[u];
                    cinit[u][v] = -mc[u];
                }
                thr_rel[u] = thr[u] - mc[u];
            }
            asm volatile("s_nop 1" ::: "memory");  // cinit feeds a pinned instruction next
        }
        for (; b < nfast; b += 2) {
            fast_step(b, s, sn);
            fast_step(b + 1, sn, s);
        }
        if constexpr (PRE) {  // back to scores for the masked loop
#pragma unroll
            for (int u = 0; u < SUB; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[u][v] += mc[u];
        }
        read_k(b + 1);  // the pipelined loop had requested the first three operands only
    }
    // ---- masked loop: blocks at the causal boundary / the end of the sequence ----
    for (; b < nblocks; ++b) {
        const bool more = b + PF < nblocks;
        if (more) dma_block(b + PF, id0, id1);
        page_ids(b + PF + 1, id0, id1);
        const int kb0 = it.kv_begin + BK * b;
        if (kb0 < wave_end) softmax_pv(s, smem[b % STAGES], kb0, std::true_type{});
        if (b + 1 < nblocks && kb0 + BK < wave_end) {
            scores(s);
            update_reference(s, kb0 + BK, std::true_type{});
        }
        read_k(b + 2);
        publish(more);
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
                ws_ml[2 * slot] = m_run[u] == -INFINITY ? -INFINITY : m_run[u] * cfac;
                ws_ml[2 * slot + 1] = l_tot;
            }
        }
    }
}

template <typename T>
static hipError_t launch_tile256_t(const pv_plan *plan, const DeviceLists &dl, const void *q, const void *k_pages,
                                   const void *v_pages, const int32_t *page_table, float scale,
                                   void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    const int n = (int)plan->tile256.size();
    const float c_signed = scale * kLog2e;
    const float c_abs = c_signed < 0.f ? -c_signed : c_signed;
    if (c_abs <= 0.25f) {
        // queries pre-multiplied by scale*log2(e): the sign travels with them
        hipLaunchKernelGGL((attn_tile256_kernel<T, true>), dim3(n), dim3(256), 0, stream,
                           dl.tile256, (const uint16_t *)q, (const uint16_t *)k_pages,
                           (const uint16_t *)v_pages, page_table, plan->max_pages_per_req,
                           plan->num_q_heads, plan->pool.num_kv_heads, plan->group, c_signed, 0u,
                           (uint16_t *)out, ws_o, ws_ml);
    } else {
        const uint32_t q_sign = scale < 0.f ? 0x80008000u : 0u;
        hipLaunchKernelGGL((attn_tile256_kernel<T, false>), dim3(n), dim3(256), 0, stream,
                           dl.tile256, (const uint16_t *)q, (const uint16_t *)k_pages,
                           (const uint16_t *)v_pages, page_table, plan->max_pages_per_req,
                           plan->num_q_heads, plan->pool.num_kv_heads, plan->group, c_abs, q_sign,
                           (uint16_t *)out, ws_o, ws_ml);
    }
    return hipGetLastError();
}

hipError_t launch_attn_tile256(const pv_plan *plan, const DeviceLists &dl, const void *q, const void *k_pages,
                               const void *v_pages, const int32_t *page_table, float scale,
                               void *out, float *ws_o, float *ws_ml, hipStream_t stream)
{
    if (plan->tile256.empty()) return hipSuccess;
    if (plan->pool.head_dim != 128) return hipErrorInvalidValue;  // the plan never does this
    for (const WorkItem &w : plan->tile256)  // what the kernel assumes of its items
        if (w.row_count != kTileRows || w.kv_end <= w.kv_begin || w.kv_begin % kKvBlock != 0 ||
            (int64_t)w.kv_end - w.kv_begin > (int64_t)kTileMaxPages * 16)
            return hipErrorInvalidValue;
    return plan->pool.dtype == PV_F16
               ? launch_tile256_t<F16>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                       ws_ml, stream)
               : launch_tile256_t<BF16>(plan, dl, q, k_pages, v_pages, page_table, scale, out, ws_o,
                                        ws_ml, stream);
}

}  // namespace pv
