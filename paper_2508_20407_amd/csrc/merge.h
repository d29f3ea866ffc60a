// Exact merge of attention partials by their log-sum-exp statistics.
//
// A partial s of a query row is (O_s, m_s, l_s): O_s = sum_j 2^(x_j - m_s) V_j and
// l_s = sum_j 2^(x_j - m_s) over the keys j of that partition, with x_j the logit in base-2
// units.  Softmax attention over the union of the partitions (the single softmax of Section
// 3's formula) is
//     O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s,      M = max_s m_s.
// The history axis split into partitions uses this; so does the JOINT layer, where the window
// causal partial is one more partition.  The SUM layer normalises the history partitions and
// the window partial separately and adds the two outputs.
#pragma once
#include "common.h"

namespace tlin {

template <int D>
__global__ __launch_bounds__(256) void merge_kernel(const MergeArgs a)
{
    constexpr int TPR = D / 4;                 // threads per row, 4 columns each
    constexpr int RPB = 256 / TPR;             // rows per block
    const int tid = threadIdx.x;
    const int64_t grow = (int64_t)blockIdx.x * RPB + tid / TPR;   // flat row index over (b,h,row)
    if (grow >= a.total_rows) return;
    const int c4 = (tid % TPR) * 4;
    // Sliding schedule: the row belongs to chunk orow / W of its head, the partials of a chunk sit
    // in its own group of slots, and chunk 0 has no history partials.
    const int rows_per_head = a.nchunks ? a.seq_rows : a.W;
    const int bh = (int)(grow / rows_per_head), orow = (int)(grow % rows_per_head);
    const int chunk = a.nchunks ? orow / a.W : 0;
    const int row = orow - chunk * a.W;
    const int b = bh / a.H, hd = bh % a.H;
    const int64_t slot0 = ((int64_t)bh * (a.nchunks ? a.nchunks : 1) + chunk) * a.nparts;
    const int nhist = (a.nchunks && chunk == 0) ? 0 : a.nhist;
    const int64_t wslot = slot0 + a.nhist;             // the window partial's slot

    const int njoint = nhist + ((a.has_window && a.joint) ? 1 : 0);
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float lse2 = -INFINITY;
    if (njoint > 0) {
        float M = -INFINITY;
        // joint slots: the history partials, then (JOINT) the window partial
        auto slot_of = [&](int s) { return s < nhist ? slot0 + s : wslot; };
        // the loops are unrolled so that the loads of several partials are in flight together:
        // with many partitions this kernel is bound by load latency, not by bytes
#pragma unroll 8
        for (int s = 0; s < njoint; ++s) M = fmaxf(M, a.Mpart[slot_of(s) * a.W + row]);
        float den = 0.f;
        f32x4 num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int s = 0; s < njoint; ++s) {
            const int64_t idx = slot_of(s) * a.W + row;
            const float w = exp2f(a.Mpart[idx] - M);
            den += w * a.Lpart[idx];
            num += w * *(const f32x4 *)(a.Opart + idx * D + c4);
        }
        o = num * (1.0f / den);
        lse2 = M + log2f(den);
    }
    if (a.has_window && !a.joint) {
        const int64_t idx = wslot * a.W + row;
        o += *(const f32x4 *)(a.Opart + idx * D + c4) * (1.0f / a.Lpart[idx]);
    }

    const int64_t off = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh + (int64_t)orow * a.o_sr + c4;
    if (c4 >= a.D) {
        // column beyond the tensors' head dimension: nothing to store
    } else if (a.out_bf16) {
        bf16x4 ob;
#pragma unroll
        for (int e = 0; e < 4; ++e) ob[e] = (__bf16)o[e];
        *(bf16x4 *)((__bf16 *)a.O + off) = ob;
    } else {
        *(f32x4 *)((float *)a.O + off) = o;
    }
    if (a.lse && c4 == 0) a.lse[grow] = lse2 * 0.6931471805599453f;
}

}  // namespace tlin
