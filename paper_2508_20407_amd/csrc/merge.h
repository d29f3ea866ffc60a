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

// SL threads ("slot lanes") share one (row, 4 columns) item: lane sl takes the partials
// sl, sl + SL, ... and the SL running results are joined through LDS.  With many partitions the
// kernel is bound by the latency of its dependent loads, not by bytes, so the partials of a row are
// spread over threads instead of being walked by one.
template <int D, int SL>
__global__ __launch_bounds__(256) void merge_kernel(const MergeArgs a)
{
    constexpr int TPR = D / 4;                 // column groups per row, 4 columns each
    constexpr int RPB = 256 / (TPR * SL);      // rows per block
    static_assert(RPB >= 1, "a row must fit in a block");
    __shared__ float red[SL > 1 ? 256 * 6 : 1];

    const int tid = threadIdx.x;
    const int cg = tid % TPR, sl = (tid / TPR) % SL, rb = tid / (TPR * SL);
    const int64_t grow = (int64_t)blockIdx.x * RPB + rb;          // flat row index over (b,h,row)
    const bool live = grow < a.total_rows;
    const int c4 = cg * 4;
    // Sliding schedule: the row belongs to chunk orow / W of its head, the partials of a chunk sit
    // in its own group of slots, and chunk 0 has no history partials.
    const int rows_per_head = a.nchunks ? a.seq_rows : a.W;
    const int bh = live ? (int)(grow / rows_per_head) : 0, orow = live ? (int)(grow % rows_per_head) : 0;
    const int chunk = a.nchunks ? orow / a.W : 0;
    const int row = orow - chunk * a.W;
    const int b = bh / a.H, hd = bh % a.H;
    const int64_t slot0 = ((int64_t)bh * (a.nchunks ? a.nchunks : 1) + chunk) * a.nparts;
    const int nhist = (a.nchunks && chunk == 0) ? 0 : a.nhist;
    const int64_t wslot = slot0 + a.nhist;             // the window partial's slot
    const int njoint = live ? nhist + ((a.has_window && a.joint) ? 1 : 0) : 0;
    // joint slots: the history partials, then (JOINT) the window partial
    auto slot_of = [&](int s) { return s < nhist ? slot0 + s : wslot; };

    // this lane's share of the joint partials, relative to its own maximum
    float M = -INFINITY, den = 0.f;
    f32x4 num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int s = sl; s < njoint; s += SL) M = fmaxf(M, a.Mpart[slot_of(s) * a.W + row]);
#pragma unroll 4
    for (int s = sl; s < njoint; s += SL) {
        const int64_t idx = slot_of(s) * a.W + row;
        const float ms = a.Mpart[idx];
        const float w = ms == -INFINITY ? 0.f : exp2f(ms - M);     // an empty partition holds -inf and zeros
        den += w * a.Lpart[idx];
        num += w * *(const f32x4 *)(a.Opart + idx * D + c4);
    }
    if (SL > 1) {
        float *mine = red + tid * 6;
        mine[0] = M; mine[1] = den; mine[2] = num[0]; mine[3] = num[1]; mine[4] = num[2]; mine[5] = num[3];
        __syncthreads();
        if (sl != 0) return;
        float Mt = M;
#pragma unroll
        for (int k = 1; k < SL; ++k) Mt = fmaxf(Mt, red[(tid + k * TPR) * 6]);
        const float w0 = M == -INFINITY ? 0.f : exp2f(M - Mt);     // a lane without partials holds -inf
        den *= w0;
        num *= w0;
#pragma unroll
        for (int k = 1; k < SL; ++k) {
            const float *o = red + (tid + k * TPR) * 6;
            const float w = o[0] == -INFINITY ? 0.f : exp2f(o[0] - Mt);
            den += w * o[1];
            num += w * f32x4{o[2], o[3], o[4], o[5]};
        }
        M = Mt;
    }
    if (!live) return;

    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float lse2 = -INFINITY;
    if (njoint > 0) {
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
