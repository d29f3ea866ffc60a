// Shared device-side definitions for the libtlinattn kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tlin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int kNumCU = 256;   // MI355X: 8 XCDs x 32 compute units
constexpr int kNumXCD = 8;

// One launch of a partial-attention kernel: a set of (batch*head, query block, key partition)
// work items, each producing either a final output tile or an unnormalised partial
// (O_part, m, l) to be merged later.
struct AttnArgs {
    const void *Q, *K, *V;
    int64_t q_sb, q_sh, q_sr;   // element strides: batch, head, row
    int64_t k_sb, k_sh, k_sr;
    int64_t v_sb, v_sh, v_sr;
    int32_t H;                  // heads per batch (to split the flat batch*head index)
    int32_t W;                  // query rows
    int32_t NK;                 // key rows
    int32_t nqb;                // query blocks per head
    int32_t q_groups;           // resident variant: workgroups per head; each takes blocks g, g+q_groups, ...
    int32_t nsplit;             // key partitions (1 for the causal kernel)
    int32_t tiles_per_split;    // key tiles (of 64 rows) per partition
    int32_t nparts;             // partial slots per (b,h) in the workspace
    int32_t part0;              // first slot this launch writes
    float c;                    // scale * log2(e): logits are handled in base-2 units
    float scale;                // logit multiplier
    // partial outputs: Opart [BH][nparts][W][D] fp32, Mpart/Lpart [BH][nparts][W] fp32
    float *Opart, *Mpart, *Lpart;
    // direct outputs (used when direct != 0: a single partition writes final values)
    void *O;
    int64_t o_sb, o_sh, o_sr;
    float *lse;                 // nullable, dense [BH][W]
    int32_t out_bf16;
    int32_t direct;
};

struct MergeArgs {
    const float *Opart, *Mpart, *Lpart;
    int32_t H, W;
    int32_t nparts;             // slots per (b,h)
    int32_t nhist;              // slots [0, nhist) hold history partitions
    int32_t has_window;         // slot nhist holds the window causal partial
    int32_t joint;              // 1: one softmax over all slots; 0: history + window, added
    void *O;
    int64_t o_sb, o_sh, o_sr;
    float *lse;                 // nullable
    int32_t out_bf16;
    int32_t total_rows;         // BH * W
};

// Workgroups are dispatched round-robin over the 8 XCDs, each with a private L2.  Map the
// hardware block id to a logical id such that consecutive logical ids run on the same XCD at
// about the same time: neighbours that read the same K/V tiles then share that L2.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks)
{
    const int per = nblocks / kNumXCD, rem = nblocks % kNumXCD;
    const int xcd = bid % kNumXCD, slot = bid / kNumXCD;
    return xcd * per + (xcd < rem ? xcd : rem) + slot;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange between the two half-waves: returns {x[lane % 32], x[lane % 32 + 32]} in every lane.
// v_permlane32_swap swaps the upper half of its first operand with the lower half of its
// second.  (The two results are copied to scalars before the bit cast: a bit cast applied
// directly to a vector element reads element 0 for both.)
__device__ __forceinline__ void xhalf_pair(float x, float &lo, float &hi)
{
    const unsigned a = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}
// max / sum over the two lanes l and l^32 (the two half-waves hold the same query column).
__device__ __forceinline__ float xhalf_max(float x)
{
    float lo, hi;
    xhalf_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float xhalf_sum(float x)
{
    float lo, hi;
    xhalf_pair(x, lo, hi);
    return lo + hi;
}

__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f)
{
    return __builtin_bit_cast(unsigned short, (__bf16)f);
}

}  // namespace tlin
