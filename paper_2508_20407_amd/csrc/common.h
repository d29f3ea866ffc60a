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
    int32_t D;                  // head dimension of the tensors; the kernel's D when equal, else smaller
    int32_t W;                  // query rows
    int32_t NK;                 // key rows
    int32_t nqb;                // query blocks per head
    int32_t q_groups;           // resident variant: workgroups per head; each takes blocks g, g+q_groups, ...
    // Sliding schedule (nchunks > 0): Q, K, V hold seq_rows rows per head; chunk c (W rows, the
    // last one shorter) queries rows [0, c*W) of K/V (history launch) or its own rows causally
    // (window launch).  The block index then also enumerates chunks, longest history first, and
    // partial slots are numbered (bh * nchunks + c) * nparts + part.
    int32_t nchunks;
    int32_t seq_rows;
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
    int32_t stream_once;        // host's choice: K/V rows are read by one workgroup only and exceed the caches
    // Layer call, history launch arguments: the workgroup of partition 0 of every (head, query block)
    // also computes the window's causal block of the same rows, and the partitions are cut so that it
    // gets fewer key tiles by that block's cost (see partition_tiles).
    int32_t fuse_window;
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
    int32_t D;                  // columns of O to store (the kernel's D, or fewer)
    int32_t total_rows;         // BH * W (sliding schedule: BH * seq_rows)
    int32_t nchunks;            // sliding schedule: chunks of W rows per head (0 otherwise); chunk 0 has no history
    int32_t seq_rows;           // sliding schedule: output rows per head
};

// Two problem sets in one launch: the history partition blocks first (the long ones), then the
// window causal blocks.  Kernel boundaries are expensive on this chip (the eight L2 caches are
// written back and invalidated at each), and the short window blocks fill the tail of the long ones.
struct PairArgs {
    AttnArgs hist, win;
    int32_t n_hist_blocks, n_win_blocks;
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

// What one workgroup works on, after the sliding-schedule indirection has been resolved.
struct Problem {
    int bh, qb, split;
    int W;            // query rows of this problem (chunk length, or the whole window)
    int NK;           // key rows
    int64_t qrow_off; // first query row inside the head's Q (and output) rows
    int64_t krow_off; // first key row inside the head's K/V rows
    int64_t slot;     // first partial slot of this (head, chunk)
    int tps;          // key tiles per partition
    bool skip;        // nothing to do (rows past a short last chunk, or an empty history)
};

// Cost of the window's causal block of query block qb, in key tiles of the history body: its tiles
// up to the diagonal, each taking QUARTERS / 4 of a history tile's time (bf16: the unpipelined
// causal body takes about 5/4 of a pipelined tile; fp32: the same body, 4/4), plus loading Q and
// writing the partial once more.  Host and device must agree on it.
__host__ __device__ constexpr int window_block_cost(int W, int qb, int BM, int BN, int QUARTERS)
{
    const int rows = (qb + 1) * BM < W ? (qb + 1) * BM : W;
    const int wt = (rows + BN - 1) / BN;
    return wt * QUARTERS / 4 + 2;
}

// Decode the logical block index.  BM: query rows per workgroup, BN: keys per tile.
template <int BM, int BN, bool CAUSAL>
__device__ __forceinline__ Problem decode_problem(const AttnArgs &a, int L, int qstep)
{
    Problem p;
    // causal blocks grow with the block index: the long ones are started first
    p.qb = CAUSAL ? qstep - 1 - L % qstep : L % qstep;
    int rest = L / qstep;
    p.split = rest % a.nsplit;
    rest /= a.nsplit;
    if (a.nchunks == 0) {
        p.bh = rest;
        p.W = a.W;
        p.NK = a.NK;
        p.qrow_off = 0;
        p.krow_off = 0;
        p.slot = (int64_t)p.bh * a.nparts;
        p.tps = a.tiles_per_split;
        p.skip = false;
        return p;
    }
    const int c = a.nchunks - 1 - rest % a.nchunks;   // longest histories first
    p.bh = rest / a.nchunks;
    const int row0 = c * a.W;
    p.W = min(a.W, a.seq_rows - row0);
    p.qrow_off = row0;
    p.slot = ((int64_t)p.bh * a.nchunks + c) * a.nparts;
    if (CAUSAL) {
        p.NK = p.W;
        p.krow_off = row0;
        p.tps = a.tiles_per_split;
    } else {
        p.NK = row0;
        p.krow_off = 0;
        const int tiles = (row0 + BN - 1) / BN;
        p.tps = (tiles + a.nsplit - 1) / a.nsplit;
    }
    p.skip = p.qb * BM >= p.W || p.NK == 0;
    return p;
}

// Key tiles [t0, t1) of an unmasked partition.  Plain: partition s takes tiles s * tps ... of the
// ceil(NK / BN).  With a.fuse_window the same tiles are cut so that partition 0, whose workgroup
// goes on to the window block, is shorter by that block's cost and no workgroup ends later than the rest.
template <int BM, int BN, int QUARTERS>
__device__ __forceinline__ void partition_tiles(const AttnArgs &a, const Problem &pr, int &t0, int &t1)
{
    const int ntiles = (pr.NK + BN - 1) / BN;
    if (!a.fuse_window) {
        t0 = pr.split * pr.tps;
        t1 = min(t0 + pr.tps, ntiles);
        return;
    }
    // the cost of the head's last (longest) window block for every query block: the workgroups of one
    // head then cut their partitions at the same tiles and keep sharing them through the XCD's L2
    const int cost = window_block_cost(a.W, a.nqb - 1, BM, BN, QUARTERS);
    const int tps = (ntiles + cost + a.nsplit - 1) / a.nsplit;
    t0 = max(pr.split * tps - cost, 0);
    t1 = min((pr.split + 1) * tps - cost, ntiles);
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

// One wave-wide direct load HBM -> LDS: 64 lanes x 16 bytes land on the 1 KB of LDS starting at
// the wave-uniform byte offset lds_base (lane i at lds_base + 16*i).  The source is addressed
// through a buffer descriptor: the tile's base address sits in scalar registers and a lane
// contributes a 32-bit byte offset (the address unit handles those faster than 64-bit per-lane
// addresses); offsets at or beyond the descriptor's size read as zeros (raw buffer, stride 0).
// Issued through inline assembly on purpose: the compiler then does not know that LDS is
// being written asynchronously and does not put a wait-for-all-loads in front of every LDS
// read; completion is tracked explicitly with wait_vmcnt() before the tile's barrier.
__device__ __forceinline__ u32x4 tile_descriptor(const char *base, unsigned bytes)
{
    const uint64_t b = (uint64_t)base;
    u32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((unsigned)b);
    d[1] = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32) & 0xffffu);   // stride 0, no swizzle
    d[2] = __builtin_amdgcn_readfirstlane(bytes);
    d[3] = 0x00020000u;                                                       // raw 32-bit data format
    return d;
}
// NT: the load carries the non-temporal hint.  For K/V rows that no other workgroup will read again
// (a single query block per head, a history far larger than the last-level cache) the hint keeps the
// stream from displacing everything else in L2 and raises the sustained HBM rate (measured on a
// 64-row window over 262144 history rows: 5.8 -> 6.9 TB/s); for small, latency-bound problems and
// for tiles that a second query block re-reads from L2 it costs a few per cent, so it is a choice
// of the host per call.
// A lane offset beyond the size of every tile descriptor: the lane's 16 bytes of LDS are cleared and
// no memory request is made.  For the chunks that rows shorter than the kernel's head dimension do
// not have (descriptors of such tensors always carry the tile's real size).
constexpr unsigned kNoChunk = 0xfffffff0u;

template <bool NT = false>
__device__ __forceinline__ void direct_load_1k(u32x4 desc, unsigned byte_off, unsigned lds_base)
{
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds"
                     :
                     : "s"(lds_base), "v"(byte_off), "s"(desc)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :
                     : "s"(lds_base), "v"(byte_off), "s"(desc)
                     : "memory", "m0");
}

__device__ __forceinline__ unsigned lds_offset(const char *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The K/V tile ring of the attention kernels (dynamic LDS, sized by the launch).
extern __shared__ __attribute__((aligned(1024))) char tlin_smem[];

__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f)
{
    return __builtin_bit_cast(unsigned short, (__bf16)f);
}

}  // namespace tlin
