// Cache-hit step: a few newest query rows against a long history (Section 4.2 of the paper: with
// the history's keys and values cached, only the last token computes, and its attention over the N
// cached rows is the one term that still grows with N).
//
// With one to four query rows the work is a matrix-vector product per head: every byte of K and V
// is used once per query, nothing is reused, and the matrix cores have nothing to offer.  This
// kernel therefore never touches LDS or the matrix cores on its main path: K and V rows stream
// from HBM straight into registers (16 bytes per lane, a wave instruction covers four 256-byte
// rows), scores are v_dot2_f32_bf16 sums reduced over the 16 lanes of a row with DPP rotations, the
// softmax is kept online per lane group, and the value rows are accumulated with v_dot2_f32_bf16
// against the bf16-rounded weight (the same rounding the matrix-core kernels apply).  Many waves
// per SIMD, each with a whole chunk of loads in flight, keep enough bytes on the way to cover HBM
// latency.
//
// A workgroup of four waves takes one partition of one (batch, head): wave w works on the 16-row
// chunks w, w + 4, ... of the partition, the four row groups of a wave keep separate softmax states,
// and the 16 states are joined through LDS at the end into one partial (O_part, m, l) in the format
// of the matrix-core kernels, which the merge kernel then joins exactly.
#pragma once
#include "common.h"

namespace tlin {

typedef __attribute__((ext_vector_type(2))) __bf16 dec_bf16x2;

// sum over the 16 lanes of a row group, result in every lane (rotations inside a row of 16 lanes)
__device__ __forceinline__ float row16_allsum(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x128, 0xf, 0xf, false));   // row_ror:8
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x124, 0xf, 0xf, false));   // row_ror:4
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x122, 0xf, 0xf, false));   // row_ror:2
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x121, 0xf, 0xf, false));   // row_ror:1
    return x;
}

__device__ __forceinline__ float dot2_bf16(unsigned a, unsigned b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, a), __builtin_bit_cast(dec_bf16x2, b), c, false);
}

// Measurement aid: a read stream with nothing else in it (every lane reads 16-byte pieces, folds them
// and keeps the result), to show what this chip delivers to a kernel that only reads; the cache-hit
// kernel is judged against it.  Reads the first 16 * pieces_per_block * gridDim.x bytes of buf.
struct StreamReadArgs {
    const void *buf;
    size_t pieces_per_block;
};
template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const StreamReadArgs a)
{
    const u32x4 *q = (const u32x4 *)a.buf + (size_t)blockIdx.x * a.pieces_per_block;
    unsigned acc = 0;
    constexpr int UNR = 16;
    size_t i = threadIdx.x;
    for (; i + (UNR - 1) * 256 < a.pieces_per_block; i += 256 * UNR) {
        u32x4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) v[u] = NT ? __builtin_nontemporal_load(q + i + u * 256) : q[i + u * 256];
#pragma unroll
        for (int u = 0; u < UNR; ++u) acc += v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; i < a.pieces_per_block; i += 256) {
        const u32x4 v = q[i];
        acc += v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    asm volatile("" ::"v"(acc));       // the folded value is "used": the loads stay
}

// WQ: query rows computed (a.W <= WQ; rows past a.W repeat row 0 and are not stored).  Head
// dimension 128.  Uses a.nsplit partitions of a.tiles_per_split * 64 key rows each.
template <int WQ>
__global__ __launch_bounds__(256) void decode_bf16_kernel(const AttnArgs a)
{
    constexpr int D = 128, CH = 16;       // rows per chunk: four wave-wide loads of four rows each
    __shared__ float Osub[16][WQ][D];
    __shared__ float msub[16][WQ], lsub[16][WQ];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;      // row inside a four-row load, 16-byte piece of the row
    const int split = blockIdx.x % a.nsplit, bh = blockIdx.x / a.nsplit;
    const int b = bh / a.H, hd = bh % a.H;
    const int NK = a.NK;
    const int row_lo = split * a.tiles_per_split * 64;
    const int row_hi = min(NK, row_lo + a.tiles_per_split * 64);
    const int nch = (row_hi - row_lo + CH - 1) / CH;        // chunks of the partition (>= 1)
    const int mine = (nch - wave + 3) / 4;                   // chunks of this wave: wave, wave + 4, ...

    const int64_t k_rb = a.k_sr * 2, v_rb = a.v_sr * 2;
    const char *Kg = (const char *)((const __bf16 *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh);
    const char *Vg = (const char *)((const __bf16 *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh);
    const __bf16 *Qg = (const __bf16 *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh;

    u32x4 q[WQ];      // this lane's eight columns of every query row, as four bf16 pairs
#pragma unroll
    for (int w = 0; w < WQ; ++w) q[w] = *(const u32x4 *)(Qg + (int64_t)(w < a.W ? w : 0) * a.q_sr + 8 * c);

    float m[WQ], l[WQ], O[WQ][8];
#pragma unroll
    for (int w = 0; w < WQ; ++w) {
        m[w] = -INFINITY;
        l[w] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) O[w][e] = 0.f;
    }

    // rows of chunk i of this wave: row_lo + (wave + 4 i) * 16 + 4 ii + g; rows past the partition's end
    // are fetched from its last row (valid memory) and masked
    auto load = [&](int i, u32x4 (&Kr)[4], u32x4 (&Vr)[4]) __attribute__((always_inline)) {
        const int r0 = row_lo + (wave + 4 * i) * CH + g;
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            const int r = min(r0 + 4 * ii, row_hi - 1);
            // non-temporal: every byte is used once (measured: 6.1 -> 6.9 TB/s)
            Kr[ii] = __builtin_nontemporal_load((const u32x4 *)(Kg + (int64_t)r * k_rb + 16 * c));
            Vr[ii] = __builtin_nontemporal_load((const u32x4 *)(Vg + (int64_t)r * v_rb + 16 * c));
        }
    };
    auto compute = [&](int i, const u32x4 (&Kr)[4], const u32x4 (&Vr)[4]) __attribute__((always_inline)) {
        const int r0 = row_lo + (wave + 4 * i) * CH + g;
        float s[4][WQ];
#pragma unroll
        for (int ii = 0; ii < 4; ++ii)
#pragma unroll
            for (int w = 0; w < WQ; ++w) {
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) acc = dot2_bf16(Kr[ii][e], q[w][e], acc);
                s[ii][w] = row16_allsum(acc);
            }
        if (r0 - g + CH > row_hi) {          // ragged last chunk of the partition (uniform over the wave)
#pragma unroll
            for (int ii = 0; ii < 4; ++ii)
                if (r0 + 4 * ii >= row_hi) {
#pragma unroll
                    for (int w = 0; w < WQ; ++w) s[ii][w] = -INFINITY;
                }
        }
#pragma unroll
        for (int w = 0; w < WQ; ++w) {
            const float mx = fmaxf(fmaxf(s[0][w], s[1][w]), fmaxf(s[2][w], s[3][w])) * a.c;
            // the reference point moves only when a score exceeds it by more than 2^8 (weights stay
            // <= 256, any reference point gives the same normalised result)
            if (__builtin_amdgcn_ballot_w64(mx > m[w] + 8.0f) != 0) {
                const float mn = fmaxf(m[w], mx);
                const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2(m[w] - mn);
                l[w] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) O[w][e] *= alpha;
                m[w] = mn;
            }
            const float mref = (m[w] == -INFINITY) ? 0.f : m[w];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const float p = fast_exp2(fmaf(s[ii][w], a.c, -mref));
                // weight rounded to bf16: (p, 0) multiplies the even columns, (0, p) the odd ones; the
                // latter's bit pattern is the rounded weight as fp32, which is what the row sum takes
                const unsigned pe = (unsigned)f32_to_bf16_bits(p);
                const unsigned po = pe << 16;
                l[w] += __builtin_bit_cast(float, po);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    O[w][2 * e] = dot2_bf16(Vr[ii][e], pe, O[w][2 * e]);
                    O[w][2 * e + 1] = dot2_bf16(Vr[ii][e], po, O[w][2 * e + 1]);
                }
            }
        }
    };

    if (mine > 0) {
        // two chunks of loads in flight: the next one is requested before the current one is used
        u32x4 K0[4], V0[4], K1[4], V1[4];
        load(0, K0, V0);
        int i = 0;
        for (; i + 2 <= mine; i += 2) {
            load(i + 1, K1, V1);
            compute(i, K0, V0);
            load(min(i + 2, mine - 1), K0, V0);
            compute(i + 1, K1, V1);
        }
        if (i < mine) compute(i, K0, V0);
    }

    // ---- join the 16 states (4 waves x 4 row groups) of the workgroup
    const int sp = wave * 4 + g;
#pragma unroll
    for (int w = 0; w < WQ; ++w) {
#pragma unroll
        for (int e = 0; e < 8; ++e) Osub[sp][w][8 * c + e] = O[w][e];
        if (c == 0) {
            msub[sp][w] = m[w];
            lsub[sp][w] = l[w];
        }
    }
    __syncthreads();
    const int64_t slot = (int64_t)bh * a.nparts + a.part0 + split;
    for (int idx = tid; idx < WQ * D; idx += 256) {
        const int w = idx / D, d = idx % D;
        if (w >= a.W) break;
        float M = -INFINITY;
#pragma unroll
        for (int k = 0; k < 16; ++k) M = fmaxf(M, msub[k][w]);
        float o = 0.f, L = 0.f;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const float wgt = msub[k][w] == -INFINITY ? 0.f : fast_exp2(msub[k][w] - M);
            o += wgt * Osub[k][w][d];
            L += wgt * lsub[k][w];
        }
        a.Opart[(slot * a.W + w) * D + d] = o;
        if (d == 0) {
            a.Mpart[slot * a.W + w] = M;
            a.Lpart[slot * a.W + w] = L;
        }
    }
}

}  // namespace tlin
