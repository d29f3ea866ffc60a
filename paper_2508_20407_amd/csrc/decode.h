// Cache-hit step: a few newest query rows against a long history (Section 4.2 of the paper: with
// the history's keys and values cached, only the last token computes, and its attention over the N
// cached rows is the one term that still grows with N).
//
// With one to four query rows the work is a matrix-vector product per head: every byte of K and V
// is used once per query, nothing is reused, and the matrix cores have nothing to offer.  This
// kernel therefore never touches LDS or the matrix cores on its main path: K and V rows stream
// from HBM straight into registers (16 bytes per lane and load, 16 lanes to a row, a wave
// instruction covers four rows or half rows), scores are sums over a lane's columns (v_dot2_f32_bf16 for bf16 inputs, fp32 FMAs
// for fp32 inputs) reduced over the lanes of a row with DPP exchanges, the softmax is kept online
// per lane group, and the value rows are accumulated per lane (bf16: v_dot2_f32_bf16 against the
// bf16-rounded weight, the same rounding the matrix-core kernels apply; fp32: FMAs with the fp32
// weight).  Several waves per SIMD, each with two chunks of loads in flight, keep enough bytes on
// the way to cover HBM latency.
//
// A workgroup of four waves takes one partition of one (batch, head): wave w works on the chunks
// w, w + 4, ... of the partition, the row groups of a wave keep separate softmax states, and the
// 16 states are joined through LDS at the end into one partial (O_part, m, l) in the format
// of the matrix-core kernels, which the merge kernel then joins exactly.
#pragma once
#include "common.h"

namespace tlin {

typedef __attribute__((ext_vector_type(2))) __bf16 dec_bf16x2;

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}

// sum over the 16 consecutive lanes that share a row, result in every one of them: neighbours
// inside a quad, the other quad of a group of eight (mirror inside eight lanes: quads are uniform
// by then), the other eight (mirror inside sixteen lanes)
__device__ __forceinline__ float row16_allsum(float x)
{
    x = dpp_add<0xB1>(x);      // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);      // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);     // row_half_mirror
    x = dpp_add<0x140>(x);     // row_mirror
    return x;
}

__device__ __forceinline__ float dot2_bf16(unsigned a, unsigned b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, a), __builtin_bit_cast(dec_bf16x2, b), c, false);
}

// (taken by value on purpose: a bit cast applied directly to an element of a vector reads element 0)
__device__ __forceinline__ float as_f32(unsigned x) { return __builtin_bit_cast(float, x); }

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

// T: element type of Q, K and V (__bf16 or float).  DK: the kernel's head dimension (a row of 256
// or 512 bytes: 128 for bf16, 64 or 128 for fp32; shorter bf16 rows are as fast on the matrix-core
// path, whose cost does not grow with the number of query rows);
// the tensors' a.D equals it, or is smaller when PAD (then a row's pieces past a.D are not read,
// and what the last piece holds past a.D -- the caller's padding, possibly NaNs -- is cleared in K
// and Q and lands in output columns that are not stored for V).  WQ: query rows computed
// (a.W <= WQ; rows past a.W repeat row 0 and are not stored).  Uses a.nsplit partitions of
// a.tiles_per_split * 64 key rows each.
template <typename T, int DK, int WQ, bool PAD>
__global__ __launch_bounds__(256) void decode_kernel(const AttnArgs a)
{
    constexpr bool BF = sizeof(T) == 2;
    constexpr int EB = sizeof(T);               // bytes per element
    constexpr int EPP = 16 / EB;                // elements per 16-byte piece
    constexpr int PIECES = DK * EB / 16;        // pieces per row: 16 or 32
    constexpr int LPR = 16;                     // lanes that share a row
    constexpr int PPL = PIECES / LPR;           // pieces of a row per lane: 1, or 2 (fp32, 128 columns)
    constexpr int RPI = 64 / LPR;               // rows per wave-wide load
    constexpr int NI = 4 / PPL;                 // wave-wide row loads per chunk (a chunk is 4 loads of K, 4 of V)
    constexpr int CH = NI * RPI;                // rows per chunk: 16 or 8
    constexpr int EL = PPL * EPP;               // columns per lane
    constexpr int NG = 4 * RPI;                 // softmax states per workgroup
    static_assert(PIECES == 16 || PIECES == 32, "rows of 256 or 512 bytes");

    constexpr int WB = WQ < 4 ? WQ : 4;         // query rows joined through LDS at a time
    __shared__ float Osub[NG][WB][DK];
    __shared__ float msub[NG][WB], lsub[NG][WB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane / LPR, c = lane % LPR;    // row inside a wave-wide load, first piece of this lane
    const int split = blockIdx.x % a.nsplit, bh = blockIdx.x / a.nsplit;
    const int b = bh / a.H, hd = bh % a.H;
    const int NK = a.NK;
    const int row_lo = split * a.tiles_per_split * 64;
    const int row_hi = min(NK, row_lo + a.tiles_per_split * 64);
    const int nch = (row_hi - row_lo + CH - 1) / CH;        // chunks of the partition (>= 1)
    const int mine = (nch - wave + 3) / 4;                   // chunks of this wave: wave, wave + 4, ...

    const int64_t k_rb = a.k_sr * EB, v_rb = a.v_sr * EB;
    const char *Kg = (const char *)((const T *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh);
    const char *Vg = (const char *)((const T *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh);
    const char *Qg = (const char *)((const T *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh);

    // this lane's pieces: byte offset inside a row, and (PAD) which of a piece's four words lie below a.D
    int pofs[PPL];
    u32x4 keep[PPL];
#pragma unroll
    for (int j = 0; j < PPL; ++j) {
        const int piece = c + LPR * j;
        pofs[j] = 16 * piece;
        keep[j] = u32x4{~0u, ~0u, ~0u, ~0u};
        if (PAD) {
            if (piece * EPP >= a.D) pofs[j] = 0;      // nothing of this piece belongs to the row: read piece 0, keep nothing
#pragma unroll
            for (int e = 0; e < 4; ++e) keep[j][e] = (piece * EPP + e * (EPP / 4) < a.D) ? ~0u : 0u;
        }
    }

    u32x4 q[WQ][PPL];      // this lane's columns of every query row
#pragma unroll
    for (int w = 0; w < WQ; ++w)
#pragma unroll
        for (int j = 0; j < PPL; ++j) {
            q[w][j] = *(const u32x4 *)(Qg + (int64_t)(w < a.W ? w : 0) * a.q_sr * EB + pofs[j]);
            if (PAD) q[w][j] &= keep[j];
        }

    float m[WQ], l[WQ], O[WQ][EL];
#pragma unroll
    for (int w = 0; w < WQ; ++w) {
        m[w] = -INFINITY;
        l[w] = 0.f;
#pragma unroll
        for (int e = 0; e < EL; ++e) O[w][e] = 0.f;
    }

    // rows of chunk i of this wave: row_lo + (wave + 4 i) * CH + RPI * ii + g; rows past the partition's
    // end are fetched from its last row (valid memory) and masked
    auto load = [&](int i, u32x4 (&Kr)[NI][PPL], u32x4 (&Vr)[NI][PPL]) __attribute__((always_inline)) {
        const int r0 = row_lo + (wave + 4 * i) * CH + g;
#pragma unroll
        for (int ii = 0; ii < NI; ++ii) {
            const int r = min(r0 + RPI * ii, row_hi - 1);
#pragma unroll
            for (int j = 0; j < PPL; ++j) {
                // non-temporal: every byte is used once (measured: 6.1 -> 6.9 TB/s)
                Kr[ii][j] = __builtin_nontemporal_load((const u32x4 *)(Kg + (int64_t)r * k_rb + pofs[j]));
                Vr[ii][j] = __builtin_nontemporal_load((const u32x4 *)(Vg + (int64_t)r * v_rb + pofs[j]));
            }
        }
    };
    auto compute = [&](int i, const u32x4 (&Kr)[NI][PPL], const u32x4 (&Vr)[NI][PPL]) __attribute__((always_inline)) {
        const int r0 = row_lo + (wave + 4 * i) * CH + g;
        float s[NI][WQ];
#pragma unroll
        for (int ii = 0; ii < NI; ++ii) {
            u32x4 kk[PPL];
#pragma unroll
            for (int j = 0; j < PPL; ++j) kk[j] = PAD ? (Kr[ii][j] & keep[j]) : Kr[ii][j];
#pragma unroll
            for (int w = 0; w < WQ; ++w) {
                float acc = 0.f;
#pragma unroll
                for (int j = 0; j < PPL; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (BF) acc = dot2_bf16(kk[j][e], q[w][j][e], acc);
                        else acc = fmaf(as_f32(kk[j][e]), as_f32(q[w][j][e]), acc);
                    }
                s[ii][w] = row16_allsum(acc);
            }
        }
        if (r0 - g + CH > row_hi) {          // ragged last chunk of the partition (uniform over the wave)
#pragma unroll
            for (int ii = 0; ii < NI; ++ii)
                if (r0 + RPI * ii >= row_hi) {
#pragma unroll
                    for (int w = 0; w < WQ; ++w) s[ii][w] = -INFINITY;
                }
        }
#pragma unroll
        for (int w = 0; w < WQ; ++w) {
            float mx = s[0][w];
#pragma unroll
            for (int ii = 1; ii < NI; ++ii) mx = fmaxf(mx, s[ii][w]);
            mx *= a.c;
            // the reference point moves only when a score exceeds it by more than 2^8 (weights stay
            // <= 256, any reference point gives the same normalised result)
            if (__builtin_amdgcn_ballot_w64(mx > m[w] + 8.0f) != 0) {
                const float mn = fmaxf(m[w], mx);
                const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2(m[w] - mn);
                l[w] *= alpha;
#pragma unroll
                for (int e = 0; e < EL; ++e) O[w][e] *= alpha;
                m[w] = mn;
            }
            const float mref = (m[w] == -INFINITY) ? 0.f : m[w];
#pragma unroll
            for (int ii = 0; ii < NI; ++ii) {
                const float p = fast_exp2(fmaf(s[ii][w], a.c, -mref));
                if (BF) {
                    // weight rounded to bf16: (p, 0) multiplies the even columns, (0, p) the odd ones; the
                    // latter's bit pattern is the rounded weight as fp32, which is what the row sum takes
                    const unsigned pe = (unsigned)f32_to_bf16_bits(p);
                    const unsigned po = pe << 16;
                    l[w] += __builtin_bit_cast(float, po);
#pragma unroll
                    for (int j = 0; j < PPL; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            O[w][8 * j + 2 * e] = dot2_bf16(Vr[ii][j][e], pe, O[w][8 * j + 2 * e]);
                            O[w][8 * j + 2 * e + 1] = dot2_bf16(Vr[ii][j][e], po, O[w][8 * j + 2 * e + 1]);
                        }
                } else {
                    l[w] += p;
#pragma unroll
                    for (int j = 0; j < PPL; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            O[w][4 * j + e] = fmaf(p, as_f32(Vr[ii][j][e]), O[w][4 * j + e]);
                }
            }
        }
    };

    if (mine > 0) {
        // two chunks of loads in flight: the next one is requested before the current one is used
        u32x4 K0[NI][PPL], V0[NI][PPL], K1[NI][PPL], V1[NI][PPL];
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

    // ---- join the states (4 waves x RPI row groups) of the workgroup, WB query rows at a time; lane c
    // holds columns (c + LPR j) * EPP ... + EPP - 1 of piece j
    const int sp = wave * RPI + g;
    const int64_t slot = (int64_t)bh * a.nparts + a.part0 + split;
#pragma unroll
    for (int w0 = 0; w0 < WQ; w0 += WB) {
        if (w0 > 0) __syncthreads();
#pragma unroll
        for (int w = 0; w < WB; ++w) {
#pragma unroll
            for (int j = 0; j < PPL; ++j)
#pragma unroll
                for (int e = 0; e < EPP; ++e) Osub[sp][w][(c + LPR * j) * EPP + e] = O[w0 + w][EPP * j + e];
            if (c == 0) {
                msub[sp][w] = m[w0 + w];
                lsub[sp][w] = l[w0 + w];
            }
        }
        __syncthreads();
        for (int idx = tid; idx < WB * DK; idx += 256) {
            const int w = idx / DK, d = idx % DK;
            if (w0 + w >= a.W) break;
            if (PAD && d >= a.D) continue;
            float M = -INFINITY;
#pragma unroll
            for (int k = 0; k < NG; ++k) M = fmaxf(M, msub[k][w]);
            float o = 0.f, L = 0.f;
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                const float wgt = msub[k][w] == -INFINITY ? 0.f : fast_exp2(msub[k][w] - M);
                o += wgt * Osub[k][w][d];
                L += wgt * lsub[k][w];
            }
            a.Opart[(slot * a.W + w0 + w) * DK + d] = o;
            if (d == 0) {
                a.Mpart[slot * a.W + w0 + w] = M;
                a.Lpart[slot * a.W + w0 + w] = L;
            }
        }
    }
}

}  // namespace tlin
