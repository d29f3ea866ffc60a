// bf16 attention over one key partition on the gfx950 matrix cores.
//
// Computes, for a block of query rows, softmax(scale * Q K^T) V over the key rows of one
// partition (Section 3 of the paper: the attention primitive; history keys are unmasked, the
// window keys are causally masked with j <= i), in the online (blocked) form: running
// maximum m, running sum l and an unnormalised accumulator per row, rescaled when the
// maximum moves.  The result is either normalised and written out, or written as a partial
// (O_part, m, l) that the merge kernel joins exactly.
//
// Mapping (wave64, v_mfma_f32_32x32x16_bf16):
//   * A wave owns QB blocks of 32 query rows.  Scores are produced TRANSPOSED,
//       S^T[key, query] = K_tile (A operand, from LDS) x Q^T (B operand, registers),
//     so a lane holds 16 keys of ONE query column (lane%32); the other 16 keys of that column
//     sit in lane^32.  Row maxima and sums are therefore in-lane reductions plus a single
//     half-wave swap, and the softmax weights, once rounded to bf16, already have the B-operand
//     layout of the second product
//       O^T[d, query] += V^T (A operand) x P^T (B operand),
//     whose accumulator again keeps one query per lane, so rescaling is a per-lane scalar.
//   * V is stored row-major [key][d]; the A operand needs 4 consecutive keys at fixed d per
//     lane, which is what ds_read_b64_tr_b16 returns (16 lanes read a 4x16 patch and get its
//     transpose).  Two such reads form one 8-element operand.
//   * K/V tiles of 64 keys go HBM -> registers -> LDS with 16-byte accesses, double buffered,
//     one barrier per tile; the next tile's global loads are in flight during compute.
//   * LDS rows are XOR-swizzled at 16-byte-chunk granularity so that the ds_read_b128 of the
//     K operand and the transposed reads of V are bank-conflict free on the 64-bank LDS.
#pragma once
#include "common.h"

namespace tlin {

template <int D> struct Swz;
template <> struct Swz<128> {   // 256-byte rows, 16 chunks
    static __device__ __forceinline__ int k(int r) { return r & 15; }
    // rows r..r+3 are read together by the transposed loads: spread them over {0,2,5,7}*32 B
    static __device__ __forceinline__ int v(int r) { return ((r & 1) << 2) ^ (((r >> 1) & 1) * 10); }
};
template <> struct Swz<64> {    // 128-byte rows, 8 chunks; two rows per 256-byte bank sweep
    static __device__ __forceinline__ int k(int r) { return (r >> 1) & 7; }
    static __device__ __forceinline__ int v(int r) { return ((r >> 1) & 1) << 2; }
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int D, int NW, int QB, bool CAUSAL>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(const AttnArgs a)
{
    constexpr int BN = 64;                 // keys per tile
    constexpr int BM = NW * QB * 32;       // query rows per workgroup
    constexpr int NT = NW * 64;
    constexpr int ROWB = D * 2;            // bytes per K/V row
    constexpr int TILE_B = BN * ROWB;
    constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    constexpr int CHUNKS = BN * CPR;
    constexpr int LPT = CHUNKS / NT;       // chunks per thread per tensor per tile
    static_assert(CHUNKS % NT == 0 && LPT >= 1, "tile does not divide over the workgroup");
    constexpr int DS = D / 16;             // contraction steps of Q K^T
    constexpr int DB = D / 32;             // 32-row blocks of O^T

    __shared__ __attribute__((aligned(1024))) char smem[4 * TILE_B];
    char *const Ks = smem;
    char *const Vs = smem + 2 * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, h = lane >> 5;

    const int L = xcd_remap(blockIdx.x, gridDim.x);
    const int qb = L % a.nqb;
    const int rest = L / a.nqb;
    const int split = rest % a.nsplit;
    const int bh = rest / a.nsplit;
    const int b = bh / a.H, hd = bh % a.H;

    int t0, t1;
    if (CAUSAL) {
        t0 = 0;
        const int kend = min(a.NK, qb * BM + BM);
        t1 = (kend + BN - 1) / BN;
    } else {
        t0 = split * a.tiles_per_split;
        t1 = min(t0 + a.tiles_per_split, (a.NK + BN - 1) / BN);
    }

    const __bf16 *Qg = (const __bf16 *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh;
    const char *Kg = (const char *)((const __bf16 *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh);
    const char *Vg = (const char *)((const __bf16 *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh);
    const int64_t k_rb = a.k_sr * 2, v_rb = a.v_sr * 2;

    // Q^T fragments (B operand): lane holds query j, contraction elements 16*s + 8*h .. +7.
    const int qrow0 = qb * BM + wave * (QB * 32);
    bf16x8 qf[QB][DS];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        const int r = min(qrow0 + qi * 32 + j, a.W - 1);
        const __bf16 *qp = Qg + (int64_t)r * a.q_sr + 8 * h;
#pragma unroll
        for (int s = 0; s < DS; ++s) qf[qi][s] = *(const bf16x8 *)(qp + 16 * s);
    }

    u32x4 kr[LPT], vr[LPT];
    auto gload = [&](int t) {
        const int key0 = t * BN;
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int cid = tid + NT * i;
            const int r = cid / CPR, cc = cid % CPR;
            const int gr = min(key0 + r, a.NK - 1);      // rows past the end repeat the last row (masked later)
            kr[i] = *(const u32x4 *)(Kg + gr * k_rb + cc * 16);
            vr[i] = *(const u32x4 *)(Vg + gr * v_rb + cc * 16);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int cid = tid + NT * i;
            const int r = cid / CPR, cc = cid % CPR;
            *(u32x4 *)(Ks + buf * TILE_B + r * ROWB + ((cc ^ Swz<D>::k(r)) << 4)) = kr[i];
            *(u32x4 *)(Vs + buf * TILE_B + r * ROWB + ((cc ^ Swz<D>::v(r)) << 4)) = vr[i];
        }
    };

    f32x16 oacc[QB][DB];
    float m[QB], l[QB];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        m[qi] = -INFINITY;
        l[qi] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[qi][db][v] = 0.f;
    }
    // The running maximum is only advanced when a row's tile maximum exceeds it by more than
    // 2^8 in the exponent: weights then stay <= 256, and the accumulator is rescaled rarely.
    // Any reference point gives the same normalised result, so this is exact.
    const float thr = 8.0f / a.c;

    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;

    if (t0 < t1) gload(t0);
    for (int t = t0; t < t1; ++t) {
        const int buf = (t - t0) & 1;
        sstore(buf);
        __syncthreads();
        if (t + 1 < t1) gload(t + 1);
        const int key0 = t * BN;
        if (CAUSAL && key0 > qrow0 + QB * 32 - 1) continue;   // tile lies after every row of this wave

        const char *Kt = Ks + buf * TILE_B;
        const char *Vt = Vs + buf * TILE_B;

        // ---- S^T = K Q^T
        f32x16 sacc[QB][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int qi = 0; qi < QB; ++qi)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[qi][kb][v] = 0.f;
            const int key = kb * 32 + j;
            const char *krow = Kt + key * ROWB;
            const int ksw = Swz<D>::k(key);
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                const bf16x8 kf = *(const bf16x8 *)(krow + (((2 * s + h) ^ ksw) << 4));
#pragma unroll
                for (int qi = 0; qi < QB; ++qi)
                    sacc[qi][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qi][s], sacc[qi][kb], 0, 0, 0);
            }
        }

        // ---- mask: keys past the end of the tensor, and (causal) keys after the query row
        const bool ragged = key0 + BN > a.NK;
        const bool diag = CAUSAL && (key0 + BN - 1 > qrow0);
        if (ragged || diag) {
#pragma unroll
            for (int qi = 0; qi < QB; ++qi) {
                const int row = qrow0 + qi * 32 + j;
                const int lim = CAUSAL ? min(row, a.NK - 1) : a.NK - 1;   // last visible key
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                        if (key > lim) sacc[qi][kb][v] = -INFINITY;
                    }
            }
        }

        // ---- online softmax, weights to bf16 in B-operand order
        bf16x8 pb[QB][2][2];
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) {
            float mx = sacc[qi][0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[qi][kb][v]);
            mx = xhalf_max(mx);
            if (__builtin_amdgcn_ballot_w64(mx > m[qi] + thr) != 0) {
                const float mn = fmaxf(m[qi], mx);
                const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2((m[qi] - mn) * a.c);
                l[qi] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[qi][db][v] *= alpha;
                m[qi] = mn;
            }
            const float mc = (m[qi] == -INFINITY) ? 0.f : m[qi] * a.c;
            float ls = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = fast_exp2(fmaf(sacc[qi][kb][v], a.c, -mc));
                    ls += p;
                    sacc[qi][kb][v] = p;
                }
            l[qi] += ls;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pb[qi][kb][t2][e] = (__bf16)sacc[qi][kb][8 * t2 + e];
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                // operand element e of half-wave h is key kb*32 + 16*t2 + 8*(e/4) + 4*h + e%4
                const int r0 = kb * 32 + 16 * t2 + 4 * h + (i16 >> 2);
                const int r1 = r0 + 8;
                const char *v0 = Vt + r0 * ROWB;
                const char *v1 = Vt + r1 * ROWB;
                const int sw0 = Swz<D>::v(r0) << 4, sw1 = Swz<D>::v(r1) << 4;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int cb = 64 * db + 32 * blk1 + 8 * (i16 & 3);
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(v0 + (cb ^ sw0)));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(v1 + (cb ^ sw1)));
                    const bf16x8 vf = __builtin_bit_cast(
                        bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                    for (int qi = 0; qi < QB; ++qi)
                        oacc[qi][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[qi][kb][t2], oacc[qi][db], 0, 0, 0);
                }
            }
    }

    // ---- epilogue.  Accumulator register v of block db is d = 32*db + 8*(v/4) + 4*h + v%4.
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        const float lt = xhalf_sum(l[qi]);
        const int row = qrow0 + qi * 32 + j;
        if (row >= a.W) continue;
        if (a.direct) {
            const float inv = 1.0f / lt;
            const int64_t off = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh + (int64_t)row * a.o_sr;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = 32 * db + 8 * g + 4 * h;
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = oacc[qi][db][4 * g + e] * inv;
                    if (a.out_bf16) {
                        bf16x4 ob;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ob[e] = (__bf16)o[e];
                        *(bf16x4 *)((__bf16 *)a.O + off + d) = ob;
                    } else {
                        *(f32x4 *)((float *)a.O + off + d) = o;
                    }
                }
            if (a.lse && h == 0) a.lse[(int64_t)bh * a.W + row] = m[qi] * a.scale + __logf(lt);
        } else {
            const int64_t slot = (int64_t)bh * a.nparts + a.part0 + (CAUSAL ? 0 : split);
            float *op = a.Opart + (slot * a.W + row) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = oacc[qi][db][4 * g + e];
                    *(f32x4 *)(op + 32 * db + 8 * g + 4 * h) = o;
                }
            if (h == 0) {
                a.Mpart[slot * a.W + row] = m[qi] * a.c;
                a.Lpart[slot * a.W + row] = lt;
            }
        }
    }
}

}  // namespace tlin
