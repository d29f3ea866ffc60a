// fp32 attention over one key partition: plain fp32 FMA arithmetic end to end (no matrix
// cores), for fp32 inputs.  Same online-softmax recurrence and same partial format as the bf16
// kernel (Section 3 of the paper: softmax(scale * Q K^T) V; window keys masked with j <= i).
//
// A workgroup of 256 threads owns 32 query rows and walks its key partition in tiles of 64
// (D=64) or 32 (D=128) keys staged in LDS.  Per tile: scores (each thread a 2 x BN/16 patch),
// a per-row softmax step (8 threads per row), then the value product (each thread 2 rows x
// D/16 columns, as float4 groups).
#pragma once
#include "common.h"

namespace tlin {

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnArgs a)
{
    constexpr int BM = 32, NT = 256;
    constexpr int BN = D == 128 ? 32 : 64;   // keys per tile (keeps static LDS under 64 KB)
    constexpr int LDQ = D + 4;           // padded row strides (floats): 16-byte aligned, bank-spread
    constexpr int LDP = BN + 4;
    constexpr int CPT = D / 64;          // float4 column groups per thread in the value product
    constexpr int SC = BN / 16;          // score columns per thread
    constexpr int SE = BN / 8;           // softmax elements per thread

    __shared__ __attribute__((aligned(16))) float Qs[BM * LDQ];
    __shared__ __attribute__((aligned(16))) float Ks[BN * LDQ];
    __shared__ __attribute__((aligned(16))) float Vs[BN * D];
    __shared__ __attribute__((aligned(16))) float Ps[BM * LDP];
    __shared__ float alpha_s[BM], m_s[BM], l_s[BM];

    const int tid = threadIdx.x;
    const int L = xcd_remap(blockIdx.x, gridDim.x);
    const Problem pr = decode_problem<BM, BN, CAUSAL>(a, L, a.nqb);
    if (pr.skip) return;                 // uniform over the workgroup
    const int qb = pr.qb, split = pr.split, bh = pr.bh;
    const int b = bh / a.H, hd = bh % a.H;
    const int qrow0 = qb * BM;
    const int Wq = pr.W, NK = pr.NK;     // query and key rows of this problem

    int t0, t1;
    if (CAUSAL) {
        t0 = 0;
        t1 = (min(NK, qrow0 + BM) + BN - 1) / BN;
    } else {
        t0 = split * pr.tps;
        t1 = min(t0 + pr.tps, (NK + BN - 1) / BN);
    }

    const float *Qg = (const float *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh + pr.qrow_off * a.q_sr;
    const float *Kg = (const float *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh + pr.krow_off * a.k_sr;
    const float *Vg = (const float *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh + pr.krow_off * a.v_sr;

    for (int i = tid; i < BM * (D / 4); i += NT) {
        const int r = i / (D / 4), c4 = i % (D / 4);
        const int gr = min(qrow0 + r, Wq - 1);
        // columns beyond the tensors' head dimension a.D count as zeros
        *(f32x4 *)(Qs + r * LDQ + 4 * c4) =
            4 * c4 < a.D ? *(const f32x4 *)(Qg + (int64_t)gr * a.q_sr + 4 * c4) : f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // score / value-product ownership: rows 2*ty, 2*ty+1; score columns tx + 16*c
    const int ty = tid >> 4, tx = tid & 15;
    // softmax ownership: row tid/8, columns SE*(tid%8) .. +SE-1; the 8 threads of a row are adjacent lanes
    const int sr = tid >> 3, sc = tid & 7;
    float m_run = -INFINITY, l_run = 0.f;

    f32x4 oacc[2][CPT];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int c = 0; c < CPT; ++c) oacc[r][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int t = t0; t < t1; ++t) {
        const int key0 = t * BN;
        __syncthreads();   // previous tile fully consumed
        for (int i = tid; i < BN * (D / 4); i += NT) {
            const int r = i / (D / 4), c4 = i % (D / 4);
            const int gr = min(key0 + r, NK - 1);
            const bool in = 4 * c4 < a.D;
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            *(f32x4 *)(Ks + r * LDQ + 4 * c4) = in ? *(const f32x4 *)(Kg + (int64_t)gr * a.k_sr + 4 * c4) : zero;
            *(f32x4 *)(Vs + r * D + 4 * c4) = in ? *(const f32x4 *)(Vg + (int64_t)gr * a.v_sr + 4 * c4) : zero;
        }
        __syncthreads();

        // ---- scores in base-2 units: s = c * <q, k>
        float s[2][SC];
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int c = 0; c < SC; ++c) s[r][c] = 0.f;
#pragma unroll 2
        for (int k = 0; k < D; k += 4) {
            f32x4 q0 = *(const f32x4 *)(Qs + (2 * ty) * LDQ + k);
            f32x4 q1 = *(const f32x4 *)(Qs + (2 * ty + 1) * LDQ + k);
#pragma unroll
            for (int c = 0; c < SC; ++c) {
                f32x4 kv = *(const f32x4 *)(Ks + (tx + 16 * c) * LDQ + k);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s[0][c] = fmaf(q0[e], kv[e], s[0][c]);
                    s[1][c] = fmaf(q1[e], kv[e], s[1][c]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int row = qrow0 + 2 * ty + r;
            const int lim = CAUSAL ? min(row, NK - 1) : NK - 1;
#pragma unroll
            for (int c = 0; c < SC; ++c) {
                const int key = key0 + tx + 16 * c;
                Ps[(2 * ty + r) * LDP + tx + 16 * c] = key > lim ? -INFINITY : s[r][c] * a.c;
            }
        }
        __syncthreads();

        // ---- softmax step for row sr
        {
            float v[SE];
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < SE; ++e) {
                v[e] = Ps[sr * LDP + SE * sc + e];
                mx = fmaxf(mx, v[e]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 1));
            mx = fmaxf(mx, __shfl_xor(mx, 2));
            mx = fmaxf(mx, __shfl_xor(mx, 4));
            const float mn = fmaxf(m_run, mx);
            const float mref = (mn == -INFINITY) ? 0.f : mn;
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < SE; ++e) {
                const float p = exp2f(v[e] - mref);
                ps += p;
                Ps[sr * LDP + SE * sc + e] = p;
            }
            ps += __shfl_xor(ps, 1);
            ps += __shfl_xor(ps, 2);
            ps += __shfl_xor(ps, 4);
            const float al = (mn == -INFINITY) ? 1.f : exp2f(m_run - mn);
            l_run = l_run * al + ps;
            m_run = mn;
            if (sc == 0) alpha_s[sr] = al;
        }
        __syncthreads();

        // ---- O = alpha * O + P V
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const float al = alpha_s[2 * ty + r];
#pragma unroll
            for (int c = 0; c < CPT; ++c) oacc[r][c] *= al;
        }
#pragma unroll 2
        for (int jn = 0; jn < BN; jn += 4) {
            const f32x4 p0 = *(const f32x4 *)(Ps + (2 * ty) * LDP + jn);
            const f32x4 p1 = *(const f32x4 *)(Ps + (2 * ty + 1) * LDP + jn);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int c = 0; c < CPT; ++c) {
                    const f32x4 vv = *(const f32x4 *)(Vs + (jn + e) * D + 4 * tx + 64 * c);
                    oacc[0][c] += p0[e] * vv;
                    oacc[1][c] += p1[e] * vv;
                }
        }
    }

    if (sc == 0) {
        m_s[sr] = m_run;
        l_s[sr] = l_run;
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int lr = 2 * ty + r, row = qrow0 + lr;
        if (row >= Wq) continue;
        const float mr = m_s[lr], lt = l_s[lr];
        if (a.direct) {
            const float inv = 1.0f / lt;
            const int64_t off = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh + (pr.qrow_off + row) * a.o_sr;
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const int d = 4 * tx + 64 * c;
                if (d >= a.D) continue;
                const f32x4 o = oacc[r][c] * inv;
                if (a.out_bf16) {
                    bf16x4 ob;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ob[e] = (__bf16)o[e];
                    *(bf16x4 *)((__bf16 *)a.O + off + d) = ob;
                } else {
                    *(f32x4 *)((float *)a.O + off + d) = o;
                }
            }
            // m is in base-2 units (c * raw); natural-log LSE = m * ln 2 + ln l
            if (a.lse && tx == 0) a.lse[(int64_t)bh * a.W + row] = mr * 0.6931471805599453f + logf(lt);
        } else {
            const int64_t slot = pr.slot + a.part0 + (CAUSAL ? 0 : split);
            float *op = a.Opart + (slot * a.W + row) * D;
#pragma unroll
            for (int c = 0; c < CPT; ++c) *(f32x4 *)(op + 4 * tx + 64 * c) = oacc[r][c];
            if (tx == 0) {
                a.Mpart[slot * a.W + row] = mr;
                a.Lpart[slot * a.W + row] = lt;
            }
        }
    }
}

}  // namespace tlin
