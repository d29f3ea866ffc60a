// bf16 history attention on the gfx950 matrix cores with two wave groups in ping-pong.
// Same arithmetic, operand mapping, LDS layout and direct-load tile ring as attn_bf16_kernel
// (see attn_bf16.h); what differs is how a wave's work is cut into phases and how the two
// waves that share a SIMD are kept in opposite phases.
//
// A wave with one instruction stream cannot hide LDS, transcendental and matrix-core latencies
// by itself, and two identical waves per SIMD drift into lockstep, so matrix cores and vector
// ALUs end up taking turns.  Here each wave alternates between two kinds of phase on 32-key
// blocks b = 0, 1, ...:
//     X(b)  matrix cores, operands streamed from LDS a few instructions ahead of their use:
//             S(b+1) = K(b+1) Q^T            and        O += V(b)^T P(b)^T
//     Y(b)  vector ALU and bookkeeping:
//             P(b+1) = softmax step on S(b+1);  rescale O if the running maximum moved;
//             tile-ring bookkeeping (wait / issue);  first operands of X(b+1) LDS -> registers
// and every phase ends at a workgroup barrier.  Waves 0..NW/2-1 (one per SIMD) start one phase
// ahead of waves NW/2..NW-1 (their SIMD partners), so in every slot between two barriers a SIMD
// has one wave in X and one in Y.  Both groups execute the same number of barriers.
//
// The row sum l is accumulated from the bf16-rounded weights (v_dot2c_f32_bf16 against ones),
// i.e. from exactly the values the value product uses.
#pragma once
#include "attn_bf16.h"

namespace tlin {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

template <int D, int NW, int NSTAGE>
__global__ __launch_bounds__(NW * 64) void attn_bf16_pp_kernel(const AttnArgs a)
{
    constexpr int BN = 64;                 // keys per tile (two blocks of 32)
    constexpr int BM = NW * 32;            // query rows per workgroup
    constexpr int ROWB = D * 2;            // bytes per K/V row
    constexpr int TILE_B = BN * ROWB;
    constexpr int BLK_B = 32 * ROWB;       // bytes per 32-key block
    constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;       // rows moved by one wave-wide direct load
    constexpr int NDMA = BN / RPI / NW;    // direct loads per wave per tensor per tile
    static_assert(NW % 2 == 0, "two wave groups");
    static_assert(BN % (RPI * NW) == 0 && NDMA >= 1, "tile does not divide over the waves");
    constexpr int DS = D / 16;             // contraction steps of Q K^T
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    constexpr int PER_TILE = 2 * NDMA;     // direct loads per wave per tile
    static_assert(NSTAGE >= 3, "ring too shallow");
    static_assert(NSTAGE * PER_TILE < 64, "too many loads in flight for vmcnt");

    extern __shared__ __attribute__((aligned(1024))) char smem[];   // 2 * NSTAGE * TILE_B bytes
    char *const Ks = smem;
    char *const Vs = smem + NSTAGE * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
    const bool second = wave >= NW / 2;    // this wave's group runs one phase behind

    const int L = xcd_remap(blockIdx.x, gridDim.x);
    const int qb = L % a.nqb;
    const int rest = L / a.nqb;
    const int split = rest % a.nsplit;
    const int bh = rest / a.nsplit;
    const int b = bh / a.H, hd = bh % a.H;

    const int t0 = split * a.tiles_per_split;
    const int t1 = min(t0 + a.tiles_per_split, (a.NK + BN - 1) / BN);
    const int ntl = t1 - t0;               // tiles of this partition (>= 1 by construction)

    const __bf16 *Qg = (const __bf16 *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh;
    const char *Kg = (const char *)((const __bf16 *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh);
    const char *Vg = (const char *)((const __bf16 *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh);
    const int64_t k_rb = a.k_sr * 2, v_rb = a.v_sr * 2;

    // Q^T fragments (B operand): lane holds query j, contraction elements 16*s + 8*h .. +7.
    const int qrow0 = qb * BM + wave * 32;
    bf16x8 qf[DS];
    {
        const int r = min(qrow0 + j, a.W - 1);
        const __bf16 *qp = Qg + (int64_t)r * a.q_sr + 8 * h;
#pragma unroll
        for (int s = 0; s < DS; ++s) qf[s] = *(const bf16x8 *)(qp + 16 * s);
        // consume them here so the wait for these loads sits before the loop, not inside it
#pragma unroll
        for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(qf[s]));
    }

    // ---- tile ring: direct HBM -> LDS loads, swizzle applied on the source side
    int drow[NDMA];
    int64_t koff[NDMA], voff[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        drow[i] = (wave * NDMA + i) * RPI + lane / CPR;
        koff[i] = drow[i] * k_rb + (((lane % CPR) ^ Swz<D>::k(drow[i])) << 4);
        voff[i] = drow[i] * v_rb + (((lane % CPR) ^ Swz<D>::v(drow[i])) << 4);
    }
    // tile index T is relative to the partition; it lives in stage T % NSTAGE
    auto issue = [&](int T) {
        const int key0 = (t0 + T) * BN;
        const unsigned kdst = __builtin_amdgcn_readfirstlane(lds_offset(Ks) + (T % NSTAGE) * TILE_B + wave * (NDMA * 1024));
        const unsigned vdst = kdst + NSTAGE * TILE_B;
        if (key0 + BN <= a.NK) {
            const char *kt = Kg + key0 * k_rb, *vt = Vg + key0 * v_rb;
#pragma unroll
            for (int i = 0; i < NDMA; ++i) {
                direct_load_1k(kt + koff[i], kdst + i * 1024);
                direct_load_1k(vt + voff[i], vdst + i * 1024);
            }
        } else {
            // ragged last tile: rows past the end repeat the last row (their scores are masked)
#pragma unroll
            for (int i = 0; i < NDMA; ++i) {
                const int64_t back = max(key0 + drow[i] - (a.NK - 1), 0);
                direct_load_1k(Kg + (key0 - back) * k_rb + koff[i], kdst + i * 1024);
                direct_load_1k(Vg + (key0 - back) * v_rb + voff[i], vdst + i * 1024);
            }
        }
    };

    // ---- per-lane LDS read offsets inside a 32-key block (the block base is added per use)
    int kbase[DS], vbase[DB];
    {
        const int ksw = Swz<D>::k(j);                      // same for keys j and j + 32
#pragma unroll
        for (int s = 0; s < DS; ++s) kbase[s] = j * ROWB + (((2 * s + h) ^ ksw) << 4);
        const int vr = 4 * h + (i16 >> 2);                 // row of the 4x16 patch this lane addresses
        const int vsw = Swz<D>::v(vr) << 4;                // unchanged by adding multiples of 8 rows
#pragma unroll
        for (int db = 0; db < DB; ++db) vbase[db] = vr * ROWB + ((64 * db + 32 * blk1 + 8 * (i16 & 3)) ^ vsw);
    }
    // block index blk counts 32-key blocks of the partition: tile blk/2, half blk%2
    auto kblock = [&](int blk) { return Ks + ((blk >> 1) % NSTAGE) * TILE_B + (blk & 1) * BLK_B; };
    auto vblock = [&](int blk) { return Vs + ((blk >> 1) % NSTAGE) * TILE_B + (blk & 1) * BLK_B; };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float thr = 8.0f / a.c;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    bf16x8 P[2];            // softmax weights of the block whose value product is next, B-operand order
    f32x16 S;               // scores waiting for their softmax step

    auto phase_end = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    auto lds_done = [&]() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); };

    // Operand i of an X phase, i = 0 .. 2*DS-1: even i is K fragment i/2 of the score block,
    // odd i is V fragment i/2 (t2 = (i/2) / DB, db = (i/2) % DB) of the value block.
    constexpr int NOPS = 2 * DS;
#ifndef TLIN_LA
#define TLIN_LA 3
#endif
    constexpr int LA = TLIN_LA;             // operands requested ahead of their use
    auto fetch = [&](const char *Kb, const char *Vb, int i) -> bf16x8 {
        if ((i & 1) == 0) return *(const bf16x8 *)(Kb + kbase[i >> 1]);
        const int t2 = (i >> 1) / DB, db = (i >> 1) % DB;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(Vb + (16 * t2) * ROWB + vbase[db]));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(Vb + (16 * t2 + 8) * ROWB + vbase[db]));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    bf16x8 ring[LA + 1];    // operands in flight; ring[0..LA-1] are filled at the end of a Y phase
    auto prefetch = [&](int score_blk, int value_blk) {
        const char *Kb = kblock(score_blk), *Vb = vblock(value_blk);
#pragma unroll
        for (int i = 0; i < LA; ++i) ring[i] = fetch(Kb, Vb, i);
    };
    // X phase: scores of block score_blk and value product of block value_blk, interleaved so
    // that the dependent score chain (one accumulator) alternates with the value products
    // (DB accumulators).  Each step requests the operand LA steps ahead, then issues one product.
    auto mfma_both = [&](int score_blk, int value_blk) {
        const char *Kb = kblock(score_blk), *Vb = vblock(value_blk);
#pragma unroll
        for (int v = 0; v < 16; ++v) S[v] = 0.f;
#pragma unroll
        for (int i = 0; i < NOPS; ++i) {
            if (i + LA < NOPS) ring[(i + LA) % (LA + 1)] = fetch(Kb, Vb, i + LA);
            const bf16x8 A = ring[i % (LA + 1)];
            if ((i & 1) == 0) {
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, qf[i >> 1], S, 0, 0, 0);
            } else {
                const int t2 = (i >> 1) / DB, db = (i >> 1) % DB;
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, P[t2], oacc[db], 0, 0, 0);
            }
            if (i + LA < NOPS) {   // the DS reads of that request: one b128 (K) or two transposed b64 (V)
                if ((i + LA) & 1) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          // one MFMA
        }
    };
    auto mfma_scores_only = [&](int score_blk) {
        const char *Kb = kblock(score_blk);
#pragma unroll
        for (int v = 0; v < 16; ++v) S[v] = 0.f;
#pragma unroll
        for (int s = 0; s < DS; ++s) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fetch(Kb, Kb, 2 * s), qf[s], S, 0, 0, 0);
    };
    auto mfma_values_only = [&](int value_blk) {
        const char *Vb = vblock(value_blk);
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int db = 0; db < DB; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fetch(Vb, Vb, 2 * (t2 * DB + db) + 1), P[t2], oacc[db], 0, 0, 0);
    };

    // Online-softmax step on S, whose register v is key key0 + 8*(v/4) + 4*h + v%4; weights go
    // to P; returns the factor by which the accumulator must be rescaled (1 unless this row's
    // maximum moved).  The running maximum only advances when the block maximum exceeds it by
    // more than 2^8 in the exponent (weights stay <= 256); any reference point gives the same
    // normalised result.
    auto softmax = [&](int key0) -> float {
        if (key0 + 32 > a.NK) {   // only the last tile of the tensor can be ragged
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (key0 + 8 * (v >> 2) + 4 * h + (v & 3) >= a.NK) S[v] = -INFINITY;
        }
        float mx = S[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, S[v]);
        mx = xhalf_max(mx);
        const bool move = mx > m + thr;
        const float mn = move ? mx : m;
        const float alpha = move ? fast_exp2((m - mn) * a.c) : 1.f;   // m = -inf: exp2(-inf) = 0
        l *= alpha;
        m = mn;
        const float mc = (m == -INFINITY) ? 0.f : m * a.c;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int e = 0; e < 8; ++e) P[t2][e] = (__bf16)fast_exp2(fmaf(S[8 * t2 + e], a.c, -mc));
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const bf16x2 pp = {P[t2][e], P[t2][e + 1]};
                l = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, l, false);
            }
        return alpha;
    };
    auto rescale = [&](float alpha) {
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
        }
    };
    // this wave's loads of tile T have landed (tiles up to `issued`-1 have been issued)
    auto wait_tile = [&](int T, int issued) {
        if (issued - 1 - T >= NSTAGE - 3 && NSTAGE > 3) {
            if (issued - 1 - T == NSTAGE - 3) wait_vmcnt<(NSTAGE - 3) * PER_TILE>();
            else wait_vmcnt<(NSTAGE - 2) * PER_TILE>();   // only reached if more were issued
        } else {
            wait_vmcnt<0>();
        }
    };

    // ---- start-up: the whole ring in flight, tile 0 visible to everybody
    int issued = 0;
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s)
        if (s < ntl) { issue(s); ++issued; }
    if (issued == NSTAGE) wait_vmcnt<(NSTAGE - 1) * PER_TILE>();
    else wait_vmcnt<0>();
    phase_end();
    if (second) phase_end();               // the second group stays one phase behind from here on

    mfma_scores_only(0);                   // S(0)
    phase_end();
    (void)softmax(t0 * BN);                // P(0); the accumulator is still zero
    if (ntl > 1) wait_tile(1, issued);
    prefetch(1, 0);
    lds_done();
    phase_end();

    for (int T = 0; T + 1 < ntl; ++T) {
        const int key0 = (t0 + T) * BN;
        // X(2T): S(2T+1), O += P(2T) V(2T)
        mfma_both(2 * T + 1, 2 * T);
        phase_end();
        // Y(2T): P(2T+1)
        rescale(softmax(key0 + 32));
        prefetch(2 * T + 2, 2 * T + 1);
        lds_done();
        phase_end();
        // X(2T+1): S(2T+2), O += P(2T+1) V(2T+1)
        mfma_both(2 * T + 2, 2 * T + 1);
        phase_end();
        // Y(2T+1): P(2T+2).  Tile T is now free in this wave's view, and was freed by the other
        // group at the latest one phase ago: refill its stage.
        rescale(softmax(key0 + BN));
        if (T + 2 < ntl) wait_tile(T + 2, issued);
        if (issued < ntl) { issue(issued); ++issued; }
        prefetch(2 * T + 3, 2 * T + 2);
        lds_done();
        phase_end();
    }
    // last tile: X(nb-2), Y(nb-2) without a successor, X(nb-1) = the last value product
    mfma_both(2 * ntl - 1, 2 * ntl - 2);
    phase_end();
    rescale(softmax((t1 - 1) * BN + 32));
    phase_end();
    mfma_values_only(2 * ntl - 1);
    if (!second) phase_end();              // balance the barrier count of the two groups

    // ---- epilogue.  Accumulator register v of block db is d = 32*db + 8*(v/4) + 4*h + v%4.
    const float lt = xhalf_sum(l);
    const int row = qrow0 + j;
    if (row >= a.W) return;
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
                for (int e = 0; e < 4; ++e) o[e] = oacc[db][4 * g + e] * inv;
                if (a.out_bf16) {
                    bf16x4 ob;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ob[e] = (__bf16)o[e];
                    *(bf16x4 *)((__bf16 *)a.O + off + d) = ob;
                } else {
                    *(f32x4 *)((float *)a.O + off + d) = o;
                }
            }
        if (a.lse && h == 0) a.lse[(int64_t)bh * a.W + row] = m * a.scale + logf(lt);
    } else {
        const int64_t slot = (int64_t)bh * a.nparts + a.part0 + split;
        float *op = a.Opart + (slot * a.W + row) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = oacc[db][4 * g + e];
                *(f32x4 *)(op + 32 * db + 8 * g + 4 * h) = o;
            }
        if (h == 0) {
            a.Mpart[slot * a.W + row] = m * a.c;
            a.Lpart[slot * a.W + row] = lt;
        }
    }
}

}  // namespace tlin
