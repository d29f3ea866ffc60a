// bf16 history attention on the gfx950 matrix cores for wide windows: 64 query rows per wave,
// one wave per SIMD, software-pipelined inside the wave.
//
// Same arithmetic, operand mapping, LDS layout and direct-load tile ring as attn_bf16_kernel
// (see attn_bf16.h).  What differs:
//   * A wave owns TWO blocks of 32 query rows, so every K or V fragment read from LDS feeds two
//     matrix instructions.  With 32 rows per wave the LDS read path is about as busy as the
//     matrix cores (1 KB of operand per 32-cycle instruction and SIMD); with 64 it is half.
//     The price is registers: 128 accumulator + 64 query-fragment registers, so a wave needs
//     the whole 512-register file of its SIMD and has no partner wave to hide its latencies.
//   * Latencies are therefore hidden inside the one instruction stream.  The unit of work is a
//     block of 32 keys, and a step b carries three independent pieces of work,
//         S(b+2) = K(b+2) Q^T            matrix cores   (scores two blocks ahead)
//         P(b+1) = softmax step on S(b+1) vector ALU     (max, exp2, row sum, round to bf16)
//         O     += V(b)^T P(b)^T          matrix cores   (value product of the oldest block)
//     written as one basic block; the operands of the matrix instructions are requested from
//     LDS LA instructions-pairs ahead of their use, and the instruction order is pinned with
//     scheduling groups: two matrix instructions, the LDS reads of one operand, a slice of the
//     softmax arithmetic, repeated.
//   * When a row's running maximum has to move (rare: only when a block maximum exceeds it by
//     2^8), the accumulator is rescaled after the value product of the step.
// The row sum l is accumulated from the bf16-rounded weights (v_dot2c_f32_bf16 against ones),
// i.e. from exactly the values the value product uses.
#pragma once
#include <type_traits>

#include "attn_bf16.h"

namespace tlin {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

template <int D, int NW, int RB, int NSTAGE>
__global__ __launch_bounds__(NW * 64) void attn_bf16_w64_kernel(const AttnArgs a)
{
    constexpr int BN = 64;                 // keys per tile (two blocks of 32)
    static_assert(RB == 1 || RB == 2, "32-row query blocks per wave");
    constexpr int BM = NW * RB * 32;       // query rows per workgroup
    constexpr int ROWB = D * 2;            // bytes per K/V row
    constexpr int TILE_B = BN * ROWB;
    constexpr int BLK_B = 32 * ROWB;       // bytes per 32-key block
    constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;       // rows moved by one wave-wide direct load
    constexpr int NDMA = BN / RPI / NW;    // direct loads per wave per tensor per tile
    static_assert(BN % (RPI * NW) == 0 && NDMA >= 1, "tile does not divide over the waves");
    constexpr int DS = D / 16;             // contraction steps of Q K^T
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    constexpr int PER_TILE = 2 * NDMA;     // direct loads per wave per tile
    static_assert(NSTAGE >= 3, "scores run one tile ahead of the value product");
    static_assert((NSTAGE - 1) * PER_TILE < 64, "too many loads in flight for vmcnt");
    constexpr int NOPS = 2 * DS;           // operands per step: DS of K, 2*DB = DS of V
    constexpr int LA = 4;                  // operands requested ahead of their use

    extern __shared__ __attribute__((aligned(1024))) char smem[];   // 2 * NSTAGE * TILE_B + NW * 4096 bytes
    char *const Ks = smem;
    char *const Vs = smem + NSTAGE * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;

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

    // Q^T fragments (B operand): lane holds query j of row block r, contraction elements 16*s + 8*h .. +7.
    const int qrow0 = qb * BM + wave * (RB * 32);
    bf16x8 qf[RB][DS];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const int row = min(qrow0 + r * 32 + j, a.W - 1);
        const __bf16 *qp = Qg + (int64_t)row * a.q_sr + 8 * h;
#pragma unroll
        for (int s = 0; s < DS; ++s) qf[r][s] = *(const bf16x8 *)(qp + 16 * s);
    }
    // consume them here so the wait for these loads sits before the loop, not inside it
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(qf[r][s]));

    // ---- tile ring: direct HBM -> LDS loads, swizzle applied on the source side
    int drow[NDMA];
    int64_t koff[NDMA], voff[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        drow[i] = (wave * NDMA + i) * RPI + lane / CPR;
        koff[i] = drow[i] * k_rb + (((lane % CPR) ^ Swz<D>::k(drow[i])) << 4);
        voff[i] = drow[i] * v_rb + (((lane % CPR) ^ Swz<D>::v(drow[i])) << 4);
    }
    // direct load number idx (0 .. PER_TILE-1: K and V alternate) of tile T, which goes to stage T % NSTAGE
    auto issue_one = [&](int T, int idx) __attribute__((always_inline)) {
        const int key0 = (t0 + T) * BN;
        const int i = idx >> 1;
        const bool isv = idx & 1;
        const unsigned dst = __builtin_amdgcn_readfirstlane(lds_offset(isv ? Vs : Ks) + (T % NSTAGE) * TILE_B + wave * (NDMA * 1024) + i * 1024);
        const char *g = isv ? Vg : Kg;
        const int64_t rb = isv ? v_rb : k_rb;
        const int64_t off = isv ? voff[i] : koff[i];
        // ragged last tile: rows past the end repeat the last row (their scores are masked)
        const int64_t back = (key0 + BN <= a.NK) ? 0 : max(key0 + drow[i] - (a.NK - 1), 0);
        direct_load_1k(g + (key0 - back) * rb + off, dst);
    };
    auto issue = [&](int T) __attribute__((always_inline)) {
#pragma unroll
        for (int idx = 0; idx < PER_TILE; ++idx) issue_one(T, idx);
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

    f32x16 oacc[RB][DB];
    float m[RB], l[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        m[r] = -INFINITY;
        l[r] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[r][db][v] = 0.f;
    }
    const float thr = 8.0f / a.c;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    // Operand i of a step, i = 0 .. NOPS-1: even i is K fragment i/2 of the score block, odd i is
    // V fragment i/2 (t2 = (i/2) / DB, db = (i/2) % DB) of the value block.
    auto fetch = [&](const char *Kb, const char *Vb, int i) __attribute__((always_inline)) -> bf16x8 {
        if ((i & 1) == 0) return *(const bf16x8 *)(Kb + kbase[i >> 1]);
        const int t2 = (i >> 1) / DB, db = (i >> 1) % DB;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(Vb + (16 * t2) * ROWB + vbase[db]));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(Vb + (16 * t2 + 8) * ROWB + vbase[db]));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // Online softmax: the running maximum of a row only advances when a block maximum exceeds it
    // by more than 2^8 in the exponent (weights stay <= 256); any reference point gives the same
    // normalised result.  Register v of a score block is key key0 + 8*(v/4) + 4*h + v%4.
    // Rescaling the accumulators is rare, and it must not make them vector-ALU operands: they
    // live in the accumulation registers, which only the matrix instructions and memory
    // instructions can address, and the register allocator keeps them there only if no other
    // instruction touches them.  So a block of 16 accumulator registers is bounced through this
    // wave's 4 KB of LDS: stored from the accumulation registers, read back as ordinary
    // registers, scaled, stored, and loaded into the accumulation registers again.
    typedef __attribute__((address_space(3))) volatile f32x16 lds_f32x16;
    lds_f32x16 *bounce = (lds_f32x16 *)(__attribute__((address_space(3))) char *)(smem + 2 * NSTAGE * TILE_B + wave * 4096) + lane;
    auto rescale = [&](float (&alpha)[RB]) __attribute__((always_inline)) {
        bool any = false;
#pragma unroll
        for (int r = 0; r < RB; ++r) any |= alpha[r] != 1.f;
        if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    *bounce = oacc[r][db];
                    f32x16 t = *bounce;
#pragma unroll
                    for (int v = 0; v < 16; ++v) t[v] *= alpha[r];
                    *bounce = t;
                    oacc[r][db] = *bounce;
                }
        }
    };

    // Pieces of the online-softmax step of row block r, cut so that they can be spread over the
    // slots of a pipeline step.  State between the pieces: mx_[r] block maximum, mc_[r] reference
    // point in base-2 units, al_[r] rescale factor.
    float mx_[RB], mc_[RB], al_[RB];
    auto sm_mask = [&](int r, f32x16 &S, int key0) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
            if (key0 + 8 * (v >> 2) + 4 * h + (v & 3) >= a.NK) S[v] = -INFINITY;
    };
    auto sm_max = [&](int r, const f32x16 &S) __attribute__((always_inline)) {
        float mx = S[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, S[v]);
        mx_[r] = mx;
    };
    auto sm_ref = [&](int r) __attribute__((always_inline)) {
        const float mx = xhalf_max(mx_[r]);
        const bool move = mx > m[r] + thr;
        const float mn = move ? mx : m[r];
        al_[r] = move ? fast_exp2((m[r] - mn) * a.c) : 1.f;   // m = -inf: exp2(-inf) = 0
        l[r] *= al_[r];
        m[r] = mn;
        mc_[r] = (mn == -INFINITY) ? 0.f : mn * a.c;
    };
    // weights 2*pr, 2*pr+1 of operand half t2 (elements 8*t2 + 2*pr, +1 of S), pr = 0..3
    auto sm_pair = [&](int r, const f32x16 &S, bf16x8 (&P)[2], int t2, int pr) __attribute__((always_inline)) {
        const int e = 2 * pr;
        P[t2][e] = (__bf16)fast_exp2(fmaf(S[8 * t2 + e], a.c, -mc_[r]));
        P[t2][e + 1] = (__bf16)fast_exp2(fmaf(S[8 * t2 + e + 1], a.c, -mc_[r]));
        const bf16x2 pp = {P[t2][e], P[t2][e + 1]};
        l[r] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, l[r], false);
    };

    // One pipeline step.  SCORES: compute Snew = scores of block score_blk.  SOFTMAX: turn Sold
    // (scores of the block starting at key old_key0) into weights Pnew.  VALUES: add the value
    // product of block value_blk with weights Pcur.  MASKED: Sold may contain keys >= NK.
    //
    // The step is written as NOPS slots separated by scheduling fences.  Slot i holds the LDS
    // reads of operand i+LA, the two matrix instructions that consume operand i (one per row
    // block), and a slice of the softmax arithmetic, which the vector ALU executes while the
    // matrix cores work: slots 0-3 find the block maxima and reference points of the two row
    // blocks, the rest exponentiate, round and sum the weights pair by pair.
    auto step = [&](auto scores, auto sm, auto vals, auto masked, int score_blk, int value_blk, int old_key0,
                    f32x16 (&Snew)[RB], f32x16 (&Sold)[RB], bf16x8 (&Pcur)[RB][2], bf16x8 (&Pnew)[RB][2],
                    int dma_tile = -1, int dma_first = 0) __attribute__((always_inline)) {
        constexpr bool SC = decltype(scores)::value, SM = decltype(sm)::value, VA = decltype(vals)::value;
        constexpr bool MK = decltype(masked)::value;
        const char *Kb = kblock(score_blk), *Vb = vblock(value_blk);
        auto used = [&](int i) { return (i & 1) ? VA : SC; };
        bf16x8 ring[LA + 1];
#pragma unroll
        for (int i = 0; i < LA; ++i)
            if (used(i)) ring[i] = fetch(Kb, Vb, i);
        if (SC) {
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int v = 0; v < 16; ++v) Snew[r][v] = 0.f;
        }
        if (SM && MK) {
#pragma unroll
            for (int r = 0; r < RB; ++r) sm_mask(r, Sold[r], old_key0);
        }
        // softmax work list: 2 + 2 setup pieces, then RB * 8 pairs over the remaining slots
        constexpr int NPAIR = RB * 8;
        constexpr int SETUP = RB == 2 ? 4 : 2;      // slots spent on maxima and reference points
        constexpr int PSLOTS = NOPS - SETUP;        // slots available for the pairs
#pragma unroll
        for (int i = 0; i < NOPS; ++i) {
            __builtin_amdgcn_sched_barrier(0);
            if (i + LA < NOPS && used(i + LA)) ring[(i + LA) % (LA + 1)] = fetch(Kb, Vb, i + LA);
            if (used(i)) {
                const bf16x8 A = ring[i % (LA + 1)];
                if ((i & 1) == 0) {
#pragma unroll
                    for (int r = 0; r < RB; ++r) Snew[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, qf[r][i >> 1], Snew[r], 0, 0, 0);
                } else {
                    const int t2 = (i >> 1) / DB, db = (i >> 1) % DB;
#pragma unroll
                    for (int r = 0; r < RB; ++r) oacc[r][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, Pcur[r][t2], oacc[r][db], 0, 0, 0);
                }
            }
            // one direct load of the tile being refilled every other slot, so that the four waves
            // do not queue up at the memory pipeline with a whole tile each
            if (SC && SM && VA && (i & 1) == 0 && (i >> 1) < PER_TILE / 2 && dma_tile >= 0) issue_one(dma_tile, dma_first + (i >> 1));
            if (SM) {
                if (i == 0) sm_max(0, Sold[0]);
                else if (i == 1) { sm_ref(0); if (RB == 2) sm_max(RB - 1, Sold[RB - 1]); }
                else if (i == 2 && RB == 2) sm_ref(RB - 1);
                else if (i >= SETUP) {
                    // pairs [lo, hi) of the work list go to this slot
                    const int lo = (i - SETUP) * NPAIR / PSLOTS, hi = (i - SETUP + 1) * NPAIR / PSLOTS;
#pragma unroll
                    for (int q = lo; q < hi; ++q) sm_pair(q / 8, Sold[q / 8], Pnew[q / 8], (q % 8) / 4, q % 4);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (SM && VA) {
            float alpha[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) alpha[r] = al_[r];
            // keep the weights in this basic block (they are first used after the branch below)
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) asm volatile("" : "+v"(Pnew[r][t2]));
            rescale(alpha);
        }
    };
    constexpr std::false_type no{};
    constexpr std::true_type yes{};

    // this wave's loads of tile T have landed, given that tiles 0 .. issued-1 have been issued
    auto wait_tile = [&](int T, int issued) __attribute__((always_inline)) {
        const int newer = issued - 1 - T;
        if (newer >= NSTAGE - 2) wait_vmcnt<(NSTAGE - 2) * PER_TILE>();
        else if (newer == NSTAGE - 3 && NSTAGE > 3) wait_vmcnt<(NSTAGE - 3) * PER_TILE>();
        else wait_vmcnt<0>();
    };

    // ---- prologue: NSTAGE-1 tiles in flight; scores of tile 0, weights of its first block
    int issued = 0;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < ntl) { issue(s); ++issued; }
    wait_tile(0, issued);
    __builtin_amdgcn_s_barrier();

    f32x16 SA[RB], SB[RB], Sx[RB];       // Sx, Px: never-used stand-ins for the arguments a step does not touch
    bf16x8 P0[RB][2], P1[RB][2], Px[RB][2];
    step(yes, no, no, no, 0, 0, 0, SB, Sx, Px, P1);                  // SB = S(0)
    step(yes, yes, no, yes, 1, 0, t0 * BN, SA, SB, Px, P0);          // SA = S(1); P0 = weights of block 0

    // ---- steady state.  Entering iteration T: SA = scores of block 2T+1, P0 = weights of block 2T.
    // The iteration reads K of tile T+1 and V of tile T; every wave has finished with tile T-1 when
    // it passes the barrier, so that stage is refilled.  Block 2T+2 (first of tile T+1) may be
    // ragged when tile T+1 is the last one of the tensor.
    auto iteration = [&](auto last, int T) __attribute__((always_inline)) {
        wait_tile(T + 1, issued);
        __builtin_amdgcn_s_barrier();
        const int refill = issued < ntl ? issued : -1;   // its loads are spread over the two steps
        const int key0 = (t0 + T) * BN;
        step(yes, yes, yes, no, 2 * T + 2, 2 * T, key0 + 32, SB, SA, P0, P1, refill, 0);                 // SB = S(2T+2), P1 = P(2T+1), O += P0 V(2T)
        step(yes, yes, yes, last, 2 * T + 3, 2 * T + 1, key0 + BN, SA, SB, P1, P0, refill, PER_TILE / 2);  // SA = S(2T+3), P0 = P(2T+2), O += P1 V(2T+1)
        if (refill >= 0) ++issued;
    };
    for (int T = 0; T + 2 < ntl; ++T) iteration(no, T);
    if (ntl >= 2) iteration(yes, ntl - 2);

    // ---- last tile: no successor to compute scores for
    {
        const int T = ntl - 1;
        step(no, yes, yes, yes, 0, 2 * T, (t0 + T) * BN + 32, Sx, SA, P0, P1);     // P1 = P(2T+1), O += P0 V(2T)
        step(no, no, yes, no, 0, 2 * T + 1, 0, Sx, SB, P1, Px);                    // O += P1 V(2T+1)
    }

    // ---- epilogue.  Accumulator register v of block db is d = 32*db + 8*(v/4) + 4*h + v%4.
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const float lt = xhalf_sum(l[r]);
        const int row = qrow0 + r * 32 + j;
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
                    for (int e = 0; e < 4; ++e) o[e] = oacc[r][db][4 * g + e] * inv;
                    if (a.out_bf16) {
                        bf16x4 ob;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ob[e] = (__bf16)o[e];
                        *(bf16x4 *)((__bf16 *)a.O + off + d) = ob;
                    } else {
                        *(f32x4 *)((float *)a.O + off + d) = o;
                    }
                }
            if (a.lse && h == 0) a.lse[(int64_t)bh * a.W + row] = m[r] * a.scale + logf(lt);
        } else {
            const int64_t slot = (int64_t)bh * a.nparts + a.part0 + split;
            float *op = a.Opart + (slot * a.W + row) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = oacc[r][db][4 * g + e];
                    *(f32x4 *)(op + 32 * db + 8 * g + 4 * h) = o;
                }
            if (h == 0) {
                a.Mpart[slot * a.W + row] = m[r] * a.c;
                a.Lpart[slot * a.W + row] = lt;
            }
        }
    }
}

}  // namespace tlin
