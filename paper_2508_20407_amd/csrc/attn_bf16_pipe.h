// bf16 attention over one unmasked key partition, software-pipelined inside the wave.
//
// Same computation, operand mapping, LDS layout and partial format as attn_bf16_body (see
// attn_bf16.h: transposed scores S^T = K Q^T on v_mfma_f32_32x32x16_bf16, weights already in
// B-operand order for O^T += V^T P^T, direct HBM -> LDS tile loads with the swizzle on the source
// side), for the unmasked history partitions of Section 3's attention with one 32-row query block
// per wave.  What differs is the order of the work inside a wave.  attn_bf16_body runs the three
// stages of a tile one after another (score products, softmax arithmetic, value products), so the
// matrix pipe idles during the softmax arithmetic and the vector pipe during the products.  Here a
// wave keeps TWO score accumulators and works on two tiles at once:
//
//     step n:   A   S(n+1)  = K(n+1) Q^T              16 matrix instructions
//                   P(n)[keys 0..31]  = 2^(c S(n) - c m), rounded to bf16, row sum       vector
//               B1  O += V(n)[keys 0..31]^T P(n)       8 matrix instructions
//                   P(n)[keys 32..63] likewise                                           vector
//               B2  O += V(n)[keys 32..63]^T P(n)      8 matrix instructions
//                   row maximum of S(n+1), reference point test                          vector
//               (rare) the reference point m moves: O and l are rescaled
//
// In every phase the matrix instructions and the vector instructions are independent of each
// other, and they are issued interleaved (one matrix instruction, its operand's LDS read a few
// slots ahead, a few vector instructions), so both pipes of the SIMD are busy at the same time
// within one wave, and the second wave of the SIMD fills what is left.  The weights of tile n are
// taken against the reference point that was fixed at the end of step n-1, which is the same
// point the classic order uses.
//
// The row sum l is accumulated from the fp32 weights with plain adds, not with v_dot2_f32_bf16 on
// the rounded ones as attn_bf16_body does: under a stream of matrix instructions a dot2 costs about
// 6 cycles of the matrix pipe (it does not execute beside it), an add costs nothing (measured on a
// single-wave stream: 42 against 34 cycles per matrix instruction with this softmax work in
// between).  The normaliser is then the exact sum of the weights while the value product uses their
// bf16 roundings, so a row is a convex combination only to within 2^-9 per weight; the difference
// stays far inside the tolerance and the log-sum-exp output becomes exact to fp32 rounding.
//
// Ring of two tiles for K and two for V; K runs one tile ahead of V.  Step n reads K(n+1) and
// V(n); at its top (after the step's single barrier) every wave has finished K(n) and V(n-1),
// whose stages take the loads of K(n+2) and V(n+1).  With two stages and the loop unrolled by
// two, every LDS address of the loop is a loop-invariant register plus an immediate.
#pragma once
#include <type_traits>
#include <utility>

#include "attn_bf16.h"

namespace tlin {

// sched_group_barrier masks
constexpr int SG_VALU = 0x002, SG_MFMA = 0x008, SG_DSR = 0x100, SG_TRANS = 0x400;

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant
// expression in the body (the scheduling builtins take literal arguments only)
template <typename F, int... I>
__device__ __forceinline__ void static_for_seq(F &&f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f) { static_for_seq(f, std::make_integer_sequence<int, N>{}); }

// CAUSAL: the window's causal attention (query i sees keys j <= i; Section 3, Causal attention).  A
// workgroup walks the key tiles up to its last row; a wave leaves the pipeline after the tile that
// holds its own rows' diagonal (later tiles lie after every row it owns) and from then on only meets
// the barriers and issues its share of the tile loads.
template <int D, int NW, bool PAD, bool NT, bool CAUSAL = false>
__device__ __forceinline__ void attn_bf16_pipe_body(const AttnArgs &a, int bid, int nblocks)
{
    constexpr int NSTAGE = 2;
    constexpr int BN = 64;                 // keys per tile
    constexpr int BM = NW * 32;            // query rows per workgroup
    constexpr int ROWB = D * 2;            // bytes per K/V row
    constexpr int TILE_B = BN * ROWB;
    constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;       // rows moved by one wave-wide direct load
    constexpr int NDMA = BN / RPI / NW;    // direct loads per wave per tensor per tile
    static_assert(BN % (RPI * NW) == 0 && NDMA >= 1, "tile does not divide over the waves");
    constexpr int DS = D / 16;             // contraction steps of Q K^T
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    static_assert((2 * NSTAGE - 1) * TILE_B + 56 * ROWB + 256 <= 65536, "LDS offsets must fit the 16-bit immediate");

    char *const Ks = tlin_smem;
    char *const Vs = tlin_smem + NSTAGE * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;

    const int L = xcd_remap(bid, nblocks);
    const Problem pr = decode_problem<BM, BN, CAUSAL>(a, L, a.nqb);
    if (pr.skip) return;                               // uniform over the workgroup
    const int qb = pr.qb, split = pr.split, bh = pr.bh;
    const int b = bh / a.H, hd = bh % a.H;
    const int Wq = pr.W, NK = pr.NK;

    int t0 = 0, t1 = (min(NK, qb * BM + BM) + BN - 1) / BN;
    if (!CAUSAL) partition_tiles<BM, BN, 5>(a, pr, t0, t1);
    const int nt = t1 - t0;                            // tiles of this partition (may be <= 0 in the sliding schedule)

    const int64_t k_rb = a.k_sr * 2, v_rb = a.v_sr * 2;
    const __bf16 *Qg = (const __bf16 *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh + pr.qrow_off * a.q_sr;
    const char *Kg = (const char *)((const __bf16 *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh) + pr.krow_off * k_rb;
    const char *Vg = (const char *)((const __bf16 *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh) + pr.krow_off * v_rb;

    // head dimension of the tensors below the kernel's D: see attn_bf16_body
    const int dchunks = PAD ? (a.D + 7) >> 3 : D / 8;
    const int straddle = (PAD && (a.D & 7)) ? (a.D >> 4) : -1;
    auto clip = [&](bf16x8 f) __attribute__((always_inline)) {
        const int keep = a.D - (16 * straddle + 8 * h);
        u32x4 u = __builtin_bit_cast(u32x4, f);
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] &= keep >= 2 * e + 2 ? ~0u : keep == 2 * e + 1 ? 0x0000ffffu : 0u;
        return __builtin_bit_cast(bf16x8, u);
    };

    const int qrow0 = qb * BM + wave * 32;
    // the last tile this wave computes on (uniform over the wave): causal, the tile of its rows' diagonal
    const int tl = CAUSAL ? min((qrow0 + 31) / BN, nt - 1) : nt - 1;
    bf16x8 qf[DS];     // Q^T fragments (B operand): lane holds query j, contraction elements 16*s + 8*h .. +7
    {
        const int r = min(qrow0 + j, Wq - 1);
        const __bf16 *qp = Qg + (int64_t)r * a.q_sr + 8 * h;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            if (PAD && 16 * s + 8 * h >= a.D) { qf[s] = bf16x8{}; continue; }
            const bf16x8 f = *(const bf16x8 *)(qp + 16 * s);
            qf[s] = (PAD && s == straddle) ? clip(f) : f;
        }
        // consume the Q registers here, so that the wait for these loads sits before the tile loop
#pragma unroll
        for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(qf[s]));
    }

    // direct loads of this wave: see attn_bf16_body
    unsigned koff[NDMA], voff[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        const int drow = (wave * NDMA + i) * RPI + lane / CPR;
        const int kc = (lane % CPR) ^ Swz<D>::k(drow), vc = (lane % CPR) ^ Swz<D>::v(drow);
        koff[i] = (PAD && kc >= dchunks) ? kNoChunk : (unsigned)(drow * k_rb) + (kc << 4);
        voff[i] = (PAD && vc >= dchunks) ? kNoChunk : (unsigned)(drow * v_rb) + (vc << 4);
    }
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_offset(Ks) + wave * (NDMA * 1024));
    // local tile index n (tile t0 + n) into ring stage `stage`
    auto issue_k = [&](int n, int stage) __attribute__((always_inline)) {
        const int key0 = (t0 + n) * BN;
        const int rows = min(BN, NK - key0);
        const u32x4 kd = tile_descriptor(Kg + key0 * k_rb, (PAD || rows < BN) ? (unsigned)(rows * k_rb) : 0xffffffffu);
#pragma unroll
        for (int i = 0; i < NDMA; ++i) direct_load_1k<NT>(kd, koff[i], lds_wave + stage * TILE_B + i * 1024);
    };
    auto issue_v = [&](int n, int stage) __attribute__((always_inline)) {
        const int key0 = (t0 + n) * BN;
        const int rows = min(BN, NK - key0);
        const u32x4 vd = tile_descriptor(Vg + key0 * v_rb, (PAD || rows < BN) ? (unsigned)(rows * v_rb) : 0xffffffffu);
#pragma unroll
        for (int i = 0; i < NDMA; ++i) direct_load_1k<NT>(vd, voff[i], lds_wave + (NSTAGE + stage) * TILE_B + i * 1024);
    };
    auto scrub = [&](int stage) __attribute__((always_inline)) {
        if (!PAD || !(a.D & 7)) return;
        if (lane < NDMA * RPI) {
            const int r = (wave * NDMA + lane / RPI) * RPI + lane % RPI;
            const int pos = (a.D >> 3) ^ Swz<D>::k(r);
            *(u32x2 *)(Ks + stage * TILE_B + r * ROWB + (pos << 4) + 8) = u32x2{0u, 0u};
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };

    // Loop-invariant LDS addresses (stage and row-block offsets are immediates at the use).
    //   K fragment of contraction step s, keys j and j + 32: row j, chunk (2 s + h) ^ swz
    //   V operand of column block db: rows 4 h + i16 / 4 (+ 8, 16, ...), columns 64 db + 32 blk1 + 8 (i16 & 3)
    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
    unsigned kaddr[DS], vaddr[DB];
#pragma unroll
    for (int s = 0; s < DS; ++s) kaddr[s] = lds_offset(Ks) + j * ROWB + (((2 * s + h) ^ Swz<D>::k(j)) << 4);
    {
        const int r0 = 4 * h + (i16 >> 2);
        const int sw = Swz<D>::v(r0) << 4;           // the same for rows r0 + 8 k
#pragma unroll
        for (int db = 0; db < DB; ++db) vaddr[db] = lds_offset(Vs) + r0 * ROWB + ((64 * db + 32 * blk1 + 8 * (i16 & 3)) ^ sw);
    }

    f32x16 oacc[DB];
    float m = -INFINITY, l = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    const float thr = 8.0f / a.c;          // reference point moves only beyond 2^8 (see attn_bf16_body)
    float mc = 0.f;                        // m * c of the current reference point
    bf16x8 pb[2][2];                       // weights of the current tile, B-operand order

    typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;

    // ---- pieces of a step.  S[kb][v]: keys kb*32 + 8*(v/4) + 4*h + v%4 of query j.
    auto qk_zero = [&](f32x16 (&S)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int v = 0; v < 16; ++v) S[kk][v] = 0.f;
    };
    auto qk_step = [&](f32x16 (&S)[2], int s, int kk, int kstage) __attribute__((always_inline)) {
        const bf16x8 kf = *(lds_bf16x8 *)(uintptr_t)(kaddr[s] + kstage * TILE_B + kk * (32 * ROWB));
        S[kk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], S[kk], 0, 0, 0);
    };
    // weights of the 16 keys of quarter (kb, t2) from S (against mc), rounded to bf16 for the value
    // product; their fp32 values are summed into l
    auto weights_q = [&](const f32x16 (&S)[2], int kb, int t2) __attribute__((always_inline)) {
        float ls = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(fmaf(S[kb][8 * t2 + e], a.c, -mc));
            const float p1 = fast_exp2(fmaf(S[kb][8 * t2 + e + 1], a.c, -mc));
            pb[kb][t2][e] = (__bf16)p0;
            pb[kb][t2][e + 1] = (__bf16)p1;
            ls += p0 + p1;
        }
        l += ls;
    };
    auto weights = [&](const f32x16 (&S)[2], int kb) __attribute__((always_inline)) {
        weights_q(S, kb, 0);
        weights_q(S, kb, 1);
    };
    // O^T += V^T P^T for the 32 keys of block kb
    auto pv_half = [&](int kb, int vstage) __attribute__((always_inline)) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const unsigned ad = vaddr[db] + vstage * TILE_B + (kb * 32 + 16 * t2) * ROWB;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)ad);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)(ad + 8 * ROWB));
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kb][t2], oacc[db], 0, 0, 0);
            }
    };
    // keys past the end of the tensor and (causal) keys after the query row
    auto mask_ragged = [&](f32x16 (&S)[2], int key0) __attribute__((always_inline)) {
        const int lim = CAUSAL ? min(qrow0 + j, NK - 1) : NK - 1;     // last visible key
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (key > lim) S[kb][v] = -INFINITY;
            }
        asm volatile("" ::: "memory");     // stays a branch around these selects (taken once per partition at most)
    };
    // does local tile nn need the mask: ragged end of the tensor, or the wave's diagonal tile
    auto needs_mask = [&](int nn) __attribute__((always_inline)) { return (t0 + nn + 1) * BN > NK || (CAUSAL && nn == tl); };
    auto row_max = [&](const f32x16 (&S)[2]) __attribute__((always_inline)) {
        float mx = S[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, S[kb][v]);
        return xhalf_max(mx);
    };
    // the reference point moves to mx where some row's maximum exceeds it by more than the threshold
    auto move_reference = [&](float mx) __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(mx > m + thr) != 0) {
            const float mn = fmaxf(m, mx);
            const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2((m - mn) * a.c);
            l *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
            m = mn;
            mc = (m == -INFINITY) ? 0.f : m * a.c;
        }
    };

    // Tile loads of step n, one wave instruction at a time: K(n+2) into the stage of K(n), then
    // V(n+1) into the stage of V(n-1); both stages were released by the step's barrier.  Beyond the
    // partition's end the last tile is fetched again into the free stage (nobody reads it), which
    // keeps the instruction stream and the load counter free of branches.
    auto dma = [&](int i, int n, int kfree, int vfree) __attribute__((always_inline)) {
        const bool isk = i < NDMA;
        const int tile = t0 + min(isk ? n + 2 : n + 1, nt - 1);
        const int key0 = tile * BN;
        const int rows = min(BN, NK - key0);
        const int64_t rb = isk ? k_rb : v_rb;
        const u32x4 d = tile_descriptor((isk ? Kg : Vg) + key0 * rb, (PAD || rows < BN) ? (unsigned)(rows * rb) : 0xffffffffu);
        const int ii = isk ? i : i - NDMA;
        direct_load_1k<NT>(d, isk ? koff[ii] : voff[ii], lds_wave + ((isk ? kfree : NSTAGE + vfree)) * TILE_B + ii * 1024);
    };
    // Schedule parameters (measured on the largest fixed workload; neighbouring values are within 1 %).
    constexpr int PIPE_KPF = 4;       // K fragments requested ahead of their product
    constexpr int PIPE_VPF = 2;       // V operands (two reads each) requested ahead of their product
    constexpr int PIPE_WA = 2;        // quarters of the tile's weights computed in phase A (the rest in phase B)
    constexpr bool PIPE_PACED = true; // tile loads spread over phase A instead of a burst behind the barrier
    constexpr int VPQ = 29;           // vector instructions per quarter of a tile's weights: 8 fma, 8 exp2, 4 convert, 9 add

    // value product number i of a tile (i = 8 kb + 4 t2 + db): its V operand, and the product
    auto v_read = [&](int i, int vstage) __attribute__((always_inline)) {
        const int kb = i / (2 * DB), t2 = (i / DB) % 2, db = i % DB;
        const unsigned ad = vaddr[db] + vstage * TILE_B + (kb * 32 + 16 * t2) * ROWB;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)ad);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)(ad + 8 * ROWB));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto pv_op = [&](int i, bf16x8 vf) __attribute__((always_inline)) {
        const int kb = i / (2 * DB), t2 = (i / DB) % 2, db = i % DB;
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kb][t2], oacc[db], 0, 0, 0);
    };

    // One step with compile-time ring stages: reads K(n+1) from stage KST, V(n) from stage VST.
    auto step = [&](const f32x16 (&Sc)[2], f32x16 (&Sn)[2], int n, auto kst, auto vst) __attribute__((always_inline)) {
        constexpr int KST = decltype(kst)::value, VST = decltype(vst)::value;
        wait_vmcnt<0>();
        scrub(KST);
        __builtin_amdgcn_s_barrier();
        if (!PIPE_PACED || (CAUSAL && n + 1 > tl)) {
#pragma unroll
            for (int i = 0; i < 2 * NDMA; ++i) dma(i, n, VST, KST);
        }
        if (CAUSAL && n + 1 > tl) {
            // this wave has no further tile to score: tile n is its last one (weights and value
            // products, unpipelined) or already behind it
            if (n == tl) {
                weights(Sc, 0);
                pv_half(0, VST);
                weights(Sc, 1);
                pv_half(1, VST);
            }
            return;
        }
        // phase A
        qk_zero(Sn);
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            // the step's 2 * NDMA load instructions, spread evenly over the contraction steps
            if (PIPE_PACED) {
#pragma unroll
                for (int i = (s * 2 * NDMA) / DS; i < ((s + 1) * 2 * NDMA) / DS; ++i) dma(i, n, VST, KST);
            }
            qk_step(Sn, s, 0, KST);
            qk_step(Sn, s, 1, KST);
        }
#pragma unroll
        for (int q = 0; q < PIPE_WA; ++q) weights_q(Sc, q >> 1, q & 1);
        // the weights belong to this phase: without a use here they would sink behind the branch below
#pragma unroll
        for (int q = 0; q < PIPE_WA; ++q) asm volatile("" : "+v"(pb[q >> 1][q & 1]));
        asm volatile("" : "+v"(l));
        // (tried and within noise: the first value operands of phase B requested at the end of this
        // phase; some of the vector instructions ahead of the first product)
#pragma unroll
        for (int i = 0; i < PIPE_KPF; ++i) __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 0);
        static_for<2 * DS>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
            if (i + PIPE_KPF < 2 * DS) __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 0);
            // the phase's vector instructions, spread evenly over the products
            constexpr int nv = (VPQ * PIPE_WA * (i + 1)) / (2 * DS) - (VPQ * PIPE_WA * i) / (2 * DS);
            if (nv > 0) __builtin_amdgcn_sched_group_barrier(SG_VALU | SG_TRANS, nv, 0);
        });
        __builtin_amdgcn_sched_barrier(0);
        if (needs_mask(n + 1)) mask_ragged(Sn, (t0 + n + 1) * BN);
        // phase B
#pragma unroll
        for (int i = 0; i < 2 * DB; ++i) pv_op(i, v_read(i, VST));
#pragma unroll
        for (int q = PIPE_WA; q < 4; ++q) weights_q(Sc, q >> 1, q & 1);
#pragma unroll
        for (int i = 2 * DB; i < 4 * DB; ++i) pv_op(i, v_read(i, VST));
        const float mx = row_max(Sn);
#pragma unroll
        for (int i = 0; i < 2 * PIPE_VPF; ++i) __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 1);
        static_for<4 * DB>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 1);
            if (i + PIPE_VPF < 4 * DB) __builtin_amdgcn_sched_group_barrier(SG_DSR, 2, 1);
            // the remaining quarters' weights during the first half's products, the row maximum after them
            constexpr int nv = i < 2 * DB ? (VPQ * (4 - PIPE_WA) * (i + 1)) / (2 * DB) - (VPQ * (4 - PIPE_WA) * i) / (2 * DB) : 3;
            if (nv > 0) __builtin_amdgcn_sched_group_barrier(SG_VALU | SG_TRANS, nv, 1);
        });
        __builtin_amdgcn_sched_barrier(0);
        move_reference(mx);
    };

    using st0 = std::integral_constant<int, 0>;
    using st1 = std::integral_constant<int, 1>;

    if (nt > 0) {
        f32x16 S0[2], S1[2];
        // prologue: K(0), then K(1) and V(0); scores and reference point of tile 0
        issue_k(0, 0);
        if (nt > 1) issue_k(1, 1);
        issue_v(0, 0);
        if (nt > 1) wait_vmcnt<3 * NDMA - NDMA>();     // K(0) has landed; K(1), V(0) may still fly
        else wait_vmcnt<NDMA>();
        scrub(0);
        __builtin_amdgcn_s_barrier();
        qk_zero(S0);
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            qk_step(S0, s, 0, 0);
            qk_step(S0, s, 1, 0);
        }
        if (needs_mask(0)) mask_ragged(S0, t0 * BN);
        move_reference(row_max(S0));

        // step n reads K(n+1) from stage (n+1) % 2 and V(n) from stage n % 2
        int n = 0;
        for (; n + 2 < nt; n += 2) {
            step(S0, S1, n, st1{}, st0{});
            step(S1, S0, n + 1, st0{}, st1{});
        }
        if (n + 1 < nt) {
            step(S0, S1, n, st1{}, st0{});
            ++n;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) S0[kk] = S1[kk];
        }
        // last tile (n = nt - 1, in S0): weights and value products only
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (CAUSAL && tl < nt - 1) {
            // this wave finished with an earlier tile
        } else if (n & 1) {
            weights(S0, 0);
            pv_half(0, 1);
            weights(S0, 1);
            pv_half(1, 1);
        } else {
            weights(S0, 0);
            pv_half(0, 0);
            weights(S0, 1);
            pv_half(1, 0);
        }
    }

    // ---- epilogue.  Accumulator register v of block db is d = 32*db + 8*(v/4) + 4*h + v%4.
    const float lt = xhalf_sum(l);
    const int row = qrow0 + j;
    if (row >= Wq) return;
    if (a.direct) {
        const float inv = 1.0f / lt;
        const int64_t off = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh + (pr.qrow_off + row) * a.o_sr;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * h;
                if (PAD && d >= a.D) continue;
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
        const int64_t slot = pr.slot + a.part0 + (CAUSAL ? 0 : split);
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

// The same in-wave pipeline for the shape whose QUERY side is the long one (Section 3, last layer of
// the context path: every history row queries the few compressed rows): all T1 key tiles stay in
// LDS for the lifetime of the workgroup, which walks over query blocks qb, qb + q_groups, ... without
// any barrier, each block running the pipeline over the resident tiles (T1 is even, so the two score
// accumulators keep their roles from block to block).  Direct output only (one partition).
template <int D, int NW, bool PAD, int T1, int TMAX>
__device__ __forceinline__ void attn_bf16_resident_pipe_body(const AttnArgs &a, int bid, int nblocks)
{
    static_assert(T1 % 2 == 0 && T1 >= 2 && T1 <= TMAX, "an even number of resident key tiles");
    constexpr int BN = 64, BM = NW * 32, ROWB = D * 2, TILE_B = BN * ROWB, CPR = ROWB / 16, RPI = 1024 / ROWB;
    constexpr int NDMA = BN / RPI / NW, DS = D / 16, DB = D / 32;
    static_assert(BN % (RPI * NW) == 0 && NDMA >= 1, "tile does not divide over the waves");
    static_assert((TMAX - 1) * TILE_B + 56 * ROWB + 256 <= 65536, "LDS offsets must fit the 16-bit immediate");

    char *const Ks = tlin_smem;
    char *const Vs = tlin_smem + TMAX * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;

    const int L = xcd_remap(bid, nblocks);
    const int qstep = a.q_groups;
    const Problem pr = decode_problem<BM, BN, false>(a, L, qstep);
    if (pr.skip) return;
    int qb = pr.qb;
    const int bh = pr.bh, b = bh / a.H, hd = bh % a.H;
    const int Wq = pr.W, NK = pr.NK;
    const bool ragged = NK < T1 * BN;

    const int64_t k_rb = a.k_sr * 2, v_rb = a.v_sr * 2;
    const __bf16 *Qg = (const __bf16 *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh;
    const char *Kg = (const char *)((const __bf16 *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh);
    const char *Vg = (const char *)((const __bf16 *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh);

    const int dchunks = PAD ? (a.D + 7) >> 3 : D / 8;
    const int straddle = (PAD && (a.D & 7)) ? (a.D >> 4) : -1;
    auto clip = [&](bf16x8 f) __attribute__((always_inline)) {
        const int keep = a.D - (16 * straddle + 8 * h);
        u32x4 u = __builtin_bit_cast(u32x4, f);
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] &= keep >= 2 * e + 2 ? ~0u : keep == 2 * e + 1 ? 0x0000ffffu : 0u;
        return __builtin_bit_cast(bf16x8, u);
    };
    // Q^T fragments of the 32 rows this wave owns in query block `blk`
    auto load_q = [&](bf16x8 (&q)[DS], int blk) __attribute__((always_inline)) {
        const int r = min(blk * BM + wave * 32 + j, Wq - 1);
        const __bf16 *qp = Qg + (int64_t)r * a.q_sr + 8 * h;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            if (PAD && 16 * s + 8 * h >= a.D) { q[s] = bf16x8{}; continue; }
            const bf16x8 f = *(const bf16x8 *)(qp + 16 * s);
            q[s] = (PAD && s == straddle) ? clip(f) : f;
        }
    };

    // ---- the whole key/value side into LDS, once: tile t lives in stage t
    {
        const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_offset(Ks) + wave * (NDMA * 1024));
#pragma unroll
        for (int t = 0; t < T1; ++t) {
            const int key0 = t * BN;
            const int rows = min(BN, NK - key0);
            const u32x4 kd = tile_descriptor(Kg + key0 * k_rb, (PAD || rows < BN) ? (unsigned)(rows * k_rb) : 0xffffffffu);
            const u32x4 vd = tile_descriptor(Vg + key0 * v_rb, (PAD || rows < BN) ? (unsigned)(rows * v_rb) : 0xffffffffu);
#pragma unroll
            for (int i = 0; i < NDMA; ++i) {
                const int drow = (wave * NDMA + i) * RPI + lane / CPR;
                const int kc = (lane % CPR) ^ Swz<D>::k(drow), vc = (lane % CPR) ^ Swz<D>::v(drow);
                direct_load_1k(kd, (PAD && kc >= dchunks) ? kNoChunk : (unsigned)(drow * k_rb) + (kc << 4), lds_wave + t * TILE_B + i * 1024);
                direct_load_1k(vd, (PAD && vc >= dchunks) ? kNoChunk : (unsigned)(drow * v_rb) + (vc << 4), lds_wave + (TMAX + t) * TILE_B + i * 1024);
            }
        }
    }
    bf16x8 qf[DS];
    load_q(qf, qb);
    wait_vmcnt<0>();
    if (PAD && (a.D & 7)) {
        // the part from a.D on of the K chunk that straddles a.D is cleared by the wave that loaded the row
        if (lane < NDMA * RPI) {
            const int r = (wave * NDMA + lane / RPI) * RPI + lane % RPI;
            const int pos = (a.D >> 3) ^ Swz<D>::k(r);
#pragma unroll
            for (int t = 0; t < T1; ++t) *(u32x2 *)(Ks + t * TILE_B + r * ROWB + (pos << 4) + 8) = u32x2{0u, 0u};
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();

    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
    unsigned kaddr[DS], vaddr[DB];
#pragma unroll
    for (int s = 0; s < DS; ++s) kaddr[s] = lds_offset(Ks) + j * ROWB + (((2 * s + h) ^ Swz<D>::k(j)) << 4);
    {
        const int r0 = 4 * h + (i16 >> 2);
        const int sw = Swz<D>::v(r0) << 4;
#pragma unroll
        for (int db = 0; db < DB; ++db) vaddr[db] = lds_offset(Vs) + r0 * ROWB + ((64 * db + 32 * blk1 + 8 * (i16 & 3)) ^ sw);
    }

    f32x16 oacc[DB];
    float m = -INFINITY, l = 0.f, mc = 0.f;
    auto reset = [&]() __attribute__((always_inline)) {
        l = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    };
    reset();
    const float thr = 8.0f / a.c;
    bf16x8 pb[2][2];
    typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;

    // ---- pieces of a step (as in attn_bf16_pipe_body)
    auto qk_zero = [&](f32x16 (&S)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int v = 0; v < 16; ++v) S[kk][v] = 0.f;
    };
    auto qk_tile = [&](f32x16 (&S)[2], const bf16x8 (&q)[DS], int tile) __attribute__((always_inline)) {
        qk_zero(S);
#pragma unroll
        for (int s = 0; s < DS; ++s)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const bf16x8 kf = *(lds_bf16x8 *)(uintptr_t)(kaddr[s] + tile * TILE_B + kk * (32 * ROWB));
                S[kk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, q[s], S[kk], 0, 0, 0);
            }
    };
    auto weights_q = [&](const f32x16 (&S)[2], int kb, int t2) __attribute__((always_inline)) {
        float ls = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(fmaf(S[kb][8 * t2 + e], a.c, -mc));
            const float p1 = fast_exp2(fmaf(S[kb][8 * t2 + e + 1], a.c, -mc));
            pb[kb][t2][e] = (__bf16)p0;
            pb[kb][t2][e + 1] = (__bf16)p1;
            ls += p0 + p1;
        }
        l += ls;
    };
    auto pv_half = [&](int kb, int tile) __attribute__((always_inline)) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const unsigned ad = vaddr[db] + tile * TILE_B + (kb * 32 + 16 * t2) * ROWB;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)ad);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)(ad + 8 * ROWB));
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kb][t2], oacc[db], 0, 0, 0);
            }
    };
    auto mask_ragged = [&](f32x16 (&S)[2], int key0) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (key >= NK) S[kb][v] = -INFINITY;
            }
        asm volatile("" ::: "memory");
    };
    auto row_max = [&](const f32x16 (&S)[2]) __attribute__((always_inline)) {
        float mx = S[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, S[kb][v]);
        return xhalf_max(mx);
    };
    auto move_reference = [&](float mx) __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(mx > m + thr) != 0) {
            const float mn = fmaxf(m, mx);
            const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2((m - mn) * a.c);
            l *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
            m = mn;
            mc = (m == -INFINITY) ? 0.f : m * a.c;
        }
    };
    // normalise and store the block's rows
    // bf16 output goes through a wave-private 4 KB staging area behind the resident tiles: a lane owns
    // one row and would store it as sixteen 8-byte pieces, each instruction touching 32 rows; turned
    // through LDS (half a row at a time, 16-byte chunk ^ (row / 2 & 7) keeps writes and reads off each
    // other's banks) a store instruction writes eight rows' 128-byte halves whole.
    constexpr bool STAGED = !PAD && (2 * TMAX * TILE_B + NW * 4096 <= 160 * 1024) && D == 128;
    char *const stg = tlin_smem + 2 * TMAX * TILE_B + wave * 4096;
    auto finish_block = [&](int blk) __attribute__((always_inline)) {
        const float lt = xhalf_sum(l);
        const int row0 = blk * BM + wave * 32;
        const int row = row0 + j;
        const float inv = 1.0f / lt;
        if (STAGED && a.out_bf16) {
            const int64_t obase = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh;
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
                for (int dd = 0; dd < 2; ++dd)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int db = 2 * hf + dd;
                        bf16x4 ob;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ob[e] = (__bf16)(oacc[db][4 * g + e] * inv);
                        const int ch = 4 * dd + g;       // 16-byte chunk of the 128-byte half row; this lane holds its half h
                        *(bf16x4 *)(stg + j * 128 + ((ch ^ ((j >> 1) & 7)) << 4) + 8 * h) = ob;
                    }
                // the wave reads what its own lanes wrote: LDS operations of a wave complete in order
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int r = (lane >> 3) + 8 * k, cc = lane & 7;
                    const u32x4 piece = *(const u32x4 *)(stg + r * 128 + ((cc ^ ((r >> 1) & 7)) << 4));
                    if (row0 + r < Wq) *(u32x4 *)((__bf16 *)a.O + obase + (int64_t)(row0 + r) * a.o_sr + 64 * hf + 8 * cc) = piece;
                }
            }
            if (row < Wq && a.lse && h == 0) a.lse[(int64_t)bh * a.W + row] = m * a.scale + logf(lt);
            return;
        }
        if (row < Wq) {
            const int64_t off = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh + (int64_t)row * a.o_sr;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = 32 * db + 8 * g + 4 * h;
                    if (PAD && d >= a.D) continue;
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
        }
    };

    constexpr int KPF = 4, VPF = 2;
    constexpr int VPQ = 29;
    // phase A: scores of key tile KT with the queries q into Sn, weights of the first two quarters of Sc
    auto phase_a = [&](const f32x16 (&Sc)[2], f32x16 (&Sn)[2], const bf16x8 (&q)[DS], auto kt) __attribute__((always_inline)) {
        constexpr int KT = decltype(kt)::value;
        qk_tile(Sn, q, KT);
        weights_q(Sc, 0, 0);
        weights_q(Sc, 0, 1);
        asm volatile("" : "+v"(pb[0][0]), "+v"(pb[0][1]), "+v"(l));
#pragma unroll
        for (int i = 0; i < KPF; ++i) __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 0);
        static_for<2 * DS>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
            if (i + KPF < 2 * DS) __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 0);
            constexpr int nv = (2 * VPQ * (i + 1)) / (2 * DS) - (2 * VPQ * i) / (2 * DS);
            if (nv > 0) __builtin_amdgcn_sched_group_barrier(SG_VALU | SG_TRANS, nv, 0);
        });
        __builtin_amdgcn_sched_barrier(0);
        if (KT == T1 - 1 && ragged) mask_ragged(Sn, KT * BN);
    };
    // phase B: value products of tile VT with the weights of Sc (second half computed here), row maximum of Sn
    auto phase_b = [&](const f32x16 (&Sc)[2], const f32x16 (&Sn)[2], auto vt) __attribute__((always_inline)) {
        constexpr int VT = decltype(vt)::value;
        pv_half(0, VT);
        weights_q(Sc, 1, 0);
        weights_q(Sc, 1, 1);
        pv_half(1, VT);
        const float mx = row_max(Sn);
#pragma unroll
        for (int i = 0; i < 2 * VPF; ++i) __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 1);
        static_for<4 * DB>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 1);
            if (i + VPF < 4 * DB) __builtin_amdgcn_sched_group_barrier(SG_DSR, 2, 1);
            constexpr int nv = i < 2 * DB ? (2 * VPQ * (i + 1)) / (2 * DB) - (2 * VPQ * i) / (2 * DB) : 3;
            if (nv > 0) __builtin_amdgcn_sched_group_barrier(SG_VALU | SG_TRANS, nv, 1);
        });
        __builtin_amdgcn_sched_barrier(0);
        return mx;
    };

    // ---- per query block: scores of tile 0, T1 - 1 pipelined steps, the last tile's weights and
    // value products, normalise and store.  The next block's queries are requested into the same
    // registers right behind their last use (the score products of the last key tile), and have the
    // rest of the block to arrive; the other wave of the SIMD, which is at another point of its own
    // block (there are no barriers here), fills the unpipelined head and tail of this one.
    f32x16 S0[2], S1[2];
    while (true) {
        qk_tile(S0, qf, 0);
        if (T1 == 1 && ragged) mask_ragged(S0, 0);
        m = row_max(S0);
        mc = (m == -INFINITY) ? 0.f : m * a.c;
        const bool has_next = qb + qstep < a.nqb;      // uniform over the workgroup
        static_for<T1 - 1>([&](auto nc) __attribute__((always_inline)) {
            constexpr int n = decltype(nc)::value;
            if constexpr (n % 2 == 0) phase_a(S0, S1, qf, std::integral_constant<int, n + 1>{});
            else phase_a(S1, S0, qf, std::integral_constant<int, n + 1>{});
            if (n == T1 - 2 && has_next) load_q(qf, qb + qstep);
            if constexpr (n % 2 == 0) move_reference(phase_b(S0, S1, nc));
            else move_reference(phase_b(S1, S0, nc));
        });
        // last tile (scores in S1, T1 being even)
        weights_q(S1, 0, 0);
        weights_q(S1, 0, 1);
        pv_half(0, T1 - 1);
        weights_q(S1, 1, 0);
        weights_q(S1, 1, 1);
        pv_half(1, T1 - 1);
        finish_block(qb);
        if (!has_next) break;
        reset();
        qb += qstep;
    }
}

}  // namespace tlin
