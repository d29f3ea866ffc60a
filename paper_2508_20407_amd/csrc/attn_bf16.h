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
//   * K/V tiles of 64 keys go HBM -> LDS directly (buffer_load_dwordx4 ... lds: each wave
//     instruction moves 1 KB, lane i landing at base + 16*i) through a ring of NSTAGE tiles,
//     the loads of the following tiles being in flight during compute.  One barrier per tile;
//     completion is tracked by hand with s_waitcnt vmcnt.  (A compute unit keeps only some
//     16-32 KB of such loads in flight; a wave that issues into a full queue waits there, so
//     the ring depth beyond two tiles buys little.)
//   * LDS rows are XOR-swizzled at 16-byte-chunk granularity so that the ds_read_b128 of the
//     K operand and the transposed reads of V are bank-conflict free on the 64-bank LDS.  The
//     direct loads write LDS linearly, so the swizzle is applied on the source side: the lane
//     that lands on chunk position c of row r fetches chunk c ^ swz(r) of that row.
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
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// RESIDENT: the whole key/value partition (at most NSTAGE tiles) is loaded into LDS once and the
// workgroup then walks over query blocks qb, qb + q_groups, ... without any further barrier, so
// its waves drift apart and one wave's matrix work overlaps another's softmax arithmetic.  Used
// where the query side is the long one.

// The work of one workgroup; `bid` of `nblocks` is its index among the blocks of this problem set.
// PAD: the tensors' head dimension a.D is smaller than the kernel's D.
// REMAP: bid is a hardware block index (mapped to a logical one here); otherwise it is the logical index.
template <int D, int NW, int QB, bool CAUSAL, int NSTAGE, bool RESIDENT = false, bool PAD = false, bool REMAP = true>
__device__ __forceinline__ void attn_bf16_body(const AttnArgs &a, int bid, int nblocks)
{
    static_assert(!(RESIDENT && CAUSAL), "the resident variant is for unmasked attention");
    constexpr int BN = 64;                 // keys per tile
    constexpr int BM = NW * QB * 32;       // query rows per workgroup
    constexpr int ROWB = D * 2;            // bytes per K/V row
    constexpr int TILE_B = BN * ROWB;
    constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;       // rows moved by one wave-wide direct load
    constexpr int NDMA = BN / RPI / NW;    // direct loads per wave per tensor per tile
    static_assert(BN % (RPI * NW) == 0 && NDMA >= 1, "tile does not divide over the waves");
    constexpr int DS = D / 16;             // contraction steps of Q K^T
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    constexpr int PD = NSTAGE - 1;         // prefetch distance in tiles
    static_assert(PD >= 1, "ring too shallow");
    static_assert(PD * 2 * NDMA < 64, "too many loads in flight for vmcnt");

    char *const Ks = tlin_smem;
    char *const Vs = tlin_smem + NSTAGE * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;

    const int L = REMAP ? xcd_remap(bid, nblocks) : bid;
    const int qstep = RESIDENT ? a.q_groups : a.nqb;   // workgroups along the query axis of one head
    const Problem pr = decode_problem<BM, BN, CAUSAL>(a, L, qstep);
    if (pr.skip) return;                               // uniform over the workgroup
    int qb = pr.qb;
    const int split = pr.split, bh = pr.bh;
    const int b = bh / a.H, hd = bh % a.H;
    const int Wq = pr.W, NK = pr.NK;                   // query and key rows of this problem

    int t0, t1;
    if (CAUSAL) {
        t0 = 0;
        const int kend = min(NK, qb * BM + BM);
        t1 = (kend + BN - 1) / BN;
    } else {
        t0 = split * pr.tps;
        t1 = min(t0 + pr.tps, (NK + BN - 1) / BN);
    }

    const int64_t k_rb = a.k_sr * 2, v_rb = a.v_sr * 2;
    const __bf16 *Qg = (const __bf16 *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh + pr.qrow_off * a.q_sr;
    const char *Kg = (const char *)((const __bf16 *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh) + pr.krow_off * k_rb;
    const char *Vg = (const char *)((const __bf16 *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh) + pr.krow_off * v_rb;

    // Tensors with a head dimension a.D below the kernel's D: whole 16-byte chunks of a row exist
    // up to dchunks; Q is taken as zero from column a.D on, and in the one chunk of a K row that
    // straddles a.D the part from a.D on (the caller's padding, which may hold anything) is
    // cleared in LDS by the wave that loaded the row, between its wait for the load and the
    // tile's barrier.
    const int dchunks = PAD ? (a.D + 7) >> 3 : D / 8;
    const int straddle = (PAD && (a.D & 7)) ? (a.D >> 4) : -1;   // contraction step whose fragment straddles a.D
    // clears the elements from column a.D on in the fragment of that step (computed where needed:
    // the mask is not kept in registers, the step is rare)
    auto clip = [&](bf16x8 f) __attribute__((always_inline)) {
        const int keep = a.D - (16 * straddle + 8 * h);     // elements this lane keeps (may be <= 0 or >= 8)
        u32x4 u = __builtin_bit_cast(u32x4, f);
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] &= keep >= 2 * e + 2 ? ~0u : keep == 2 * e + 1 ? 0x0000ffffu : 0u;
        return __builtin_bit_cast(bf16x8, u);
    };

    int qrow0 = qb * BM + wave * (QB * 32);
    bf16x8 qf[QB][DS];
    // Q^T fragments (B operand): lane holds query j, contraction elements 16*s + 8*h .. +7.
    // fragment of contraction step s of the query row at qp (columns from a.D on count as zeros)
    auto q_fragment = [&](const __bf16 *qp, int s) __attribute__((always_inline)) {
        if (PAD && 16 * s + 8 * h >= a.D) return bf16x8{};
        const bf16x8 f = *(const bf16x8 *)(qp + 16 * s);
        return (PAD && s == straddle) ? clip(f) : f;
    };
    auto load_q = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) {
            const int r = min(qrow0 + qi * 32 + j, Wq - 1);
            const __bf16 *qp = Qg + (int64_t)r * a.q_sr + 8 * h;
#pragma unroll
            for (int s = 0; s < DS; ++s) qf[qi][s] = q_fragment(qp, s);
        }
        // Consume the Q registers here, so that the wait for these loads sits before the tile loop
        // and not inside it, where it would also wait for the tile loads in flight.
#pragma unroll
        for (int qi = 0; qi < QB; ++qi)
#pragma unroll
            for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(qf[qi][s]));
    };
    if (!RESIDENT) load_q();

    // Direct load i of this wave covers tile rows (wave*NDMA + i)*RPI .. +RPI-1; this lane lands
    // on row drow[i], chunk position lane % CPR, and so fetches chunk (lane % CPR) ^ swz(row).
    int drow[NDMA];
    unsigned koff[NDMA], voff[NDMA];       // byte offsets inside a tile (the host bounds the row strides)
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        drow[i] = (wave * NDMA + i) * RPI + lane / CPR;
        // rows shorter than the kernel's D (a.D < D): chunks past the end of a row are not in
        // memory; their places in LDS are cleared instead (they only meet zero columns of Q, and the
        // output columns they produce are not stored)
        const int kc = (lane % CPR) ^ Swz<D>::k(drow[i]), vc = (lane % CPR) ^ Swz<D>::v(drow[i]);
        koff[i] = (PAD && kc >= dchunks) ? kNoChunk : (unsigned)(drow[i] * k_rb) + (kc << 4);
        voff[i] = (PAD && vc >= dchunks) ? kNoChunk : (unsigned)(drow[i] * v_rb) + (vc << 4);
    }
    auto issue = [&](int t, int stage) __attribute__((always_inline)) {
        const int key0 = t * BN;
        const unsigned kdst = __builtin_amdgcn_readfirstlane(lds_offset(Ks) + stage * TILE_B + wave * (NDMA * 1024));
        const unsigned vdst = kdst + NSTAGE * TILE_B;
        // rows past the end of the tensor (ragged last tile) lie beyond the descriptor's size and
        // arrive as zeros; their scores are masked
        const int rows = min(BN, NK - key0);
        const u32x4 kd = tile_descriptor(Kg + key0 * k_rb, (PAD || rows < BN) ? (unsigned)(rows * k_rb) : 0xffffffffu);
        const u32x4 vd = tile_descriptor(Vg + key0 * v_rb, (PAD || rows < BN) ? (unsigned)(rows * v_rb) : 0xffffffffu);
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            direct_load_1k(kd, koff[i], kdst + i * 1024);
            direct_load_1k(vd, voff[i], vdst + i * 1024);
        }
    };

    // PAD, a.D not a multiple of 8: clears elements a.D .. of the straddling chunk (8 bytes: a.D is
    // a multiple of 4) in the K rows of a stage that this wave loaded; lane i takes the i-th of them
    auto scrub = [&](int stage) __attribute__((always_inline)) {
        if (!PAD || !(a.D & 7)) return;
        if (lane < NDMA * RPI) {
            const int r = (wave * NDMA + lane / RPI) * RPI + lane % RPI;      // tile row
            const int pos = (a.D >> 3) ^ Swz<D>::k(r);                        // where its straddling chunk sits
            *(u32x2 *)(Ks + stage * TILE_B + r * ROWB + (pos << 4) + 8) = u32x2{0u, 0u};
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // written before the barrier is passed
    };

    f32x16 oacc[QB][DB];
    float m[QB], l[QB];
    auto reset = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) {
            m[qi] = -INFINITY;
            l[qi] = 0.f;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[qi][db][v] = 0.f;
        }
    };
    reset();
    // The running maximum is only advanced when a row's tile maximum exceeds it by more than
    // 2^8 in the exponent: weights then stay <= 256, and the accumulator is rescaled rarely.
    // Any reference point gives the same normalised result, so this is exact.
    const float thr = 8.0f / a.c;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
    bf16x8 pb[QB][2][2];   // softmax weights of the current tile, B-operand order

    // ---- scores and online softmax of one tile: S^T = K Q^T, mask, update m/l, weights -> pb
    auto scores_softmax = [&](const char *Kt, int key0) __attribute__((always_inline)) {
        f32x16 sacc[QB][2];
        // Register budget decides how the K fragments come from LDS.  AHEAD: all fragments of the
        // tile are requested back to back before the first product.  Otherwise one 32-key block
        // at a time, under the compiler's own waits (the resident variant also holds the next
        // block's queries and would spill; its waves are not in lock-step, so it gains nothing).
        constexpr bool AHEAD = QB == 1 && !RESIDENT;
        if constexpr (AHEAD) {
            // Requests go out in the order the products consume them (contraction step outer,
            // 32-key block inner), and every product waits only until its own operand has
            // arrived: LDS reads complete in order, so operand number i of n is there once at most
            // n-1-i reads are outstanding.  The reads and the waits are written as assembly because
            // the compiler otherwise waits for all of them before the first product.  (Outstanding
            // reads the compiler adds on its own can only make a wait longer, never too short.)
            bf16x8 kf[2][DS];
            const unsigned kaddr = lds_offset(Kt) + j * ROWB;
            const int ksw = Swz<D>::k(j);                 // same for keys j and j + 32
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                const unsigned addr = kaddr + (((2 * s + h) ^ ksw) << 4);
                asm volatile("ds_read_b128 %0, %1" : "=v"(kf[0][s]) : "v"(addr));
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(kf[1][s]) : "v"(addr), "n"(32 * ROWB));
            }
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[0][kk][v] = 0.f;
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(kf[0][s]) : "n"(2 * DS - 1 - 2 * s));
                sacc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][s], qf[0][s], sacc[0][0], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);       // keep each product between its wait and the next
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(kf[1][s]) : "n"(2 * DS - 2 - 2 * s));
                sacc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][s], qf[0][s], sacc[0][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                bf16x8 kf[DS];
                const int key = kb * 32 + j;
                const char *krow = Kt + key * ROWB;
                const int ksw = Swz<D>::k(key);
#pragma unroll
                for (int s = 0; s < DS; ++s) kf[s] = *(const bf16x8 *)(krow + (((2 * s + h) ^ ksw) << 4));
#pragma unroll
                for (int qi = 0; qi < QB; ++qi)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sacc[qi][kb][v] = 0.f;
#pragma unroll
                for (int s = 0; s < DS; ++s)
#pragma unroll
                    for (int qi = 0; qi < QB; ++qi)
                        sacc[qi][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[qi][s], sacc[qi][kb], 0, 0, 0);
            }
        }

        // mask: keys past the end of the tensor, and (causal) keys after the query row
        const bool ragged = key0 + BN > NK;
        const bool diag = CAUSAL && (key0 + BN - 1 > qrow0);
        if (ragged || diag) {
#pragma unroll
            for (int qi = 0; qi < QB; ++qi) {
                const int row = qrow0 + qi * 32 + j;
                const int lim = CAUSAL ? min(row, NK - 1) : NK - 1;   // last visible key
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                        if (key > lim) sacc[qi][kb][v] = -INFINITY;
                    }
            }
        }

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
            // weights, rounded to bf16; the row sum is accumulated from the rounded values (the ones
            // the value product uses) with v_dot2c_f32_bf16 against (1, 1): two weights per instruction
            float ls = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const __bf16 p0 = (__bf16)fast_exp2(fmaf(sacc[qi][kb][8 * t2 + e], a.c, -mc));
                        const __bf16 p1 = (__bf16)fast_exp2(fmaf(sacc[qi][kb][8 * t2 + e + 1], a.c, -mc));
                        pb[qi][kb][t2][e] = p0;
                        pb[qi][kb][t2][e + 1] = p1;
                        const bf16x2 pp = {p0, p1};
                        ls = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, ls, false);
                    }
            l[qi] += ls;
        }
    };

    // ---- O^T += V^T P^T for the tile whose weights are in pb
    auto accumulate = [&](const char *Vt) __attribute__((always_inline)) {
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
    };

    // A tile is skipped by a wave when it lies after every row the wave owns (causal only).
    auto active = [&](int t) { return !CAUSAL || t * BN <= qrow0 + QB * 32 - 1; };

    // Ring protocol.  Before the loop the loads of tiles t0 .. t0+PD-1 are issued.  Iteration t
    // waits until this wave's loads of tile t have landed, meets the other waves at the barrier
    // (now the whole tile is visible, and every wave has finished reading tile t-1), then issues the loads of tile t+PD into the
    // stage that was released, and computes on tile t.
    constexpr int PER_TILE = 2 * NDMA;
    if (RESIDENT) {
        // the partition has at most NSTAGE tiles (checked by the host): tile t lives in stage t
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < t1) issue(s, s);
        load_q();
        wait_vmcnt<0>();
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < t1) scrub(s);
        __builtin_amdgcn_s_barrier();
    } else {
#pragma unroll
        for (int s = 0; s < PD; ++s)
            if (t0 + s < t1) issue(t0 + s, s);
    }
  do {
    bf16x8 qn[QB][DS];   // resident variant: the next block's queries, requested before this block's work
    if (RESIDENT) {
        if (qb + qstep < a.nqb) {
            const int nrow0 = (qb + qstep) * BM + wave * (QB * 32);
#pragma unroll
            for (int qi = 0; qi < QB; ++qi) {
                const int r = min(nrow0 + qi * 32 + j, Wq - 1);
                const __bf16 *qp = Qg + (int64_t)r * a.q_sr + 8 * h;
#pragma unroll
                for (int s = 0; s < DS; ++s) qn[qi][s] = q_fragment(qp, s);
            }
        }
        for (int t = 0; t < t1; ++t) {
            scores_softmax(Ks + t * TILE_B, t * BN);
            accumulate(Vs + t * TILE_B);
        }
    } else {
        for (int t = t0; t < t1; ++t) {
            const int n = t - t0;
            if (t + PD - 1 < t1) wait_vmcnt<(PD - 1) * PER_TILE>();   // PD-1 younger tiles may still fly
            else wait_vmcnt<0>();
            scrub(n % NSTAGE);
            __builtin_amdgcn_s_barrier();
            if (t + PD < t1) issue(t + PD, (n + PD) % NSTAGE);
            if (active(t)) {
                scores_softmax(Ks + (n % NSTAGE) * TILE_B, t * BN);
                accumulate(Vs + (n % NSTAGE) * TILE_B);
            }
        }
    }

    // ---- epilogue.  Accumulator register v of block db is d = 32*db + 8*(v/4) + 4*h + v%4.
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        const float lt = xhalf_sum(l[qi]);
        const int row = qrow0 + qi * 32 + j;
        if (row >= Wq) continue;
        if (a.direct) {
            const float inv = 1.0f / lt;
            const int64_t off = (int64_t)b * a.o_sb + (int64_t)hd * a.o_sh + (pr.qrow_off + row) * a.o_sr;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = 32 * db + 8 * g + 4 * h;
                    if (PAD && d >= a.D) continue;       // column beyond the tensors' head dimension
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
            if (a.lse && h == 0) a.lse[(int64_t)bh * a.W + row] = m[qi] * a.scale + logf(lt);
        } else {
            const int64_t slot = pr.slot + a.part0 + (CAUSAL ? 0 : split);
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
    if (RESIDENT) {
        qb += qstep;
        if (qb < a.nqb) {
            qrow0 = qb * BM + wave * (QB * 32);
#pragma unroll
            for (int qi = 0; qi < QB; ++qi)
#pragma unroll
                for (int s = 0; s < DS; ++s) qf[qi][s] = qn[qi][s];
            reset();
        }
    }
  } while (RESIDENT && qb < a.nqb);
}

}  // namespace tlin

#include "attn_bf16_pipe.h"

namespace tlin {

// Which shapes run the software-pipelined body: the unmasked partitions with one query block per
// wave and a ring of two tiles (measured against attn_bf16_body on every such shape: faster, none
// slower), and the stand-alone causal kernel.  The causal window blocks that ride in a layer call's
// launch, the resident variant for odd tile counts and the deeper rings keep the classic body.
template <int D, int NW, int QB, bool CAUSAL, int NSTAGE, bool RESIDENT>
constexpr bool use_pipe_body()
{
    // (the stand-alone causal kernel: at head dimension 128 only, measured 5 % faster at 4096 rows; at 64
    // the classic body with its ring of four is 1-3 % ahead)
    return !RESIDENT && QB == 1 && NSTAGE == 2 && (!CAUSAL || D == 128);
}

// NT (pipelined shapes only): the tile loads carry the non-temporal hint, see direct_load_1k.
template <int D, int NW, int QB, bool CAUSAL, int NSTAGE, bool RESIDENT = false, bool PAD = false, bool NT = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NSTAGE == 2 && NW < 8 ? 2 : 1, 8)))
void attn_bf16_kernel(const AttnArgs a)
{
    static_assert(!NT || use_pipe_body<D, NW, QB, CAUSAL, NSTAGE, RESIDENT>(), "only the pipelined body has a non-temporal variant");
    if constexpr (use_pipe_body<D, NW, QB, CAUSAL, NSTAGE, RESIDENT>()) attn_bf16_pipe_body<D, NW, PAD, NT, CAUSAL>(a, blockIdx.x, gridDim.x);
    else attn_bf16_body<D, NW, QB, CAUSAL, NSTAGE, RESIDENT, PAD>(a, blockIdx.x, gridDim.x);
}

// Resident key/value side with the in-wave pipeline (an even number T1 of key tiles).
template <int D, int T1, int TMAX, bool PAD = false>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(1, 8)))
void attn_bf16_resident_pipe_kernel(const AttnArgs a)
{
    attn_bf16_resident_pipe_body<D, 8, PAD, T1, TMAX>(a, blockIdx.x, gridDim.x);
}

// History partition blocks and window causal blocks of one call in a single launch.
template <int D, int NW, int NSTAGE, bool PAD = false, bool NT = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NSTAGE == 2 && NW < 8 ? 2 : 1, 8)))
void attn_bf16_pair_kernel(const PairArgs f)
{
    static_assert(!NT || use_pipe_body<D, NW, 1, false, NSTAGE, false>(), "only the pipelined body has a non-temporal variant");
    // logical index of the window block this workgroup computes, or -1
    int win_block = (int)blockIdx.x < f.n_hist_blocks ? -1 : xcd_remap(blockIdx.x - f.n_hist_blocks, f.n_win_blocks);
    if ((int)blockIdx.x < f.n_hist_blocks) {
        if constexpr (use_pipe_body<D, NW, 1, false, NSTAGE, false>()) {
            attn_bf16_pipe_body<D, NW, PAD, NT>(f.hist, blockIdx.x, f.n_hist_blocks);
            if (f.hist.fuse_window) {
                // the workgroup of partition 0 goes on to the window's causal block of the same rows
                // (causal blocks are numbered from the last query block down)
                const Problem pr = decode_problem<NW * 32, 64, false>(f.hist, xcd_remap(blockIdx.x, f.n_hist_blocks), f.hist.nqb);
                if (pr.split == 0) {
                    win_block = pr.bh * f.win.nqb + (f.win.nqb - 1 - pr.qb);
                    __syncthreads();      // every wave is done with the history tiles in LDS
                }
            }
        } else {
            attn_bf16_body<D, NW, 1, false, NSTAGE, false, PAD>(f.hist, blockIdx.x, f.n_hist_blocks);
        }
    }
    if (win_block >= 0) attn_bf16_body<D, NW, 1, true, NSTAGE, false, PAD, false>(f.win, win_block, 0);
}

}  // namespace tlin
