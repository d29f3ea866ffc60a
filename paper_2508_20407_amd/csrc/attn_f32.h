// fp32 attention over one key partition on the gfx950 matrix cores, fp32 operands and fp32
// accumulation throughout (v_mfma_f32_32x32x2_f32: no operand is rounded below fp32), for fp32
// inputs.  Same online-softmax recurrence, same partial format and the same transposed mapping
// as the bf16 kernel (Section 3 of the paper: softmax(scale * Q K^T) V; window keys masked with
// j <= i).
//
// Mapping (wave64; a wave owns 32 query rows, lane = (query j = lane % 32, half h = lane / 32)):
//   * A 32x32x2 product contracts over two indices, one per half-wave.  Which two is free as long
//     as both operands agree, and the pairings are chosen so that no data ever moves between
//     lanes:
//       scores  S^T[key, query] = K Q^T : step (t, e) pairs d = 8t + e (h = 0) with d = 8t + 4 + e
//               (h = 1).  A lane then needs K[key j][8t + 4h .. +3] - one 16-byte LDS read per four
//               products - and Q[query j][8t + 4h .. +3], which it keeps in registers.
//       values  O^T[d, query] += V^T P^T : the score accumulator leaves key 8g + 4h + e of the tile
//               in register 4g + e of half h, so step (g, e) pairs key 8g + e with key 8g + 4 + e:
//               the B operand is that accumulator register as it stands (after the exponential),
//               and the A operand is V[key 8g + 4h + e][32 db + j], one 4-byte LDS read.
//   * K/V tiles of 32 keys go HBM -> LDS directly (1 KB per wave instruction) through a ring of
//     two tiles, one barrier per tile, as in the bf16 kernel (two-wave workgroups: one tile, two
//     barriers).  LDS rows are XOR-swizzled per
//     16-byte chunk on the source side of the load: K chunk ^ (row & 15), so that the 16 lanes of a
//     128-bit read cover all 64 banks; V chunk ^ 8 for rows with bit 2 set, so that the two
//     half-waves (rows 4 apart, same columns) read different halves of the bank sweep.
//   * Tensors with a head dimension a.D below the kernel's D: a.D is a multiple of 4, so 16-byte
//     chunks are either whole or absent; the places of absent chunks are cleared in LDS by the load
//     (lane offsets beyond the tile descriptor's size: zeros, no memory request) and meet zero
//     columns of Q, and output columns from a.D on are not stored.
#pragma once
#include "common.h"

namespace tlin {

struct SwzF32 {
    static __device__ __forceinline__ int k(int r) { return r & 15; }
    static __device__ __forceinline__ int v(int r) { return ((r >> 2) & 1) << 3; }
};

// The work of one workgroup; `bid` of `nblocks` is its index among the blocks of this problem set.
// REMAP: bid is a hardware block index (mapped to a logical one here); otherwise it is the logical index.
template <int D, int NW, bool CAUSAL, bool REMAP = true>
__device__ __forceinline__ void attn_f32_body(const AttnArgs &a, int bid, int nblocks)
{
    constexpr int BN = 32;                 // keys per tile
    constexpr int BM = NW * 32;            // query rows per workgroup
    constexpr int ROWB = D * 4;            // bytes per K/V row
    constexpr int TILE_B = BN * ROWB;
    constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;       // rows moved by one wave-wide direct load
    constexpr int NDMA = BN / RPI / NW;    // direct loads per wave per tensor per tile
    static_assert(BN % (RPI * NW) == 0 && NDMA >= 1, "tile does not divide over the waves");
    // Two-wave workgroups (few query rows) keep a single tile in LDS, so that four of them share a
    // compute unit and every SIMD has two waves: their loads are hidden by the other workgroups.
    constexpr int NSTAGE = NW == 2 ? 1 : 2;
    constexpr int DT = D / 8;              // 16-byte operand fragments per row and half-wave
    constexpr int DB = D / 32;             // 32-row blocks of O^T
    static_assert(2 * NDMA < 64, "too many loads in flight for vmcnt");

    char *const Ks = tlin_smem;
    char *const Vs = tlin_smem + NSTAGE * TILE_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;

    const int L = REMAP ? xcd_remap(bid, nblocks) : bid;
    const Problem pr = decode_problem<BM, BN, CAUSAL>(a, L, a.nqb);
    if (pr.skip) return;                   // uniform over the workgroup
    const int qb = pr.qb, split = pr.split, bh = pr.bh;
    const int b = bh / a.H, hd = bh % a.H;
    const int Wq = pr.W, NK = pr.NK;       // query and key rows of this problem

    int t0 = 0, t1 = (min(NK, qb * BM + BM) + BN - 1) / BN;
    if (!CAUSAL) partition_tiles<BM, BN, 4>(a, pr, t0, t1);

    const int64_t k_rb = a.k_sr * 4, v_rb = a.v_sr * 4;
    const float *Qg = (const float *)a.Q + (int64_t)b * a.q_sb + (int64_t)hd * a.q_sh + pr.qrow_off * a.q_sr;
    const char *Kg = (const char *)((const float *)a.K + (int64_t)b * a.k_sb + (int64_t)hd * a.k_sh) + pr.krow_off * k_rb;
    const char *Vg = (const char *)((const float *)a.V + (int64_t)b * a.v_sb + (int64_t)hd * a.v_sh) + pr.krow_off * v_rb;

    // ---- Q^T fragments (B operand of the score product), register resident
    const int qrow0 = qb * BM + wave * 32;
    f32x4 qf[DT];
    {
        const int r = min(qrow0 + j, Wq - 1);
        const float *qp = Qg + (int64_t)r * a.q_sr + 4 * h;
#pragma unroll
        for (int t = 0; t < DT; ++t)
            qf[t] = 8 * t + 4 * h < a.D ? *(const f32x4 *)(qp + 8 * t) : f32x4{0.f, 0.f, 0.f, 0.f};
        // consume the registers here, so that the wait for these loads sits before the tile loop
#pragma unroll
        for (int t = 0; t < DT; ++t) asm volatile("" : "+v"(qf[t]));
    }

    // ---- direct loads: load i of this wave covers tile rows (wave*NDMA + i)*RPI .. +RPI-1; this lane
    // lands on chunk position lane % CPR of row drow and fetches chunk (lane % CPR) ^ swz(row)
    const int dchunks = a.D / 4;
    unsigned koff[NDMA], voff[NDMA];
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        const int drow = (wave * NDMA + i) * RPI + lane / CPR;
        const int kc = (lane % CPR) ^ SwzF32::k(drow), vc = (lane % CPR) ^ SwzF32::v(drow);
        koff[i] = kc >= dchunks ? kNoChunk : (unsigned)(drow * k_rb) + (kc << 4);
        voff[i] = vc >= dchunks ? kNoChunk : (unsigned)(drow * v_rb) + (vc << 4);
    }
    auto issue = [&](int t, int stage) __attribute__((always_inline)) {
        const int key0 = t * BN;
        const unsigned kdst = __builtin_amdgcn_readfirstlane(lds_offset(Ks) + stage * TILE_B + wave * (NDMA * 1024));
        const unsigned vdst = kdst + NSTAGE * TILE_B;
        // rows past the end of the tensor lie beyond the descriptor's size and arrive as zeros
        const int rows = min(BN, NK - key0);
        const u32x4 kd = tile_descriptor(Kg + key0 * k_rb, (a.D < D || rows < BN) ? (unsigned)(rows * k_rb) : 0xffffffffu);
        const u32x4 vd = tile_descriptor(Vg + key0 * v_rb, (a.D < D || rows < BN) ? (unsigned)(rows * v_rb) : 0xffffffffu);
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            direct_load_1k(kd, koff[i], kdst + i * 1024);
            direct_load_1k(vd, voff[i], vdst + i * 1024);
        }
    };

    // ---- state: running maximum (raw logit units), running sum, O^T accumulator
    float m = -INFINITY, l = 0.f;
    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    // The running maximum only moves when a tile maximum exceeds it by more than 2^8 in the
    // exponent: weights stay <= 256 and the accumulator is rescaled rarely.  Any reference point
    // gives the same normalised result.
    const float thr = 8.0f / a.c;

    // per-lane parts of the LDS addresses
    const unsigned kfrag = j * ROWB;                       // + ((2t + h) ^ k(j)) * 16
    const int ksw = SwzF32::k(j);
    unsigned vfrag[DB];                                    // + key * ROWB
#pragma unroll
    for (int db = 0; db < DB; ++db) vfrag[db] = 128 * (db ^ h) + 4 * j + 4 * h * ROWB;   // row 4h, chunk ^ 8h

    // Causal: tiles after every row this wave owns are not computed by it, but the wave still
    // loads its share of them for the others and meets them at the barriers (second loop).
    const int t1w = CAUSAL ? min(t1, (qrow0 + 31) / BN + 1) : t1;
    if (t0 < t1) issue(t0, 0);
    for (int t = t0; t < t1w; ++t) {
        const int n = t - t0;
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();      // tile t is complete, and (two stages) every wave has left tile t-1
        if (NSTAGE == 2 && t + 1 < t1) issue(t + 1, (n + 1) % NSTAGE);
        const int key0 = t * BN;
        const char *Kt = Ks + (n % NSTAGE) * TILE_B;
        const char *Vt = Vs + (n % NSTAGE) * TILE_B;

        // ---- scores S^T = K Q^T
        // The contraction over D runs as chains of 32 terms, each started from zero and added to
        // the total when complete: the rounding error of an fp32 chain grows with its length, and
        // the error of a score is what limits the accuracy of the weights (short rows most of all,
        // where nothing averages out).
        f32x16 s;
#pragma unroll
        for (int c4 = 0; c4 < DT / 4; ++c4) {
            f32x16 part;
#pragma unroll
            for (int v = 0; v < 16; ++v) part[v] = 0.f;
#pragma unroll
            for (int t8 = 4 * c4; t8 < 4 * c4 + 4; ++t8) {
                const f32x4 kf = *(const f32x4 *)(Kt + kfrag + (((2 * t8 + h) ^ ksw) << 4));
#pragma unroll
                for (int e = 0; e < 4; ++e) part = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[e], qf[t8][e], part, 0, 0, 0);
            }
            if (c4 == 0) s = part;
            else
#pragma unroll
                for (int v = 0; v < 16; ++v) s[v] += part[v];
        }

        // ---- mask: keys past the end of the tensor, and (causal) keys after the query row
        const int row = qrow0 + j;
        if (key0 + BN > NK || (CAUSAL && key0 + BN - 1 > qrow0)) {
            const int lim = CAUSAL ? min(row, NK - 1) : NK - 1;   // last visible key
            const int rel = lim - key0 - 4 * h;                    // the same, counted from this lane's first key
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + (v & 3) > rel) s[v] = -INFINITY;
        }

        // ---- online softmax
        float mx = s[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
        mx = xhalf_max(mx);
        if (__builtin_amdgcn_ballot_w64(mx > m + thr) != 0) {
            const float mn = fmaxf(m, mx);
            const float alpha = (mn == -INFINITY) ? 1.f : fast_exp2((m - mn) * a.c);
            l *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
            m = mn;
        }
        // (s - m) * c rather than fma(s, c, -m*c): the key that holds the maximum gets weight exactly 1
        const float mref = (m == -INFINITY) ? 0.f : m;
        float ls = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = fast_exp2((s[v] - mref) * a.c);
            ls += s[v];
        }
        l += ls;

        // ---- O^T += V^T P^T: register 4g + e of this half-wave is key 8g + 4h + e.  The tile's
        // product is summed on its own and then added to the running accumulator: two short
        // summation chains (16 steps, then one addition per tile) round less than one long one.
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            f32x16 pv;
#pragma unroll
            for (int v = 0; v < 16; ++v) pv[v] = 0.f;
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float vf = *(const float *)(Vt + vfrag[db] + (8 * g + e) * ROWB);
                    pv = __builtin_amdgcn_mfma_f32_32x32x2f32(vf, s[4 * g + e], pv, 0, 0, 0);
                }
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][v] += pv[v];
            __builtin_amdgcn_sched_barrier(0);     // keeps the next block's V reads (registers) behind this block
        }
        if (NSTAGE == 1 && t + 1 < t1) {
            __builtin_amdgcn_s_barrier();          // every wave has left the tile that is overwritten now
            issue(t + 1, 0);
        }
    }

    for (int t = t1w; CAUSAL && t < t1; ++t) {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (NSTAGE == 2 && t + 1 < t1) issue(t + 1, (t - t0 + 1) % NSTAGE);
        if (NSTAGE == 1 && t + 1 < t1) {
            __builtin_amdgcn_s_barrier();
            issue(t + 1, 0);
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
                if (d >= a.D) continue;            // column beyond the tensors' head dimension
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

template <int D, int NW, bool CAUSAL>
__global__ __launch_bounds__(NW * 64) void attn_f32_kernel(const AttnArgs a)
{
    attn_f32_body<D, NW, CAUSAL>(a, blockIdx.x, gridDim.x);
}

// History partition blocks and window causal blocks of one call in a single launch.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_f32_pair_kernel(const PairArgs f)
{
    // logical index of the window block this workgroup computes, or -1
    int win_block = (int)blockIdx.x < f.n_hist_blocks ? -1 : xcd_remap(blockIdx.x - f.n_hist_blocks, f.n_win_blocks);
    if ((int)blockIdx.x < f.n_hist_blocks) {
        attn_f32_body<D, NW, false>(f.hist, blockIdx.x, f.n_hist_blocks);
        if (f.hist.fuse_window) {
            // the workgroup of partition 0 goes on to the window's causal block of the same rows
            // (causal blocks are numbered from the last query block down)
            const Problem pr = decode_problem<NW * 32, 32, false>(f.hist, xcd_remap(blockIdx.x, f.n_hist_blocks), f.hist.nqb);
            if (pr.split == 0) {
                win_block = pr.bh * f.win.nqb + (f.win.nqb - 1 - pr.qb);
                __syncthreads();      // every wave is done with the history tiles in LDS
            }
        }
    }
    if (win_block >= 0) attn_f32_body<D, NW, true, false>(f.win, win_block, 0);
}

}  // namespace tlin
