// libtlinattn: C-ABI entry points (see include/tlinattn.h), argument validation, partition
// planning and kernel launches.  gfx950 only.
#include "tlinattn.h"
#include "tlinattn_profile.h"

#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

#include "attn_bf16.h"
#include "attn_f32.h"
#include "decode.h"
#include "merge.h"

using namespace tlin;

// Workspace of tlin_layer_attn_static_ws: split partials of the history axis and the window
// partial, for callers that cannot bring device memory of their own.  Host code never uses this
// name as an address; static_scratch() asks the runtime for the array's address on the current device.
static __device__ __align__(256) unsigned char scratch[TLIN_STATIC_WS_BYTES];

namespace {

constexpr int kVersion = 200;   // 0.2.0
constexpr int kMaxRows = 1 << 30;

// One kernel launch, reporting the status of this launch only: errors that the caller's earlier
// work left behind stay where they are (nothing here reads or clears the runtime's last error).
// Every kernel of the library takes a single argument structure by value.
template <typename Args>
tlin_status launch_kernel(const void *kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st, const Args &a)
{
    void *argv[] = {const_cast<Args *>(&a)};
    return hipLaunchKernel(kernel, grid, block, argv, lds_bytes, st) == hipSuccess ? TLIN_OK : TLIN_ERR_HIP;
}

// The kernels and the partition planning are written for MI355X: gfx950, 256 compute units in 8
// XCDs (kNumCU, kNumXCD).  Checked once per device ordinal, after argument validation and before
// the first launch on that device.
tlin_status check_device()
{
    static std::atomic<uint64_t> good{0}, bad{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TLIN_ERR_HIP;
    if (dev < 0 || dev >= 64) return TLIN_ERR_UNSUPPORTED;
    const uint64_t bit = (uint64_t)1 << dev;
    if (good.load(std::memory_order_acquire) & bit) return TLIN_OK;
    if (bad.load(std::memory_order_acquire) & bit) return TLIN_ERR_UNSUPPORTED;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return TLIN_ERR_HIP;
    const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0 && prop.multiProcessorCount == kNumCU;
    (ok ? good : bad).fetch_or(bit, std::memory_order_release);
    return ok ? TLIN_OK : TLIN_ERR_UNSUPPORTED;
}

struct Strides { int64_t b, h, r; };

// Kernel shape chosen for a bf16 problem: NW waves, QB query blocks of 32 rows per wave.
struct Shape { int nw, qb; int bm() const { return nw * qb * 32; } };

Shape wave_shape(int W)
{
    if (W > 128) return {8, 1};
    if (W > 64) return {4, 1};
    return {2, 1};
}

// Head dimensions other than 64 and 128 run in the next of the two kernel sizes: the kernels
// treat the missing columns of Q as zeros and do not store the extra output columns.
int dpad(int D) { return D <= 64 ? 64 : 128; }

// Keys per tile: 32 KB of K and V per tile in both kernels.  Query rows per workgroup: the same
// shapes for both input types.
int key_tile(int in_dtype, int) { return in_dtype == TLIN_F32 ? 32 : 64; }
// bf16 at head dimension 64 and below stays with four waves for long windows too: its pipelined body
// takes 153 registers, so three waves fit a SIMD, which is three four-wave workgroups per compute
// unit but only one of eight waves (12 heads x 36, 256 window rows over 131072 / 999754 history
// rows: 0.135 / 0.911 ms per step against 0.148 / 0.940 ms with eight-wave workgroups).
Shape kernel_shape(int in_dtype, int W, int D)
{
    const Shape s = wave_shape(W);
    if (in_dtype == TLIN_BF16 && dpad(D) == 64 && s.nw == 8) return {4, 1};
    return s;
}
int query_block(int in_dtype, int W, int D) { return kernel_shape(in_dtype, W, D).bm(); }

// Workgroups the chip holds at once for a given kernel shape (LDS- and register-limited).
int resident_wgs(int in_dtype, int W, int D)
{
    if (in_dtype == TLIN_F32) {
        // fp32 kernel: two waves per SIMD keep the matrix cores busy (8 waves per compute unit); its
        // tile ring takes 64 KB of the 160 KB of LDS at D = 128 and 32 KB at D = 64 (half of that in
        // the two-wave shape)
        const int nw = wave_shape(W).nw;
        const int by_waves = 8 / nw, by_lds = (dpad(D) == 128 ? 2 : 4) * (nw == 2 ? 2 : 1);
        return kNumCU * (by_waves < by_lds ? by_waves : by_lds);
    }
    // head dimension 64: tiles and register sets are half as large, three workgroups share a
    // compute unit (measured best for few heads); 128: an eight-wave workgroup fills a compute unit
    // alone (registers), two of the smaller ones share it (two-tile LDS ring of 64 KB each)
    if (dpad(D) == 64) return kNumCU * 3;
    return kNumCU * (wave_shape(W).nw == 8 ? 1 : 2);
}

// ---- measurement aid: per-kernel timing with HIP events on the launch stream
enum KernelClass { KC_HISTORY = 0, KC_WINDOW = 1, KC_MERGE = 2, KC_COUNT = 3 };

struct Timed { int cls; hipEvent_t start, stop; };
struct Profiler {
    std::atomic<bool> on{false};
    std::vector<Timed> used;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
    std::mutex mu;
} g_prof;

// Brackets one launch with events when profiling is enabled.
struct LaunchTimer {
    bool active = false;
    Timed t{};
    hipStream_t st;
    LaunchTimer(int cls, hipStream_t s) : st(s)
    {
        if (!g_prof.on) return;
        std::lock_guard<std::mutex> lk(g_prof.mu);
        if (g_prof.pool.empty()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
            g_prof.pool.push_back({a, b});
        }
        t = {cls, g_prof.pool.back().first, g_prof.pool.back().second};
        g_prof.pool.pop_back();
        active = hipEventRecord(t.start, st) == hipSuccess;
        if (!active) g_prof.pool.push_back({t.start, t.stop});
    }
    ~LaunchTimer()
    {
        if (!active) return;
        const bool ok = hipEventRecord(t.stop, st) == hipSuccess;
        std::lock_guard<std::mutex> lk(g_prof.mu);
        if (ok) g_prof.used.push_back(t);
        else g_prof.pool.push_back({t.start, t.stop});
    }
};

bool dense(const int64_t s[3]) { return s[0] == 0 && s[1] == 0 && s[2] == 0; }

Strides resolve(const int64_t s[3], int H, int rows, int D)
{
    if (dense(s)) return {(int64_t)H * rows * D, (int64_t)rows * D, (int64_t)D};
    return {s[0], s[1], s[2]};
}

tlin_status check_strides(const int64_t s[3], int D, int elem_bytes)
{
    const int per16 = 16 / elem_bytes;
    // rows are read in 16-byte pieces: a row holds D elements rounded up to whole pieces
    const int row_elems = (D + per16 - 1) / per16 * per16;
    if (dense(s)) return TLIN_OK;   // whether a dense layout is possible is checked per call, for the tensors it uses
    if (s[2] < row_elems || s[0] < 0 || s[1] < 0) return TLIN_ERR_INVALID_ARG;
    // a tile of 64 rows is addressed with 32-bit byte offsets
    if (s[2] * elem_bytes >= (int64_t)1 << 25) return TLIN_ERR_INVALID_ARG;
    if (s[0] % per16 || s[1] % per16 || s[2] % per16) return TLIN_ERR_INVALID_ARG;
    return TLIN_OK;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// A tensor given without strides is dense, which needs rows of whole 16-byte pieces.
enum Tensor { T_Q = 1, T_KH = 2, T_VH = 4, T_KW = 8, T_VW = 16, T_O = 32 };
tlin_status check_dense_rows(const tlin_params *p, int used)
{
    const int in16 = 16 / (p->in_dtype == TLIN_F32 ? 4 : 2), out16 = 16 / (p->out_dtype == TLIN_F32 ? 4 : 2);
    const struct { int bit; const int64_t *s; int per16; } t[] = {
        {T_Q, p->q_stride, in16}, {T_KH, p->kh_stride, in16}, {T_VH, p->vh_stride, in16},
        {T_KW, p->kw_stride, in16}, {T_VW, p->vw_stride, in16}, {T_O, p->o_stride, out16}};
    for (const auto &x : t)
        if ((used & x.bit) && dense(x.s) && p->D % x.per16) return TLIN_ERR_INVALID_ARG;
    return TLIN_OK;
}

tlin_status check_common(const tlin_params *p, bool need_history, bool allow_empty_history)
{
    if (!p) return TLIN_ERR_INVALID_ARG;
    if (p->B < 1 || p->H < 1 || p->W < 1) return TLIN_ERR_INVALID_ARG;
    if (p->W > kMaxRows || p->N > kMaxRows) return TLIN_ERR_INVALID_ARG;   // tile counts and row indices are 32-bit
    if ((int64_t)p->B * p->H > (1 << 24)) return TLIN_ERR_INVALID_ARG;
    if (need_history && (p->N < (allow_empty_history ? 0 : 1))) return TLIN_ERR_INVALID_ARG;
    if (p->in_dtype != TLIN_F32 && p->in_dtype != TLIN_BF16) return TLIN_ERR_INVALID_ARG;
    if (p->out_dtype != TLIN_F32 && p->out_dtype != TLIN_BF16) return TLIN_ERR_INVALID_ARG;
    if (p->D < 8 || p->D > 128 || p->D % 4) return TLIN_ERR_UNSUPPORTED;
    if (!(p->scale > 0.f) || !isfinite(p->scale)) return TLIN_ERR_INVALID_ARG;
    if (p->num_splits < 0) return TLIN_ERR_INVALID_ARG;
    const int eb = p->in_dtype == TLIN_F32 ? 4 : 2;
    const int ob = p->out_dtype == TLIN_F32 ? 4 : 2;
    tlin_status st;
    if ((st = check_strides(p->q_stride, p->D, eb))) return st;
    if ((st = check_strides(p->kh_stride, p->D, eb))) return st;
    if ((st = check_strides(p->vh_stride, p->D, eb))) return st;
    if ((st = check_strides(p->kw_stride, p->D, eb))) return st;
    if ((st = check_strides(p->vw_stride, p->D, eb))) return st;
    if ((st = check_strides(p->o_stride, p->D, ob))) return st;
    return TLIN_OK;
}

// Partition plan for the history axis.
struct Plan { int nsplit, tiles_per_split; };

Plan plan_history(const tlin_params *p)
{
    if (p->N < 1) return {0, 0};
    const int bn = key_tile(p->in_dtype, dpad(p->D));
    const int ntiles = (p->N + bn - 1) / bn;
    int want;
    if (p->num_splits > 0) {
        want = p->num_splits;
    } else {
        // Enough workgroups to occupy every compute unit, but at least 8 tiles per partition: the
        // merge reads every partial, and with short partitions it would cost more than they save.
        const int64_t base = (int64_t)p->B * p->H * ((p->W + query_block(p->in_dtype, p->W, p->D) - 1) / query_block(p->in_dtype, p->W, p->D));
        const int64_t target = resident_wgs(p->in_dtype, p->W, p->D);
        want = (int)((target + base - 1) / base);
        // (a handful of (head, query block) items cannot fill the chip anyway: there the partials
        // are few in total and short partitions pay)
        const int min_tiles = base <= 4 ? 2 : 8;
        const int cap = ntiles / min_tiles > 1 ? ntiles / min_tiles : 1;
        if (want > cap) want = cap;
    }
    if (want < 1) want = 1;
    if (want > ntiles) want = ntiles;
    if (want > 1024) want = 1024;
    const int tps = (ntiles + want - 1) / want;
    return {(ntiles + tps - 1) / tps, tps};   // no partition is empty
}

// The cache-hit shape (a few query rows over a long history) runs in the streaming kernel of
// decode.h when called through tlin_history_attn.
int decode_max_rows(const tlin_params *p)
{
    // fp32 inputs: the matrix-core path pays for a whole 32-row tile of fp32 products whatever W is
    // (1.39 ms over 131072 rows of 32 heads x 128 against 0.62 ms here)
    if (p->in_dtype == TLIN_F32) return 8;
    // bf16 at head dimension 128: three and four rows are a little faster in the two-wave matrix-core
    // shape (0.309 against 0.323 ms over 131072 rows; both read at the rate of a plain non-temporal
    // read stream), and so are shorter rows at any W
    return p->D == 128 ? 2 : 0;
}
bool use_decode(const tlin_params *p)
{
    return p->W <= decode_max_rows(p) && p->N >= 1024;
}

// One workgroup per partition; four per compute unit (they are small: four waves; more partitions
// only lengthen the merge), at least 256 rows each.
Plan plan_decode(const tlin_params *p)
{
    const int ntiles = (p->N + 63) / 64;
    int want;
    if (p->num_splits > 0) {
        want = p->num_splits;
    } else {
        const int64_t bh = (int64_t)p->B * p->H;
        want = (int)((4 * (int64_t)kNumCU + bh - 1) / bh);
        const int cap = ntiles / 4 > 1 ? ntiles / 4 : 1;
        if (want > cap) want = cap;
    }
    if (want < 1) want = 1;
    if (want > ntiles) want = ntiles;
    if (want > 1024) want = 1024;
    const int tps = (ntiles + want - 1) / want;
    return {(ntiles + tps - 1) / tps, tps};
}

// Sliding schedule: chunks of W rows over a sequence of N rows; every chunk's history is cut into
// the same number of partitions (their length grows with the chunk index).
struct SlidePlan { int nchunks, nsplit, nparts; };

SlidePlan plan_slide(const tlin_params *p)
{
    const int nchunks = (p->N + p->W - 1) / p->W;
    const int bn = key_tile(p->in_dtype, dpad(p->D));
    const int qblk = query_block(p->in_dtype, p->W, p->D);
    const int nqb = (p->W + qblk - 1) / qblk;
    int want;
    if (p->num_splits > 0) {
        want = p->num_splits;
    } else {
        // With many chunks the work items (head, chunk, query block) already outnumber the compute
        // units several times and the long ones start first; split only short sequences.
        const int64_t items = (int64_t)p->B * p->H * nqb * (nchunks > 1 ? nchunks - 1 : 1);
        const int64_t target = 2 * (int64_t)resident_wgs(p->in_dtype, p->W, p->D);
        want = (int)((target + items - 1) / items);
    }
    // at least 4 tiles per partition in the longest history
    const int max_tiles = (int)(((int64_t)(nchunks - 1) * p->W + bn - 1) / bn);
    const int cap = max_tiles / 4 > 1 ? max_tiles / 4 : 1;
    if (want > cap) want = cap;
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    return {nchunks, want, want + 1};
}

size_t slide_ws_bytes(const tlin_params *p, const SlidePlan &pl)
{
    const size_t rows = (size_t)p->B * p->H * pl.nchunks * pl.nparts * p->W;
    return rows * dpad(p->D) * sizeof(float) + 2 * rows * sizeof(float);
}

size_t ws_bytes_for(const tlin_params *p, int nparts)
{
    const size_t rows = (size_t)p->B * p->H * nparts * p->W;
    return rows * dpad(p->D) * sizeof(float) + 2 * rows * sizeof(float);
}

struct Workspace { float *O, *M, *L; };

Workspace carve(void *ws, const tlin_params *p, int nparts)
{
    const size_t rows = (size_t)p->B * p->H * nparts * p->W;
    float *base = (float *)ws;
    return {base, base + rows * dpad(p->D), base + rows * dpad(p->D) + rows};
}

// More than 64 KB of dynamic LDS has to be allowed once per kernel and device.  `done` is the
// calling kernel's own record: one bit per device ordinal.
tlin_status allow_lds(const void *kernel, int lds_bytes, std::atomic<uint64_t> &done)
{
    if (lds_bytes <= 64 * 1024) return TLIN_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TLIN_ERR_HIP;
    const uint64_t bit = (uint64_t)1 << dev;
    if (done.load(std::memory_order_acquire) & bit) return TLIN_OK;
    // two threads may both get here: setting the attribute twice is harmless
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess) return TLIN_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
    return TLIN_OK;
}

template <int D, int NW, int QB, bool CAUSAL, int NSTAGE, bool RESIDENT, bool PAD, bool NT>
tlin_status launch_bf16_kernel(const AttnArgs &a, int grid, hipStream_t st)
{
    constexpr int lds_bytes = 2 * NSTAGE * 64 * D * 2;
    static_assert(lds_bytes <= 160 * 1024, "LDS ring exceeds the 160 KB of a gfx950 compute unit");
    auto kernel = attn_bf16_kernel<D, NW, QB, CAUSAL, NSTAGE, RESIDENT, PAD, NT>;
    static std::atomic<uint64_t> lds_allowed{0};
    if (allow_lds((const void *)kernel, lds_bytes, lds_allowed) != TLIN_OK) return TLIN_ERR_HIP;
    return launch_kernel((const void *)kernel, dim3(grid), dim3(NW * 64), lds_bytes, st, a);
}

// The non-temporal variant exists for the pipelined shapes only.
template <int D, int NW, int QB, bool CAUSAL, int NSTAGE, bool RESIDENT, bool PAD>
tlin_status launch_bf16_shape_pad(const AttnArgs &a, int grid, hipStream_t st)
{
    if constexpr (use_pipe_body<D, NW, QB, CAUSAL, NSTAGE, RESIDENT>()) {
        if (a.stream_once) return launch_bf16_kernel<D, NW, QB, CAUSAL, NSTAGE, RESIDENT, PAD, true>(a, grid, st);
    }
    return launch_bf16_kernel<D, NW, QB, CAUSAL, NSTAGE, RESIDENT, PAD, false>(a, grid, st);
}

// The variant with a.D below the kernel's D is a kernel of its own, so that the exact sizes carry
// none of its code.
template <int D, int NW, int QB, bool CAUSAL, int NSTAGE, bool RESIDENT = false>
tlin_status launch_bf16_shape(const AttnArgs &a, int grid, hipStream_t st)
{
    if (a.D != D) return launch_bf16_shape_pad<D, NW, QB, CAUSAL, NSTAGE, RESIDENT, true>(a, grid, st);
    return launch_bf16_shape_pad<D, NW, QB, CAUSAL, NSTAGE, RESIDENT, false>(a, grid, st);
}

template <int D, int T1, int TMAX>
tlin_status launch_resident_pipe(const AttnArgs &a, int grid, hipStream_t st)
{
    // the resident tiles and, behind them, 4 KB per wave for turning the output rows
    constexpr int lds_bytes = 2 * TMAX * 64 * D * 2 + 8 * 4096;
    static_assert(lds_bytes <= 160 * 1024, "resident tiles exceed the 160 KB of a gfx950 compute unit");
    static std::atomic<uint64_t> lds_allowed[2] = {{0}, {0}};
    const bool pad = a.D != D;
    const void *kernel = pad ? (const void *)attn_bf16_resident_pipe_kernel<D, T1, TMAX, true>
                             : (const void *)attn_bf16_resident_pipe_kernel<D, T1, TMAX, false>;
    if (allow_lds(kernel, lds_bytes, lds_allowed[pad]) != TLIN_OK) return TLIN_ERR_HIP;
    return launch_kernel(kernel, dim3(grid), dim3(512), lds_bytes, st, a);
}

// Ring depth per kernel shape (measured): a compute unit keeps little more than one tile of loads
// in flight, so a deep ring only makes waves wait at the issue of loads that cannot start yet.  Two
// stages also let two of the smaller workgroups share a compute unit.
template <int D, bool CAUSAL>
tlin_status launch_bf16(const AttnArgs &a, Shape s, int grid, hipStream_t st)
{
    constexpr int NS = (CAUSAL && D != 128) ? 4 : 2;
    if (s.nw == 8) return launch_bf16_shape<D, 8, 1, CAUSAL, NS>(a, grid, st);
    if (s.nw == 4) return launch_bf16_shape<D, 4, 1, CAUSAL, NS>(a, grid, st);
    return launch_bf16_shape<D, 2, 1, CAUSAL, NS>(a, grid, st);
}

// fp32 kernel: a ring of two 32-key tiles of K and V (64 KB at D = 128, no attribute needed).
template <int D, bool CAUSAL>
tlin_status launch_f32(const AttnArgs &a, Shape s, int grid, hipStream_t st)
{
    constexpr int lds_bytes = 2 * 2 * 32 * D * 4;    // the two-wave shape keeps one tile: half of it
    static_assert(lds_bytes <= 64 * 1024, "fp32 tile ring must fit the default dynamic LDS limit");
    if (s.nw == 8) return launch_kernel((const void *)attn_f32_kernel<D, 8, CAUSAL>, dim3(grid), dim3(512), lds_bytes, st, a);
    if (s.nw == 4) return launch_kernel((const void *)attn_f32_kernel<D, 4, CAUSAL>, dim3(grid), dim3(256), lds_bytes, st, a);
    return launch_kernel((const void *)attn_f32_kernel<D, 2, CAUSAL>, dim3(grid), dim3(128), lds_bytes / 2, st, a);
}

// Window blocks launched behind the history blocks run when the compute units are already taken, as
// a tail of their own (1.5 to 5 % of the larger workloads' kernel time).  Where the partitions are
// long enough to absorb it, partition 0's workgroup computes the window block too and gets that
// much less history (partition_tiles): every partition stays non-empty when the tiles number at
// least nsplit^2 and a partition is at least four such blocks long.  BM, BN, quarters: the kernel's
// query rows per workgroup, keys per tile and cost ratio (window_block_cost).
bool fuses_window(const PairArgs &f, int BM, int BN, int quarters)
{
    const int tiles = (f.hist.NK + BN - 1) / BN, ns = f.hist.nsplit;
    const int cost = window_block_cost(f.hist.W, f.hist.nqb - 1, BM, BN, quarters);
    return f.hist.nchunks == 0 && f.n_win_blocks > 0 && ns >= 2 && tiles >= ns * ns && tiles / ns >= 4 * cost;
}

template <int D>
tlin_status launch_f32_pair(const PairArgs &f, Shape s, hipStream_t st)
{
    constexpr int lds_bytes = 2 * 2 * 32 * D * 4;
    PairArgs g = f;
    if (fuses_window(f, s.nw * 32, 32, 4)) {
        g.hist.fuse_window = 1;
        g.n_win_blocks = 0;
    }
    const dim3 grid(g.n_hist_blocks + g.n_win_blocks);
    if (s.nw == 8) return launch_kernel((const void *)attn_f32_pair_kernel<D, 8>, grid, dim3(512), lds_bytes, st, g);
    if (s.nw == 4) return launch_kernel((const void *)attn_f32_pair_kernel<D, 4>, grid, dim3(256), lds_bytes, st, g);
    return launch_kernel((const void *)attn_f32_pair_kernel<D, 2>, grid, dim3(128), lds_bytes / 2, st, g);
}

// Key tiles the resident variant keeps in LDS (128 KB of keys and values).
int resident_tiles(int D) { return D == 128 ? 4 : 8; }

// The resident variant pays when the key/value side fits in LDS as a whole and every workgroup
// has several query blocks to walk over: long query side, short unsplit key side.
bool use_resident(const tlin_params *p, bool causal, const AttnArgs &a)
{
    if (causal || p->in_dtype != TLIN_BF16 || !a.direct || a.nsplit != 1) return false;
    if (p->W <= 128) return false;
    const int ntiles = (a.NK + 63) / 64;
    const int64_t blocks = (int64_t)p->B * p->H * ((p->W + 255) / 256);      // the resident kernels are eight-wave ones
    return ntiles <= resident_tiles(dpad(p->D)) && blocks >= 4 * (int64_t)kNumCU;
}

// K/V rows of a history are read by exactly one workgroup when the window is a single query block,
// and stream through the caches without reuse when they exceed the last-level cache (256 MB)
// several times over: then the tile loads carry the non-temporal hint.  Not for the sliding
// schedule, whose chunks re-read each other's history.
bool streams_once(const tlin_params *p, const AttnArgs &a, int nqb)
{
    const int64_t kv_bytes = 2 * (int64_t)p->B * p->H * a.NK * p->D * 2;
    return p->in_dtype == TLIN_BF16 && nqb == 1 && a.nchunks == 0 && kv_bytes >= ((int64_t)192 << 20);
}

// Launch one partial-attention kernel over `nsplit` key partitions (or the causal window).
tlin_status launch_attn(const tlin_params *p, bool causal, AttnArgs a, hipStream_t st)
{
    const int qblk = query_block(p->in_dtype, p->W, p->D);
    a.nqb = (p->W + qblk - 1) / qblk;
    a.stream_once = !causal && streams_once(p, a, a.nqb);
    if (use_resident(p, causal, a)) {
        // one workgroup per compute unit, spread evenly over the heads
        a.nqb = (p->W + 255) / 256;
        const int64_t bh = (int64_t)p->B * p->H;
        int64_t g = (kNumCU + bh - 1) / bh;
        if (g > a.nqb) g = a.nqb;
        a.q_groups = (int)g;
        const int64_t grid64 = bh * g;
        if (grid64 > 0x7fffffff) return TLIN_ERR_INVALID_ARG;
        LaunchTimer timer(KC_HISTORY, st);
        // an even number of key tiles at head dimension 128: the pipelined variant
        const int ntiles = (a.NK + 63) / 64;
        if (dpad(p->D) == 128 && ntiles == 4) return launch_resident_pipe<128, 4, 4>(a, (int)grid64, st);
        if (dpad(p->D) == 128 && ntiles == 2) return launch_resident_pipe<128, 2, 4>(a, (int)grid64, st);
        return dpad(p->D) == 128 ? launch_bf16_shape<128, 8, 1, false, 4, true>(a, (int)grid64, st)
                                 : launch_bf16_shape<64, 8, 1, false, 8, true>(a, (int)grid64, st);
    }
    const int64_t grid64 = (int64_t)p->B * p->H * a.nqb * a.nsplit * (a.nchunks ? a.nchunks : 1);
    if (grid64 > 0x7fffffff) return TLIN_ERR_INVALID_ARG;
    const int grid = (int)grid64;
    LaunchTimer timer(causal ? KC_WINDOW : KC_HISTORY, st);
    const Shape s = kernel_shape(p->in_dtype, p->W, p->D);
    if (p->in_dtype == TLIN_BF16) {
        if (dpad(p->D) == 128) return causal ? launch_bf16<128, true>(a, s, grid, st) : launch_bf16<128, false>(a, s, grid, st);
        return causal ? launch_bf16<64, true>(a, s, grid, st) : launch_bf16<64, false>(a, s, grid, st);
    }
    if (dpad(p->D) == 128) return causal ? launch_f32<128, true>(a, s, grid, st) : launch_f32<128, false>(a, s, grid, st);
    return causal ? launch_f32<64, true>(a, s, grid, st) : launch_f32<64, false>(a, s, grid, st);
}

template <typename T, int DK, bool PAD>
const void *decode_kernel_for(int W)
{
    return W == 1 ? (const void *)decode_kernel<T, DK, 1, PAD> : W == 2 ? (const void *)decode_kernel<T, DK, 2, PAD>
         : W <= 4 ? (const void *)decode_kernel<T, DK, 4, PAD> : (const void *)decode_kernel<T, DK, 8, PAD>;
}
const void *decode_kernel_f32(int W, int D)
{
    if (dpad(D) == 128) return D == 128 ? decode_kernel_for<float, 128, false>(W) : decode_kernel_for<float, 128, true>(W);
    return D == 64 ? decode_kernel_for<float, 64, false>(W) : decode_kernel_for<float, 64, true>(W);
}

tlin_status launch_decode(const tlin_params *p, const AttnArgs &a, hipStream_t st)
{
    const int64_t grid64 = (int64_t)p->B * p->H * a.nsplit;
    if (grid64 > 0x7fffffff || p->W > decode_max_rows(p)) return TLIN_ERR_INVALID_ARG;
    LaunchTimer timer(KC_HISTORY, st);
    const void *kernel = p->in_dtype == TLIN_F32 ? decode_kernel_f32(p->W, p->D)
                       : p->W == 1             ? (const void *)decode_kernel<__bf16, 128, 1, false>
                                               : (const void *)decode_kernel<__bf16, 128, 2, false>;
    return launch_kernel(kernel, dim3((unsigned)grid64), dim3(256), 0, st, a);
}

tlin_status launch_merge(const tlin_params *p, MergeArgs m, hipStream_t st)
{
    m.H = p->H;
    m.W = p->W;
    m.out_bf16 = p->out_dtype == TLIN_BF16;
    m.D = p->D;
    const int64_t total = (int64_t)p->B * p->H * (m.nchunks ? m.seq_rows : p->W);
    if (total > 0x7fffffff) return TLIN_ERR_INVALID_ARG;
    m.total_rows = (int)total;
    // threads per (row, 4 columns) item: more when a row has many partials to walk
    const int joint = m.nhist + (m.has_window && m.joint ? 1 : 0);
    const int sl = joint > 16 ? 8 : joint > 6 ? 4 : 1;
    const int rpb = 256 / (dpad(p->D) / 4 * sl);
    const int grid = (int)((total + rpb - 1) / rpb);
    LaunchTimer timer(KC_MERGE, st);
    const void *kernel;
    if (dpad(p->D) == 128) kernel = sl == 8 ? (const void *)merge_kernel<128, 8> : sl == 4 ? (const void *)merge_kernel<128, 4> : (const void *)merge_kernel<128, 1>;
    else kernel = sl == 8 ? (const void *)merge_kernel<64, 8> : sl == 4 ? (const void *)merge_kernel<64, 4> : (const void *)merge_kernel<64, 1>;
    return launch_kernel(kernel, dim3(grid), dim3(256), 0, st, m);
}

AttnArgs base_args(const tlin_params *p, const void *Q, const void *K, const void *V, const int64_t ks[3],
                   const int64_t vs[3], int nk)
{
    AttnArgs a = {};
    a.Q = Q; a.K = K; a.V = V;
    const Strides q = resolve(p->q_stride, p->H, p->W, p->D);
    const Strides k = resolve(ks, p->H, nk, p->D);
    const Strides v = resolve(vs, p->H, nk, p->D);
    a.q_sb = q.b; a.q_sh = q.h; a.q_sr = q.r;
    a.k_sb = k.b; a.k_sh = k.h; a.k_sr = k.r;
    a.v_sb = v.b; a.v_sh = v.h; a.v_sr = v.r;
    a.H = p->H; a.W = p->W; a.NK = nk;
    a.D = p->D;
    a.nsplit = 1; a.tiles_per_split = 0x3fffffff;
    a.scale = p->scale;
    a.c = p->scale * 1.4426950408889634f;
    return a;
}

void set_direct(AttnArgs &a, const tlin_params *p, void *O, float *lse)
{
    const Strides o = resolve(p->o_stride, p->H, p->W, p->D);
    a.direct = 1;
    a.O = O; a.o_sb = o.b; a.o_sh = o.h; a.o_sr = o.r;
    a.lse = lse;
    a.out_bf16 = p->out_dtype == TLIN_BF16;
}

void set_partial(AttnArgs &a, const Workspace &w, int nparts, int part0)
{
    a.direct = 0;
    a.Opart = w.O; a.Mpart = w.M; a.Lpart = w.L;
    a.nparts = nparts; a.part0 = part0;
}

MergeArgs merge_args(const tlin_params *p, const Workspace &w, int nparts, int nhist, bool has_window, bool joint,
                     void *O, float *lse)
{
    MergeArgs m = {};
    m.Opart = w.O; m.Mpart = w.M; m.Lpart = w.L;
    m.nparts = nparts; m.nhist = nhist; m.has_window = has_window; m.joint = joint;
    const Strides o = resolve(p->o_stride, p->H, p->W, p->D);
    m.O = O; m.o_sb = o.b; m.o_sh = o.h; m.o_sr = o.r;
    m.lse = lse;
    return m;
}

template <int D, int NW, int NSTAGE, bool PAD, bool NT>
tlin_status launch_pair_kernel(const PairArgs &f, hipStream_t st)
{
    constexpr int lds_bytes = 2 * NSTAGE * 64 * D * 2;
    static_assert(lds_bytes <= 160 * 1024, "LDS ring exceeds the 160 KB of a gfx950 compute unit");
    auto kernel = attn_bf16_pair_kernel<D, NW, NSTAGE, PAD, NT>;
    static std::atomic<uint64_t> lds_allowed{0};
    if (allow_lds((const void *)kernel, lds_bytes, lds_allowed) != TLIN_OK) return TLIN_ERR_HIP;
    if constexpr (use_pipe_body<D, NW, 1, false, NSTAGE, false>()) {
        if (fuses_window(f, NW * 32, 64, 5)) {
            PairArgs g = f;
            g.hist.fuse_window = 1;
            g.n_win_blocks = 0;
            return launch_kernel((const void *)kernel, dim3(g.n_hist_blocks), dim3(NW * 64), lds_bytes, st, g);
        }
    }
    return launch_kernel((const void *)kernel, dim3(f.n_hist_blocks + f.n_win_blocks), dim3(NW * 64), lds_bytes, st, f);
}

template <int D, int NW, int NSTAGE, bool PAD>
tlin_status launch_pair_shape_pad(const PairArgs &f, hipStream_t st)
{
    if constexpr (use_pipe_body<D, NW, 1, false, NSTAGE, false>()) {
        if (f.hist.stream_once) return launch_pair_kernel<D, NW, NSTAGE, PAD, true>(f, st);
    }
    return launch_pair_kernel<D, NW, NSTAGE, PAD, false>(f, st);
}

template <int D, int NW, int NSTAGE>
tlin_status launch_pair_shape(const PairArgs &f, hipStream_t st)
{
    if (f.hist.D != D) return launch_pair_shape_pad<D, NW, NSTAGE, true>(f, st);
    return launch_pair_shape_pad<D, NW, NSTAGE, false>(f, st);
}

// History partials and window partial of the same rows: one launch for both problem sets.
tlin_status launch_partials(const tlin_params *p, const AttnArgs &ah, const AttnArgs &aw, hipStream_t hs)
{
    const int qblk = query_block(p->in_dtype, p->W, p->D);
    const int nqb = (p->W + qblk - 1) / qblk;
    const int64_t per_set = (int64_t)p->B * p->H * nqb * (ah.nchunks ? ah.nchunks : 1);
    const int64_t nh = per_set * ah.nsplit, nw = per_set;
    if (nh + nw <= 0x7fffffff) {
        PairArgs f = {};
        f.hist = ah;
        f.win = aw;
        f.hist.nqb = f.win.nqb = nqb;
        f.hist.stream_once = streams_once(p, ah, nqb);
        f.n_hist_blocks = (int)nh;
        f.n_win_blocks = (int)nw;
        const Shape s = kernel_shape(p->in_dtype, p->W, p->D);
        LaunchTimer timer(KC_HISTORY, hs);
        if (p->in_dtype == TLIN_F32) return dpad(p->D) == 128 ? launch_f32_pair<128>(f, s, hs) : launch_f32_pair<64>(f, s, hs);
        if (dpad(p->D) == 128) {
            if (s.nw == 8) return launch_pair_shape<128, 8, 2>(f, hs);
            if (s.nw == 4) return launch_pair_shape<128, 4, 2>(f, hs);
            return launch_pair_shape<128, 2, 2>(f, hs);
        }
        if (s.nw == 8) return launch_pair_shape<64, 8, 2>(f, hs);
        if (s.nw == 4) return launch_pair_shape<64, 4, 2>(f, hs);
        return launch_pair_shape<64, 2, 3>(f, hs);
    }
    tlin_status st;
    if ((st = launch_attn(p, false, ah, hs))) return st;
    return launch_attn(p, true, aw, hs);
}

tlin_status check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return TLIN_OK;
    if (!ws || !aligned(ws, 256) || have < need) return TLIN_ERR_WORKSPACE;
    return TLIN_OK;
}

// Argument checks of the layer call (host only).
tlin_status check_layer_args(const tlin_params *p, const void *Q_win, const void *K_hist, const void *V_hist,
                             const void *K_win, const void *V_win, const void *O)
{
    tlin_status st = check_common(p, true, true);
    if (st) return st;
    if ((st = check_dense_rows(p, T_Q | T_KW | T_VW | T_O | (p->N > 0 ? T_KH | T_VH : 0)))) return st;
    if (p->combine != TLIN_COMBINE_SUM && p->combine != TLIN_COMBINE_JOINT) return TLIN_ERR_INVALID_ARG;
    if (!Q_win || !K_win || !V_win || !O) return TLIN_ERR_INVALID_ARG;
    if (p->N > 0 && (!K_hist || !V_hist)) return TLIN_ERR_INVALID_ARG;
    if (!aligned(Q_win, 16) || !aligned(K_win, 16) || !aligned(V_win, 16) || !aligned(O, 16)) return TLIN_ERR_INVALID_ARG;
    if (p->N > 0 && (!aligned(K_hist, 16) || !aligned(V_hist, 16))) return TLIN_ERR_INVALID_ARG;
    return TLIN_OK;
}

// The launches of a layer call; arguments and workspace have been checked.
tlin_status layer_attn(const tlin_params *p, const void *Q_win, const void *K_hist, const void *V_hist,
                       const void *K_win, const void *V_win, void *O, void *ws, hipStream_t hs)
{
    if (p->N == 0) {
        // Empty history: the layer is the window causal attention in both combine modes.
        AttnArgs a = base_args(p, Q_win, K_win, V_win, p->kw_stride, p->vw_stride, p->W);
        set_direct(a, p, O, nullptr);
        return launch_attn(p, true, a, hs);
    }
    const Plan pl = plan_history(p);
    const int nparts = pl.nsplit + 1;
    const Workspace w = carve(ws, p, nparts);

    AttnArgs ah = base_args(p, Q_win, K_hist, V_hist, p->kh_stride, p->vh_stride, p->N);
    ah.nsplit = pl.nsplit;
    ah.tiles_per_split = pl.tiles_per_split;
    set_partial(ah, w, nparts, 0);
    AttnArgs aw = base_args(p, Q_win, K_win, V_win, p->kw_stride, p->vw_stride, p->W);
    set_partial(aw, w, nparts, pl.nsplit);
    tlin_status st;
    if ((st = launch_partials(p, ah, aw, hs))) return st;
    return launch_merge(p, merge_args(p, w, nparts, pl.nsplit, true, p->combine == TLIN_COMBINE_JOINT, O, nullptr), hs);
}

// Address of this device's copy of `scratch`, looked up once per device ordinal with that device
// current (every GPU holds its own copy of the array at its own address).
tlin_status static_scratch(void **out)
{
    static std::mutex mu;
    static void *addr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TLIN_ERR_HIP;
    std::lock_guard<std::mutex> lk(mu);
    if (!addr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TLIN_ERR_HIP;
        addr[dev] = ptr;
    }
    *out = addr[dev];
    return TLIN_OK;
}

}  // namespace

extern "C" {

size_t tlin_workspace_bytes(const tlin_params *p)
{
    if (check_common(p, true, true) != TLIN_OK) return 0;
    const Plan pl = plan_history(p);
    size_t need = ws_bytes_for(p, pl.nsplit + 1);
    if (use_decode(p)) {
        const size_t dec = ws_bytes_for(p, plan_decode(p).nsplit);
        if (dec > need) need = dec;
    }
    return need;
}

int32_t tlin_num_splits(const tlin_params *p)
{
    if (check_common(p, true, false) != TLIN_OK) return 0;
    return use_decode(p) ? plan_decode(p).nsplit : plan_history(p).nsplit;
}

tlin_status tlin_history_attn(const tlin_params *p, const void *Q_win, const void *K_hist, const void *V_hist,
                              void *O, float *lse, void *ws, size_t ws_bytes, void *stream)
{
    tlin_status st = check_common(p, true, false);
    if (st) return st;
    if ((st = check_dense_rows(p, T_Q | T_KH | T_VH | T_O))) return st;
    if (!Q_win || !K_hist || !V_hist || !O) return TLIN_ERR_INVALID_ARG;
    if (!aligned(Q_win, 16) || !aligned(K_hist, 16) || !aligned(V_hist, 16) || !aligned(O, 16)) return TLIN_ERR_INVALID_ARG;
    if (lse && !aligned(lse, 4)) return TLIN_ERR_INVALID_ARG;
    hipStream_t hs = (hipStream_t)stream;
    AttnArgs a = base_args(p, Q_win, K_hist, V_hist, p->kh_stride, p->vh_stride, p->N);
    if (use_decode(p)) {
        const Plan pd = plan_decode(p);
        if ((st = check_ws(ws, ws_bytes, ws_bytes_for(p, pd.nsplit)))) return st;
        if ((st = check_device())) return st;
        const Workspace w = carve(ws, p, pd.nsplit);
        a.nsplit = pd.nsplit;
        a.tiles_per_split = pd.tiles_per_split;
        set_partial(a, w, pd.nsplit, 0);
        if ((st = launch_decode(p, a, hs))) return st;
        return launch_merge(p, merge_args(p, w, pd.nsplit, pd.nsplit, false, true, O, lse), hs);
    }
    const Plan pl = plan_history(p);
    a.nsplit = pl.nsplit;
    a.tiles_per_split = pl.tiles_per_split;
    if (pl.nsplit == 1) {
        if ((st = check_device())) return st;
        set_direct(a, p, O, lse);
        return launch_attn(p, false, a, hs);
    }
    if ((st = check_ws(ws, ws_bytes, ws_bytes_for(p, pl.nsplit)))) return st;
    if ((st = check_device())) return st;
    const Workspace w = carve(ws, p, pl.nsplit);
    set_partial(a, w, pl.nsplit, 0);
    if ((st = launch_attn(p, false, a, hs))) return st;
    return launch_merge(p, merge_args(p, w, pl.nsplit, pl.nsplit, false, true, O, lse), hs);
}

tlin_status tlin_window_causal_attn(const tlin_params *p, const void *Q_win, const void *K_win, const void *V_win,
                                    void *O, float *lse, void *ws, size_t ws_bytes, void *stream)
{
    (void)ws;
    (void)ws_bytes;
    tlin_status st = check_common(p, false, false);
    if (st) return st;
    if ((st = check_dense_rows(p, T_Q | T_KW | T_VW | T_O))) return st;
    if (!Q_win || !K_win || !V_win || !O) return TLIN_ERR_INVALID_ARG;
    if (!aligned(Q_win, 16) || !aligned(K_win, 16) || !aligned(V_win, 16) || !aligned(O, 16)) return TLIN_ERR_INVALID_ARG;
    if (lse && !aligned(lse, 4)) return TLIN_ERR_INVALID_ARG;
    if ((st = check_device())) return st;
    AttnArgs a = base_args(p, Q_win, K_win, V_win, p->kw_stride, p->vw_stride, p->W);
    set_direct(a, p, O, lse);
    return launch_attn(p, true, a, (hipStream_t)stream);
}

tlin_status tlin_layer_attn(const tlin_params *p, const void *Q_win, const void *K_hist, const void *V_hist,
                            const void *K_win, const void *V_win, void *O, void *ws, size_t ws_bytes, void *stream)
{
    tlin_status st = check_layer_args(p, Q_win, K_hist, V_hist, K_win, V_win, O);
    if (st) return st;
    if (p->N > 0 && (st = check_ws(ws, ws_bytes, ws_bytes_for(p, plan_history(p).nsplit + 1)))) return st;
    if ((st = check_device())) return st;
    return layer_attn(p, Q_win, K_hist, V_hist, K_win, V_win, O, ws, (hipStream_t)stream);
}

tlin_status tlin_layer_attn_static_ws(const tlin_params *p, const void *Q_win, const void *K_hist, const void *V_hist,
                                      const void *K_win, const void *V_win, void *O, void *stream)
{
    tlin_status st = check_layer_args(p, Q_win, K_hist, V_hist, K_win, V_win, O);
    if (st) return st;
    const size_t need = p->N > 0 ? ws_bytes_for(p, plan_history(p).nsplit + 1) : 0;
    if (need > TLIN_STATIC_WS_BYTES) return TLIN_ERR_WORKSPACE;
    if ((st = check_device())) return st;
    void *ws = nullptr;
    if (need > 0 && (st = static_scratch(&ws))) return st;
    return layer_attn(p, Q_win, K_hist, V_hist, K_win, V_win, O, ws, (hipStream_t)stream);
}

size_t tlin_slide_workspace_bytes(const tlin_params *p)
{
    if (check_common(p, true, false) != TLIN_OK) return 0;
    const SlidePlan pl = plan_slide(p);
    return slide_ws_bytes(p, pl);
}

tlin_status tlin_slide_layer_attn(const tlin_params *p, const void *Q, const void *K_hist, const void *V_hist,
                                  const void *K_win, const void *V_win, void *O, void *ws, size_t ws_bytes,
                                  void *stream)
{
    tlin_status st = check_common(p, true, false);
    if (st) return st;
    if ((st = check_dense_rows(p, T_Q | T_KH | T_VH | T_KW | T_VW | T_O))) return st;
    if (p->combine != TLIN_COMBINE_SUM && p->combine != TLIN_COMBINE_JOINT) return TLIN_ERR_INVALID_ARG;
    if (!Q || !K_hist || !V_hist || !K_win || !V_win || !O) return TLIN_ERR_INVALID_ARG;
    if (!aligned(Q, 16) || !aligned(K_hist, 16) || !aligned(V_hist, 16) || !aligned(K_win, 16) || !aligned(V_win, 16) ||
        !aligned(O, 16))
        return TLIN_ERR_INVALID_ARG;
    hipStream_t hs = (hipStream_t)stream;
    const SlidePlan pl = plan_slide(p);
    if ((int64_t)p->B * p->H * pl.nchunks * pl.nparts > 0x7fffffff) return TLIN_ERR_INVALID_ARG;
    if ((st = check_ws(ws, ws_bytes, slide_ws_bytes(p, pl)))) return st;
    if ((st = check_device())) return st;
    // partial slots: (b*H + h, chunk, part), W rows each
    const size_t rows = (size_t)p->B * p->H * pl.nchunks * pl.nparts * p->W;
    float *base = (float *)ws;
    const Workspace w = {base, base + rows * dpad(p->D), base + rows * dpad(p->D) + rows};

    // every tensor has p->N rows per head
    const Strides q = resolve(p->q_stride, p->H, p->N, p->D);
    const Strides o = resolve(p->o_stride, p->H, p->N, p->D);
    auto args = [&](const void *K, const void *V, const int64_t ks[3], const int64_t vs[3]) {
        AttnArgs a = base_args(p, Q, K, V, ks, vs, p->N);
        a.q_sb = q.b; a.q_sh = q.h; a.q_sr = q.r;
        a.nchunks = pl.nchunks;
        a.seq_rows = p->N;
        return a;
    };
    AttnArgs ah = args(K_hist, V_hist, p->kh_stride, p->vh_stride);
    ah.nsplit = pl.nsplit;
    set_partial(ah, w, pl.nparts, 0);
    AttnArgs aw = args(K_win, V_win, p->kw_stride, p->vw_stride);
    set_partial(aw, w, pl.nparts, pl.nsplit);
    if (pl.nchunks > 1) {
        if ((st = launch_partials(p, ah, aw, hs))) return st;
    } else if ((st = launch_attn(p, true, aw, hs))) {
        return st;
    }

    MergeArgs m = merge_args(p, w, pl.nparts, pl.nsplit, true, p->combine == TLIN_COMBINE_JOINT, O, nullptr);
    m.o_sb = o.b; m.o_sh = o.h; m.o_sr = o.r;
    m.nchunks = pl.nchunks;
    m.seq_rows = p->N;
    return launch_merge(p, m, hs);
}

tlin_status tlin_profile_stream_read(const void *buf, size_t bytes, int32_t nontemporal, void *stream)
{
    if (!buf || !aligned(buf, 16) || bytes < ((size_t)1 << 20)) return TLIN_ERR_INVALID_ARG;
    tlin_status st = check_device();
    if (st) return st;
    const int blocks = 8 * kNumCU;
    const StreamReadArgs a = {buf, bytes / 16 / blocks};
    const void *kernel = nontemporal ? (const void *)stream_read_kernel<true> : (const void *)stream_read_kernel<false>;
    return launch_kernel(kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, a);
}

tlin_status tlin_profile_enable(int32_t enable)
{
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.on = enable != 0;
    return TLIN_OK;
}

tlin_status tlin_profile_read(double ms[3], int64_t launches[3])
{
    if (!ms || !launches) return TLIN_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (int i = 0; i < KC_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
    tlin_status rc = TLIN_OK;
    for (const Timed &t : g_prof.used) {
        float e = 0.f;
        if (hipEventSynchronize(t.stop) != hipSuccess || hipEventElapsedTime(&e, t.start, t.stop) != hipSuccess) {
            rc = TLIN_ERR_HIP;
        } else {
            ms[t.cls] += e;
            launches[t.cls] += 1;
        }
        g_prof.pool.push_back({t.start, t.stop});
    }
    g_prof.used.clear();
    return rc;
}

const char *tlin_status_string(int status)
{
    switch (status) {
    case TLIN_OK: return "ok";
    case TLIN_ERR_INVALID_ARG: return "invalid argument";
    case TLIN_ERR_UNSUPPORTED: return "unsupported head dimension or dtype";
    case TLIN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case TLIN_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int32_t tlin_version(void) { return kVersion; }

}  // extern "C"
