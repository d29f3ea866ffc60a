/*
 * libtlinattn - TLinFormer's window-over-history attention for AMD MI355X (gfx950).
 *
 * The paper (arXiv 2508.20407) builds its linear-cost connectivity out of one primitive,
 *
 *     Attention(Q, K, V) = softmax(Q K^T / sqrt(d_k)) V              (Section 3)
 *
 * applied with different sources for Q and K/V.  The only terms of its cost model that grow
 * with the sequence length (Section 4.1, Appendix A: the D*N*W terms) are attentions in which a
 * bounded window of W query rows attends an N-row history, and every generation-path layer
 * also runs causal attention inside the window.  This library is exactly those operations:
 *
 *   tlin_history_attn        W window queries x N history keys/values, no mask
 *                            (Focused attention and the first-layer Cross attention, Section 3)
 *   tlin_window_causal_attn  causal attention inside the window, query i sees keys j <= i
 *                            (Causal attention / "Internal Cohesion", Section 3)
 *   tlin_layer_attn          both for the same W rows, combined (Section 3, generation path)
 *   tlin_slide_layer_attn    tlin_layer_attn for every chunk of a sequence at once, each chunk's
 *                            history being all earlier chunks (training schedule, Section 5.1)
 *
 * Conventions common to all entry points
 *   - All tensor pointers and the workspace are DEVICE pointers owned by the caller.  The
 *     library never allocates, frees or keeps them.  Inputs are read-only; O must not alias
 *     an input.  Layout is [B, H, rows, D] with D contiguous; batch/head/row strides are given
 *     in elements (0 in every slot of a stride triple = dense).  Rows are read and written in
 *     16-byte pieces: every stride must be a multiple of 16 bytes, and a row must own D elements
 *     rounded up to whole pieces (so bf16 with D = 36 needs a row stride of at least 40, and a
 *     dense layout needs D itself to be whole pieces).  What the inputs hold between D and the end
 *     of the last piece is ignored; in O those elements are left untouched.
 *   - Calls enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and return without synchronising.  Calls using the same workspace must be ordered on
 *     one stream.  Nothing else is enqueued (no copies, no memsets), so a call can be captured
 *     into a HIP graph once the same call shape has run once outside a capture on that device
 *     (the first launch of a kernel raises its LDS limit, which is not a stream operation).
 *   - Errors are reported by return code only.  Argument validation runs on the host before
 *     any HIP call, so it behaves the same on a machine without a GPU.
 *   - Each (b, h) is an independent attention problem; there is no positional term, bias,
 *     dropout or key/value head sharing.  Non-finite inputs give unspecified outputs.
 *   - Results are exact softmax attention up to rounding: bf16 inputs are multiplied with fp32
 *     accumulation (on the matrix cores; with the dot-product instructions of the vector unit
 *     where one or two query rows meet a long history), softmax weights are rounded to bf16
 *     before the second product; fp32 inputs use fp32 arithmetic throughout (fp32 matrix
 *     instructions, or fp32 multiply-adds of the vector unit for up to eight query rows over a
 *     long history; nothing is rounded below fp32).
 *   - Accuracy envelope.  bf16 inputs: |O - exact| <= 2e-2 (mean <= 5e-3) for inputs of unit
 *     scale.  fp32 inputs: a logit is an fp32 sum of D products and carries an absolute error of
 *     a few 2^-24 of its own size, which the exponential turns into the same RELATIVE error of
 *     the weight; the result is within 1e-5 of the exact one, relative to max(|O|, rms(O)),
 *     while the logits scale * <q, k> stay within about 10 nats in magnitude, and within 1e-6 per
 *     nat of logit magnitude beyond that.
 */
#ifndef TLINATTN_H
#define TLINATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TLIN_OK = 0,
    TLIN_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad stride/alignment/scale */
    TLIN_ERR_UNSUPPORTED = 2, /* head dimension or dtype combination not implemented, or the current
                                 device is not an MI355X (gfx950 with 256 compute units) */
    TLIN_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or smaller than required */
    TLIN_ERR_HIP = 4          /* a HIP runtime call or kernel launch of this call failed (errors left
                                 behind by the caller's earlier work are neither reported nor cleared) */
} tlin_status;

typedef enum { TLIN_F32 = 0, TLIN_BF16 = 1 } tlin_dtype;

/* How tlin_layer_attn joins the history result and the window result.  The paper only says
 * the two "are combined" (Section 3); both natural readings are provided.
 *   SUM   : two independent softmaxes, outputs added.
 *   JOINT : a single softmax over history keys and causally visible window keys together,
 *           i.e. rows [N, N+W) of causal attention over the concatenated sequence - the
 *           connectivity drawn in Figure 2(b). */
typedef enum { TLIN_COMBINE_SUM = 0, TLIN_COMBINE_JOINT = 1 } tlin_combine;

typedef struct {
    int32_t B, H;        /* batch, heads: B*H independent problems, each >= 1 */
    int32_t W;           /* window (query) rows, >= 1; W and N are at most 2^30 */
    int32_t N;           /* history rows; >= 1 for tlin_history_attn, >= 0 for tlin_layer_attn,
                            ignored by tlin_window_causal_attn; sequence rows (>= 1) for
                            tlin_slide_layer_attn, whose chunk length is W */
    int32_t D;           /* head dimension: a multiple of 4 in [8, 128]; 64 and 128 are the native
                            sizes, others run in the next of the two (see the layout rules) */
    int32_t in_dtype;    /* tlin_dtype of Q, K, V */
    int32_t out_dtype;   /* tlin_dtype of O */
    float scale;         /* logit multiplier, finite and > 0; 1/sqrt(D) gives the paper's formula */
    int32_t num_splits;  /* partitions of the history axis; 0 = choose automatically */
    int32_t combine;     /* tlin_combine, used by tlin_layer_attn only */
    /* element strides {batch, head, row}; all three 0 = dense.  Row strides must be >= D, keep
     * every row 16-byte aligned and stay below 32 MiB. */
    int64_t q_stride[3], kh_stride[3], vh_stride[3], kw_stride[3], vw_stride[3], o_stride[3];
} tlin_params;

/* Bytes of device workspace sufficient for any of the three calls below with these
 * parameters (split partials of the history axis plus the window partial).  Pure host
 * arithmetic.  Returns 0 if the parameters are invalid. */
size_t tlin_workspace_bytes(const tlin_params *p);

/* Number of history partitions the library will use for these parameters (>= 1), or 0 if the
 * parameters are invalid.  Pure host arithmetic. */
int32_t tlin_num_splits(const tlin_params *p);

/* O[b,h,i,:] = sum_j softmax_j(scale * <Q[b,h,i,:], K_hist[b,h,j,:]>) * V_hist[b,h,j,:],
 * j over all N history rows, no mask (Section 3: Focused / Cross attention; cost D*N*W,
 * Appendix A).  The history axis is processed in partitions that are merged exactly by
 * their log-sum-exp statistics.
 *   Q_win [B,H,W,D], K_hist/V_hist [B,H,N,D] in in_dtype; O [B,H,W,D] in out_dtype.
 *   lse: nullable, dense fp32 [B,H,W]; receives log(sum_j exp(scale * <q_i, k_j>)).
 *   ws : workspace of at least tlin_workspace_bytes(p) bytes, 256-byte aligned. */
tlin_status tlin_history_attn(const tlin_params *p, const void *Q_win, const void *K_hist,
                              const void *V_hist, void *O, float *lse, void *ws, size_t ws_bytes,
                              void *stream);

/* Causal attention inside the window: as above with keys K_win/V_win [B,H,W,D] and the
 * sum restricted to j <= i (Section 3: Causal attention, mask keeps positions j <= i; query
 * row i is aligned with key row i).  p->N is ignored. */
tlin_status tlin_window_causal_attn(const tlin_params *p, const void *Q_win, const void *K_win,
                                    const void *V_win, void *O, float *lse, void *ws,
                                    size_t ws_bytes, void *stream);

/* One generation-path attention layer (Section 3): history attention and window causal
 * attention of the same W query rows, joined per p->combine.  With N == 0 (empty history:
 * the first chunk of the sliding schedule of Section 5.1) both modes return the window
 * causal attention; K_hist/V_hist may then be NULL. */
tlin_status tlin_layer_attn(const tlin_params *p, const void *Q_win, const void *K_hist,
                            const void *V_hist, const void *K_win, const void *V_win, void *O,
                            void *ws, size_t ws_bytes, void *stream);

/* tlin_layer_attn for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels, with the split partials kept in a device array that is part of the library's code
 * object (TLIN_STATIC_WS_BYTES per GPU, held from the library's load to the end of the process).
 * The call allocates nothing; the array's address is looked up once per device, on the first call
 * made with that device current.  Parameters whose tlin_workspace_bytes(p) exceeds
 * TLIN_STATIC_WS_BYTES are rejected with TLIN_ERR_WORKSPACE before anything is launched
 * (p->num_splits can lower the need).  Every partial that is read has been written by the same
 * call, so nothing in the array needs clearing between calls; it keeps the previous call's
 * contents.  All calls on one GPU share the array: calls that overlap on one GPU (different
 * streams, or threads) race; order them on one stream. */
#define TLIN_STATIC_WS_BYTES ((size_t)64 << 20)
tlin_status tlin_layer_attn_static_ws(const tlin_params *p, const void *Q_win, const void *K_hist,
                                      const void *V_hist, const void *K_win, const void *V_win,
                                      void *O, void *stream);

/* The sliding schedule of Section 5.1 over a whole sequence in one call: the sequence of
 * p->N rows is cut into chunks of p->W rows (the last one may be shorter); chunk c is a window
 * whose history is every earlier chunk, so row c*W + i attends rows [0, c*W) of K_hist/V_hist
 * without a mask and rows [c*W, c*W + i] of K_win/V_win causally, joined per p->combine.
 * Chunk 0 has an empty history.  Equivalent to one tlin_layer_attn call per chunk; done as
 * a few launches for all chunks together, the longest histories scheduled first.
 *   Q, K_hist, V_hist, K_win, V_win: [B,H,N,D] in in_dtype; O [B,H,N,D] in out_dtype.
 *   K_hist/V_hist may be the same buffers as K_win/V_win (one projection for both roles).
 *   p->num_splits: partitions per chunk history; 0 = choose automatically.
 *   ws: at least tlin_slide_workspace_bytes(p) bytes, 256-byte aligned (two or more fp32
 *       partials per output row: size it before choosing very long sequences).
 * tlin_slide_workspace_bytes returns 0 for invalid parameters. */
size_t tlin_slide_workspace_bytes(const tlin_params *p);
tlin_status tlin_slide_layer_attn(const tlin_params *p, const void *Q, const void *K_hist,
                                  const void *V_hist, const void *K_win, const void *V_win, void *O,
                                  void *ws, size_t ws_bytes, void *stream);

/* Text for a tlin_status value; any other integer gives "unknown status". */
const char *tlin_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t tlin_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TLINATTN_H */
