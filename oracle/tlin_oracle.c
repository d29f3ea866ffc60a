/*
 * CPU oracle for TLinFormer's window-over-history attention.  TEST INFRASTRUCTURE ONLY:
 * nothing on the product path may call, link or import this file.  It shares no code with
 * the GPU library.
 *
 * Everything is evaluated from the definition, in fp64, one query row at a time, with the
 * whole row of logits materialised and a two-pass softmax (maximum first, then the sum).
 * Inputs are fp32 or bf16 values widened exactly to fp64.
 *
 *   Attention(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V            (Section 3, displayed formula;
 *                                                               the caller passes the scale)
 *   history : row i of the window attends every history row j in [0,N), no mask
 *             (Focused / Cross attention of Section 3: the key/value set is the whole
 *             sequence, the query set a bounded window)
 *   window  : causal attention, row i attends window rows j <= i   (Section 3, Causal)
 *   layer   : the two results for the same window rows "are combined" (Section 3, generation
 *             path).  The operator is not given; two readings are implemented:
 *               SUM   - two separate softmaxes, outputs added
 *               JOINT - one softmax over history keys and causally visible window keys
 *                       together (Figure 2(b): a generation node has full edges from all
 *                       history inputs and causal edges from the window inputs)
 *
 * Pins (tests/test_oracle_pins.py): library scaled-dot-product attention in fp64 for all
 * three patterns (JOINT = rows [N,N+W) of causal attention over the concatenation), closed
 * forms (two-key sigmoid, rational-weight worked example, Q=0 mean, N=1, constant V),
 * invariances (key shift, joint row permutation), log-sum-exp against a library routine.
 * The choice of SUM as the combine operator is parity unpinned beyond "sum of two pinned
 * parts".  The sliding schedule (slide) is pinned by: JOINT with Kh = Kw, Vh = Vw is plain causal
 * attention over the whole sequence (library routine); SUM is the sum of a library unmasked
 * attention over the earlier chunks and a library causal attention inside the chunk.
 *
 * Layout: dense [B,H,rows,D], D contiguous.  `rows` (nullable) selects query rows: when
 * given, only those rows are computed for every (b,h) and the outputs have nrows rows.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_SUM = 0, ORC_JOINT = 1 };

static inline double widen(const void *p, int dtype, size_t i)
{
    if (dtype == ORC_F32) return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* logits s[j] = scale * <q, K[j,:]> for j in [0,n) */
static void logits(const double *q, const void *K, int dtype, size_t kbase, int n, int D,
                   double scale, double *s)
{
    for (int j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int k = 0; k < D; ++k) acc += q[k] * widen(K, dtype, kbase + (size_t)j * D + k);
        s[j] = scale * acc;
    }
}

static double row_max(const double *s, int n)
{
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) if (s[j] > m) m = s[j];
    return m;
}

/* o[k] += sum_j exp(s[j]-m)/z * V[j,k] */
static void weighted_values(const double *s, int n, double m, double z, const void *V, int dtype,
                            size_t vbase, int D, double *o)
{
    for (int j = 0; j < n; ++j) {
        double w = exp(s[j] - m) / z;
        for (int k = 0; k < D; ++k) o[k] += w * widen(V, dtype, vbase + (size_t)j * D + k);
    }
}

/* Softmax attention of one query over n keys; returns log-sum-exp of the logits. */
static double attend(const double *q, const void *K, const void *V, int dtype, size_t base, int n,
                     int D, double scale, double *s, double *o)
{
    logits(q, K, dtype, base, n, D, scale, s);
    double m = row_max(s, n);
    double z = 0.0;
    for (int j = 0; j < n; ++j) z += exp(s[j] - m);
    for (int k = 0; k < D; ++k) o[k] = 0.0;
    weighted_values(s, n, m, z, V, dtype, base, D, o);
    return m + log(z);
}

static int check(int B, int H, int W, int D, const int *rows, int nrows)
{
    if (B < 1 || H < 1 || W < 1 || D < 1) return -1;
    if (rows) {
        if (nrows < 0) return -1;
        for (int r = 0; r < nrows; ++r) if (rows[r] < 0 || rows[r] >= W) return -1;
    }
    return 0;
}

/* Unmasked attention of W window rows over N history rows.  O: [B,H,R,D], lse: [B,H,R]
 * (nullable), R = rows ? nrows : W.  Returns 0, -1 on bad arguments, -2 out of memory. */
int tlin_oracle_history(const void *Q, const void *Kh, const void *Vh, int dtype, int B, int H, int W,
                        int N, int D, double scale, const int *rows, int nrows, double *O, double *lse)
{
    if (check(B, H, W, D, rows, nrows) || N < 1 || !Q || !Kh || !Vh || !O) return -1;
    const int R = rows ? nrows : W;
    const long total = (long)B * H * R;
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
        double *q = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !q) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (long u = 0; u < total; ++u) {
                long bh = u / R;
                int r = (int)(u % R);
                int i = rows ? rows[r] : r;
                for (int k = 0; k < D; ++k) q[k] = widen(Q, dtype, ((size_t)bh * W + i) * D + k);
                double l = attend(q, Kh, Vh, dtype, (size_t)bh * N * D, N, D, scale, s, O + (size_t)u * D);
                if (lse) lse[u] = l;
            }
        }
        free(s);
        free(q);
    }
    return fail ? -2 : 0;
}

/* Causal attention inside the window: row i attends window rows 0..i. */
int tlin_oracle_window_causal(const void *Q, const void *Kw, const void *Vw, int dtype, int B, int H,
                              int W, int D, double scale, const int *rows, int nrows, double *O,
                              double *lse)
{
    if (check(B, H, W, D, rows, nrows) || !Q || !Kw || !Vw || !O) return -1;
    const int R = rows ? nrows : W;
    const long total = (long)B * H * R;
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)W);
        double *q = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !q) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (long u = 0; u < total; ++u) {
                long bh = u / R;
                int r = (int)(u % R);
                int i = rows ? rows[r] : r;
                for (int k = 0; k < D; ++k) q[k] = widen(Q, dtype, ((size_t)bh * W + i) * D + k);
                double l = attend(q, Kw, Vw, dtype, (size_t)bh * W * D, i + 1, D, scale, s, O + (size_t)u * D);
                if (lse) lse[u] = l;
            }
        }
        free(s);
        free(q);
    }
    return fail ? -2 : 0;
}

/* History attention and window causal attention of the same rows, combined.  N may be 0:
 * then both modes return the window causal attention alone (first chunk of the sliding
 * schedule of Section 5.1, whose history is empty). */
int tlin_oracle_layer(const void *Q, const void *Kh, const void *Vh, const void *Kw, const void *Vw,
                      int dtype, int B, int H, int W, int N, int D, double scale, int combine,
                      const int *rows, int nrows, double *O)
{
    if (check(B, H, W, D, rows, nrows) || N < 0 || !Q || !Kw || !Vw || !O) return -1;
    if (N > 0 && (!Kh || !Vh)) return -1;
    if (combine != ORC_SUM && combine != ORC_JOINT) return -1;
    const int R = rows ? nrows : W;
    const long total = (long)B * H * R;
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * ((size_t)N + (size_t)W));
        double *q = (double *)malloc(sizeof(double) * (size_t)D);
        double *t = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !q || !t) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (long u = 0; u < total; ++u) {
                long bh = u / R;
                int r = (int)(u % R);
                int i = rows ? rows[r] : r;
                double *o = O + (size_t)u * D;
                for (int k = 0; k < D; ++k) q[k] = widen(Q, dtype, ((size_t)bh * W + i) * D + k);
                if (combine == ORC_SUM) {
                    attend(q, Kw, Vw, dtype, (size_t)bh * W * D, i + 1, D, scale, s, o);
                    if (N > 0) {
                        attend(q, Kh, Vh, dtype, (size_t)bh * N * D, N, D, scale, s, t);
                        for (int k = 0; k < D; ++k) o[k] += t[k];
                    }
                } else {
                    /* one softmax over the N history logits followed by the i+1 window logits */
                    if (N > 0) logits(q, Kh, dtype, (size_t)bh * N * D, N, D, scale, s);
                    logits(q, Kw, dtype, (size_t)bh * W * D, i + 1, D, scale, s + N);
                    int n = N + i + 1;
                    double m = row_max(s, n);
                    double z = 0.0;
                    for (int j = 0; j < n; ++j) z += exp(s[j] - m);
                    for (int k = 0; k < D; ++k) o[k] = 0.0;
                    if (N > 0) weighted_values(s, N, m, z, Vh, dtype, (size_t)bh * N * D, D, o);
                    weighted_values(s + N, i + 1, m, z, Vw, dtype, (size_t)bh * W * D, D, o);
                }
            }
        }
        free(s);
        free(q);
        free(t);
    }
    return fail ? -2 : 0;
}

/* The sliding schedule of Section 5.1 over a whole sequence of L rows in one call: the sequence
 * is cut into chunks of W rows (the last one may be shorter); chunk c is a window whose history
 * is every earlier chunk, rows [0, c*W), and chunk 0 has an empty history.  Row p = c*W + i
 * therefore attends history rows [0, c*W) of Kh/Vh without a mask and window rows
 * [c*W, c*W + i] of Kw/Vw, combined as in tlin_oracle_layer.  All tensors are [B,H,L,D];
 * `rows` (nullable) selects sequence positions. */
int tlin_oracle_slide(const void *Q, const void *Kh, const void *Vh, const void *Kw, const void *Vw,
                      int dtype, int B, int H, int L, int W, int D, double scale, int combine,
                      const int *rows, int nrows, double *O)
{
    if (check(B, H, L, D, rows, nrows) || W < 1 || !Q || !Kh || !Vh || !Kw || !Vw || !O) return -1;
    if (combine != ORC_SUM && combine != ORC_JOINT) return -1;
    const int R = rows ? nrows : L;
    const long total = (long)B * H * R;
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * ((size_t)L + 1));
        double *q = (double *)malloc(sizeof(double) * (size_t)D);
        double *t = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !q || !t) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (long u = 0; u < total; ++u) {
                long bh = u / R;
                int r = (int)(u % R);
                int p = rows ? rows[r] : r;
                int N = (p / W) * W;            /* history rows of this position's chunk */
                int nw = p - N + 1;             /* visible window rows */
                size_t base = (size_t)bh * L * D;
                size_t wbase = base + (size_t)N * D;
                double *o = O + (size_t)u * D;
                for (int k = 0; k < D; ++k) q[k] = widen(Q, dtype, base + (size_t)p * D + k);
                if (combine == ORC_SUM) {
                    attend(q, Kw, Vw, dtype, wbase, nw, D, scale, s, o);
                    if (N > 0) {
                        attend(q, Kh, Vh, dtype, base, N, D, scale, s, t);
                        for (int k = 0; k < D; ++k) o[k] += t[k];
                    }
                } else {
                    if (N > 0) logits(q, Kh, dtype, base, N, D, scale, s);
                    logits(q, Kw, dtype, wbase, nw, D, scale, s + N);
                    int n = N + nw;
                    double m = row_max(s, n);
                    double z = 0.0;
                    for (int j = 0; j < n; ++j) z += exp(s[j] - m);
                    for (int k = 0; k < D; ++k) o[k] = 0.0;
                    if (N > 0) weighted_values(s, N, m, z, Vh, dtype, base, D, o);
                    weighted_values(s + N, nw, m, z, Vw, dtype, wbase, D, o);
                }
            }
        }
        free(s);
        free(q);
        free(t);
    }
    return fail ? -2 : 0;
}

int tlin_oracle_threads(void)
{
    int n = 1;
#pragma omp parallel
    {
#pragma omp single
        n =
#ifdef _OPENMP
            omp_get_num_threads();
#else
            1;
#endif
    }
    return n;
}
