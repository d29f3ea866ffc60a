/* Exercises every entry point of the CPU oracle on small shapes, row subsets, the empty history and
 * bad arguments; meant to be built together with oracle/tlin_oracle.c under AddressSanitizer and
 * UndefinedBehaviorSanitizer.  Values are checked against facts that need no second implementation
 * (rows are convex combinations: V = 1 gives 1, or 2 for the sum of two softmaxes). */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int tlin_oracle_history(const void *Q, const void *Kh, const void *Vh, int dtype, int B, int H, int W,
                        int N, int D, double scale, const int *rows, int nrows, double *O, double *lse);
int tlin_oracle_window_causal(const void *Q, const void *Kw, const void *Vw, int dtype, int B, int H,
                              int W, int D, double scale, const int *rows, int nrows, double *O, double *lse);
int tlin_oracle_layer(const void *Q, const void *Kh, const void *Vh, const void *Kw, const void *Vw,
                      int dtype, int B, int H, int W, int N, int D, double scale, int combine,
                      const int *rows, int nrows, double *O);
int tlin_oracle_slide(const void *Q, const void *Kh, const void *Vh, const void *Kw, const void *Vw,
                      int dtype, int B, int H, int L, int W, int D, double scale, int combine,
                      const int *rows, int nrows, double *O);

static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static uint32_t rng = 12345u;
static float frand(void) { rng = rng * 1664525u + 1013904223u; return (float)(rng >> 8) / (1 << 24) - 0.5f; }

/* exact-size buffers, so that any read or write past an end is caught */
static void *tensor(int dtype, size_t n, int ones)
{
    if (dtype == 0) {
        float *p = (float *)malloc(n * sizeof(float));
        for (size_t i = 0; i < n; ++i) p[i] = ones ? 1.0f : frand();
        return p;
    }
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) {
        float f = ones ? 1.0f : frand();
        uint32_t u;
        __builtin_memcpy(&u, &f, 4);
        p[i] = (uint16_t)(u >> 16);
    }
    return p;
}

static int all_near(const double *o, size_t n, double v)
{
    for (size_t i = 0; i < n; ++i) if (!(fabs(o[i] - v) < 1e-12)) return 0;
    return 1;
}

int main(void)
{
    static const int shapes[][5] = {{1, 1, 1, 1, 1}, {2, 3, 5, 7, 4}, {1, 2, 33, 65, 8}, {1, 1, 8, 1, 3}};   /* B H W N D */
    for (int dtype = 0; dtype < 2; ++dtype)
        for (unsigned si = 0; si < sizeof shapes / sizeof *shapes; ++si) {
            const int B = shapes[si][0], H = shapes[si][1], W = shapes[si][2], N = shapes[si][3], D = shapes[si][4];
            const size_t bh = (size_t)B * H;
            void *Q = tensor(dtype, bh * W * D, 0), *Kh = tensor(dtype, bh * N * D, 0), *Vh = tensor(dtype, bh * N * D, 1);
            void *Kw = tensor(dtype, bh * W * D, 0), *Vw = tensor(dtype, bh * W * D, 1);
            double *O = (double *)malloc(bh * W * D * sizeof(double)), *lse = (double *)malloc(bh * W * sizeof(double));
            CHECK(tlin_oracle_history(Q, Kh, Vh, dtype, B, H, W, N, D, 0.3, NULL, 0, O, lse) == 0 && all_near(O, bh * W * D, 1.0));
            CHECK(tlin_oracle_window_causal(Q, Kw, Vw, dtype, B, H, W, D, 0.3, NULL, 0, O, lse) == 0 && all_near(O, bh * W * D, 1.0));
            CHECK(tlin_oracle_layer(Q, Kh, Vh, Kw, Vw, dtype, B, H, W, N, D, 0.3, 0, NULL, 0, O) == 0 && all_near(O, bh * W * D, 2.0));
            CHECK(tlin_oracle_layer(Q, Kh, Vh, Kw, Vw, dtype, B, H, W, N, D, 0.3, 1, NULL, 0, O) == 0 && all_near(O, bh * W * D, 1.0));
            CHECK(tlin_oracle_layer(Q, NULL, NULL, Kw, Vw, dtype, B, H, W, 0, D, 0.3, 0, NULL, 0, O) == 0 && all_near(O, bh * W * D, 1.0));
            const int rows[2] = {W - 1, 0};                    /* a row subset, unsorted */
            const int nr = W > 1 ? 2 : 1;
            CHECK(tlin_oracle_history(Q, Kh, Vh, dtype, B, H, W, N, D, 0.3, rows, nr, O, lse) == 0 && all_near(O, bh * nr * D, 1.0));
            CHECK(tlin_oracle_layer(Q, Kh, Vh, Kw, Vw, dtype, B, H, W, N, D, 0.3, 1, rows, nr, O) == 0 && all_near(O, bh * nr * D, 1.0));
            /* the sliding schedule over the window tensors as a sequence of W rows, in chunks of 1, 3 and W + 2 */
            const int chunks[3] = {1, 3, W + 2};
            for (int ci = 0; ci < 3; ++ci) {
                const int chunk = chunks[ci];
                CHECK(tlin_oracle_slide(Q, Kw, Vw, Kw, Vw, dtype, B, H, W, chunk, D, 0.3, 1, NULL, 0, O) == 0 && all_near(O, bh * W * D, 1.0));
                CHECK(tlin_oracle_slide(Q, Kw, Vw, Kw, Vw, dtype, B, H, W, chunk, D, 0.3, 0, rows, nr, O) == 0);
            }
            const int bad[1] = {W};
            CHECK(tlin_oracle_history(Q, Kh, Vh, dtype, B, H, W, N, D, 0.3, bad, 1, O, lse) == -1);
            CHECK(tlin_oracle_history(Q, Kh, Vh, dtype, B, H, W, 0, D, 0.3, NULL, 0, O, lse) == -1);
            CHECK(tlin_oracle_layer(Q, NULL, Vh, Kw, Vw, dtype, B, H, W, N, D, 0.3, 0, NULL, 0, O) == -1);
            CHECK(tlin_oracle_slide(Q, Kw, Vw, Kw, Vw, dtype, B, H, W, 0, D, 0.3, 1, NULL, 0, O) == -1);
            free(Q); free(Kh); free(Vh); free(Kw); free(Vw); free(O); free(lse);
        }
    printf(fails ? "oracle driver: %d failures\n" : "oracle driver ok\n", fails);
    return fails != 0;
}
