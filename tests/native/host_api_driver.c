/* Host-side checks of libtlinattn's planning and argument validation, meant to be built together
 * with the library's source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only)
 * and run on a machine without a GPU: every call below returns before any HIP call. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "tlinattn.h"
#include "tlinattn_profile.h"

static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static tlin_params params(int B, int H, int W, int N, int D, int dt)
{
    tlin_params p;
    memset(&p, 0, sizeof p);
    p.B = B; p.H = H; p.W = W; p.N = N; p.D = D;
    p.in_dtype = dt; p.out_dtype = dt;
    p.scale = 0.125f;
    return p;
}

int main(void)
{
    void *fake = (void *)(uintptr_t)(1u << 20);   /* aligned, never dereferenced: validation fails first */
    static const int Ws[] = {1, 7, 64, 65, 128, 129, 512, 4096, 100000};
    static const int Ns[] = {1, 63, 64, 65, 1000, 131072, 1 << 30};
    static const int Ds[] = {8, 12, 36, 64, 100, 128};
    for (int dt = 0; dt < 2; ++dt)
        for (unsigned wi = 0; wi < sizeof Ws / sizeof *Ws; ++wi)
            for (unsigned ni = 0; ni < sizeof Ns / sizeof *Ns; ++ni)
                for (unsigned di = 0; di < sizeof Ds / sizeof *Ds; ++di)
                    for (int bh = 1; bh <= 4096; bh *= 64) {
                        tlin_params p = params(1, bh, Ws[wi], Ns[ni], Ds[di], dt);
                        for (int ns = 0; ns <= 2000; ns = ns ? ns * 37 : 1) {
                            p.num_splits = ns;
                            const int s = tlin_num_splits(&p);
                            const size_t ws = tlin_workspace_bytes(&p);
                            CHECK(s >= 1 && s <= 1024);
                            CHECK(ws >= (size_t)bh * (s + 1) * Ws[wi] * 4);
                            const int tile = dt == TLIN_F32 ? 32 : 64;
                            CHECK(s <= (Ns[ni] + tile - 1) / tile);        /* no partition is empty */
                        }
                        p.num_splits = 0;
                        tlin_params q = p;                                  /* sliding schedule over N rows */
                        if (Ws[wi] <= Ns[ni]) CHECK(tlin_slide_workspace_bytes(&q) > 0);
                    }
    /* error paths: each returns a status, none touches the device */
    tlin_params p = params(2, 3, 64, 1024, 64, TLIN_BF16);
    CHECK(tlin_history_attn(NULL, fake, fake, fake, fake, NULL, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    CHECK(tlin_history_attn(&p, NULL, fake, fake, fake, NULL, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    CHECK(tlin_history_attn(&p, (char *)fake + 2, fake, fake, fake, NULL, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    p.num_splits = 4;
    CHECK(tlin_history_attn(&p, fake, fake, fake, fake, NULL, NULL, 0, NULL) == TLIN_ERR_WORKSPACE);
    CHECK(tlin_history_attn(&p, fake, fake, fake, fake, NULL, fake, 16, NULL) == TLIN_ERR_WORKSPACE);
    CHECK(tlin_layer_attn(&p, fake, NULL, fake, fake, fake, fake, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    p.combine = 7;
    CHECK(tlin_layer_attn(&p, fake, fake, fake, fake, fake, fake, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    p.combine = 0; p.D = 30;
    CHECK(tlin_window_causal_attn(&p, fake, fake, fake, fake, NULL, NULL, 0, NULL) == TLIN_ERR_UNSUPPORTED);
    p.D = 64; p.N = (1 << 30) + 1;
    CHECK(tlin_slide_layer_attn(&p, fake, fake, fake, fake, fake, fake, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    p.N = 1024; p.q_stride[0] = 1; p.q_stride[1] = 8; p.q_stride[2] = 24;   /* row stride < D */
    CHECK(tlin_history_attn(&p, fake, fake, fake, fake, NULL, fake, 1u << 30, NULL) == TLIN_ERR_INVALID_ARG);
    /* the static-workspace layer call: same argument checks, and its size limit, all on the host */
    tlin_params sp = params(1, 32, 512, 131072, 128, TLIN_BF16);
    CHECK(tlin_workspace_bytes(&sp) <= TLIN_STATIC_WS_BYTES);
    CHECK(tlin_layer_attn_static_ws(&sp, NULL, fake, fake, fake, fake, fake, NULL) == TLIN_ERR_INVALID_ARG);
    CHECK(tlin_layer_attn_static_ws(&sp, fake, fake, fake, fake, (char *)fake + 8, fake, NULL) == TLIN_ERR_INVALID_ARG);
    sp.B = 4;
    CHECK(tlin_workspace_bytes(&sp) > TLIN_STATIC_WS_BYTES);
    CHECK(tlin_layer_attn_static_ws(&sp, fake, fake, fake, fake, fake, fake, NULL) == TLIN_ERR_WORKSPACE);
    sp.combine = 9;
    CHECK(tlin_layer_attn_static_ws(&sp, fake, fake, fake, fake, fake, fake, NULL) == TLIN_ERR_INVALID_ARG);
    double ms[3]; int64_t n[3];
    CHECK(tlin_profile_read(NULL, n) == TLIN_ERR_INVALID_ARG);
    CHECK(tlin_profile_read(ms, n) == TLIN_OK && n[0] == 0 && n[1] == 0 && n[2] == 0);
    for (int s = -1; s < 8; ++s) CHECK(tlin_status_string(s) != NULL);
    CHECK(tlin_version() >= 100);
    printf(fails ? "host api driver: %d failures\n" : "host api driver ok\n", fails);
    return fails != 0;
}
