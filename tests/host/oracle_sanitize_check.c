/* Drives every routine of the CPU oracle (oracle/vgg_ref.c, compiled into this program) on small
 * exactly-sized heap buffers, odd sizes included, so that a build with -fsanitize=address,undefined
 * reports any access outside a buffer or undefined arithmetic.  Prints "ok" when all calls return 0. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/vgg_ref.c"

static double *buf(size_t n, unsigned *seed)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) {
        *seed = *seed * 1664525u + 1013904223u;
        p[i] = ((double)(*seed >> 8) / (double)(1u << 24)) - 0.5;
    }
    return p;
}

int main(void)
{
    unsigned seed = 7u;
    int bad = 0;
    const int shapes[][5] = {{1, 1, 1, 1, 1}, {2, 3, 5, 4, 6}, {3, 2, 4, 7, 2}, {1, 5, 3, 2, 9}, {2, 4, 4, 8, 8}};
    for (size_t s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
        const int N = shapes[s][0], Cin = shapes[s][1], Cout = shapes[s][2], H = shapes[s][3], W = shapes[s][4];
        double *x = buf((size_t)N * Cin * H * W, &seed), *w = buf((size_t)Cout * Cin * 9, &seed), *b = buf(Cout, &seed);
        double *y = buf((size_t)N * Cout * H * W, &seed), *g = buf((size_t)N * Cout * H * W, &seed);
        double *dx = buf((size_t)N * Cin * H * W, &seed), *dw = buf((size_t)Cout * Cin * 9, &seed), *db = buf(Cout, &seed);
        bad |= ref_conv3x3_fwd(N, Cin, Cout, H, W, x, w, b, 1, y);
        bad |= ref_conv3x3_fwd(N, Cin, Cout, H, W, x, w, NULL, 0, y);
        bad |= ref_conv3x3_bwd_data(N, Cin, Cout, H, W, g, w, dx);
        bad |= ref_conv3x3_bwd_weight(N, Cin, Cout, H, W, x, g, dw, db);
        bad |= ref_relu_bwd((size_t)N * Cout * H * W, y, g, g);
        if (H % 2 == 0 && W % 2 == 0) {
            double *p = buf((size_t)N * Cout * (H / 2) * (W / 2), &seed);
            uint8_t *arg = (uint8_t *)malloc((size_t)N * Cout * (H / 2) * (W / 2));
            bad |= ref_maxpool2x2(N, Cout, H, W, y, p, arg);
            bad |= ref_maxpool2x2_bwd(N, Cout, H, W, p, arg, y);
            free(p); free(arg);
        }
        free(x); free(w); free(b); free(y); free(g); free(dx); free(dw); free(db);
    }
    const int fcs[][3] = {{1, 1, 1}, {10, 10, 10}, {3, 7, 5}, {2, 33, 4}};
    for (size_t s = 0; s < sizeof fcs / sizeof fcs[0]; ++s) {
        const int N = fcs[s][0], In = fcs[s][1], Out = fcs[s][2];
        double *a = buf((size_t)N * In, &seed), *w = buf((size_t)Out * In, &seed), *b = buf(Out, &seed);
        double *z = buf((size_t)N * Out, &seed), *p = buf((size_t)N * Out, &seed), *dz = buf((size_t)N * Out, &seed);
        double *dw = buf((size_t)Out * In, &seed), *db = buf(Out, &seed), *da = buf((size_t)N * In, &seed);
        int32_t *lab = (int32_t *)malloc((size_t)N * sizeof(int32_t));
        for (int n = 0; n < N; ++n) lab[n] = (n * 7) % Out;
        double loss = 0.0;
        bad |= ref_fc(N, In, Out, a, w, b, 1, z);
        bad |= ref_fc(N, In, Out, a, w, NULL, 0, z);
        bad |= ref_softmax(N, Out, z, p);
        bad |= ref_softmax_vjp(N, Out, p, z, dz);
        bad |= ref_softmax_xent(N, Out, p, lab, &loss, dz);
        bad |= ref_fc_bwd(N, In, Out, a, w, dz, dw, db, da);
        bad |= ref_fc_bwd(N, In, Out, a, w, dz, dw, db, NULL);
        bad |= ref_sgd((size_t)Out * In, w, dw, 0.01);
        free(a); free(w); free(b); free(z); free(p); free(dz); free(dw); free(db); free(da); free(lab);
    }
    if (bad || ref_num_threads() < 1) { printf("a routine returned an error\n"); return 1; }
    printf("ok\n");
    return 0;
}
