/* Driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of the CPU oracle
 * (tests/test_oracle_sanitize.py compiles it together with oracle/bapipe_oracle.c).
 * Every oracle function runs on small seeded tensors held in exactly-sized heap blocks, over
 * the filter / stride / padding combinations the workloads use plus ragged ones, so that a
 * read or write one element outside a tensor, a signed overflow or a misaligned access
 * aborts the run.  Two cheap identities are checked on the way (adjointness of the input
 * gradient, linearity of the weight gradient) so that the outputs are used.  Exit code 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void orc_round_bf16(double *a, size_t n);
void orc_conv2d_fwd(const double *x, const double *w, const double *b, double *y, int N, int Cin, int H, int W, int Cout, int kh, int kw, int st, int pad);
void orc_conv2d_dgrad(const double *dy, const double *w, double *dx, int N, int Cin, int H, int W, int Cout, int kh, int kw, int st, int pad);
void orc_conv2d_wgrad(const double *x, const double *dy, double *dw, double *db, int N, int Cin, int H, int W, int Cout, int kh, int kw, int st, int pad);
void orc_relu_fwd(const double *x, double *y, size_t n);
void orc_relu_bwd(const double *y, const double *dy, double *dx, size_t n);
void orc_maxpool_fwd(const double *x, double *y, uint8_t *idx, int N, int C, int H, int W, int kh, int kw, int st, int pad);
void orc_maxpool_bwd(const double *dy, const uint8_t *idx, double *dx, int N, int C, int H, int W, int kh, int kw, int st, int pad);
void orc_avgpool_fwd(const double *x, double *y, int N, int C, int H, int W, int kh, int kw);
void orc_avgpool_bwd(const double *dy, double *dx, int N, int C, int H, int W, int kh, int kw);
void orc_lstm_fwd(const double *x, const double *w, const double *b, double *y, double *gates, double *cells, int N, int In, int Hd, int T, int round16);
void orc_lstm_bwd(const double *x, const double *y, const double *w, const double *gates, const double *cells, const double *dy, double *dx, double *dw, double *db, double *D, int N, int In, int Hd, int T, int round16);
void orc_bn_fwd(const double *x, const double *gamma, const double *beta, double eps, double *y, double *mean, double *invstd, int N, int C, int HW);
void orc_bn_bwd(const double *x, const double *dy, const double *gamma, const double *mean, const double *invstd, double *dx, double *dgamma, double *dbeta, int N, int C, int HW);
void orc_linear_fwd(const double *x, const double *w, const double *b, double *y, int N, int In, int Out);
void orc_linear_dgrad(const double *dy, const double *w, double *dx, int N, int In, int Out);
void orc_linear_wgrad(const double *x, const double *dy, double *dw, double *db, int N, int In, int Out);
void orc_softmax_fwd(const double *z, double *p, int N, int K);
double orc_xent_bwd(const double *z, const int32_t *label, double scale, double *dz, int N, int K);
void orc_sgd_step(double *w, const double *g, double lr, size_t n);

static uint64_t rng_state = 0x20121254u;
static double rnd(void)
{
    rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double *tensor(size_t n, int fill)
{
    double *p = malloc(n * sizeof(double) + (n == 0));
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = fill ? rnd() : 0.0;
    return p;
}
static double dot(const double *a, const double *b, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}
static int failures = 0;
static void close_to(double a, double b, const char *what)
{
    if (!(fabs(a - b) <= 1e-9 * (1.0 + fabs(a) + fabs(b)))) {
        fprintf(stderr, "MISMATCH %s: %.17g vs %.17g\n", what, a, b);
        ++failures;
    }
}

static void conv_case(int N, int Ci, int H, int W, int Co, int k, int st, int pad)
{
    const int Ho = (H + 2 * pad - k) / st + 1, Wo = (W + 2 * pad - k) / st + 1;
    const size_t nx = (size_t)N * Ci * H * W, ny = (size_t)N * Co * Ho * Wo, nw = (size_t)Co * Ci * k * k;
    double *x = tensor(nx, 1), *w = tensor(nw, 1), *b = tensor(Co, 1), *y = tensor(ny, 0), *g = tensor(ny, 1);
    double *dx = tensor(nx, 0), *dw = tensor(nw, 0), *db = tensor(Co, 0), *zero_b = tensor(Co, 0);
    orc_conv2d_fwd(x, w, zero_b, y, N, Ci, H, W, Co, k, k, st, pad);
    orc_conv2d_dgrad(g, w, dx, N, Ci, H, W, Co, k, k, st, pad);
    orc_conv2d_wgrad(x, g, dw, db, N, Ci, H, W, Co, k, k, st, pad);
    close_to(dot(y, g, ny), dot(x, dx, nx), "conv <y,g> = <x,dx>");
    close_to(dot(y, g, ny), dot(w, dw, nw), "conv <y,g> = <w,dw>");
    orc_conv2d_fwd(x, w, b, y, N, Ci, H, W, Co, k, k, st, pad);
    orc_conv2d_wgrad(x, g, dw, NULL, N, Ci, H, W, Co, k, k, st, pad);
    free(x); free(w); free(b); free(y); free(g); free(dx); free(dw); free(db); free(zero_b);
}

static void pool_case(int N, int C, int H, int W, int k, int st, int pad)
{
    const int Ho = (H + 2 * pad - k) / st + 1, Wo = (W + 2 * pad - k) / st + 1;
    const size_t nx = (size_t)N * C * H * W, ny = (size_t)N * C * Ho * Wo;
    double *x = tensor(nx, 1), *y = tensor(ny, 0), *g = tensor(ny, 1), *dx = tensor(nx, 0);
    uint8_t *idx = malloc(ny + (ny == 0));
    orc_maxpool_fwd(x, y, idx, N, C, H, W, k, k, st, pad);
    orc_maxpool_bwd(g, idx, dx, N, C, H, W, k, k, st, pad);
    double sg = 0.0, sd = 0.0;
    for (size_t i = 0; i < ny; ++i) sg += g[i];
    for (size_t i = 0; i < nx; ++i) sd += dx[i];
    close_to(sg, sd, "max-pool gradient mass");
    free(x); free(y); free(g); free(dx); free(idx);
}

int main(void)
{
    static const int convs[][8] = {
        {2, 3, 7, 5, 4, 3, 1, 1}, {1, 2, 9, 8, 3, 3, 2, 1}, {2, 4, 7, 7, 2, 1, 2, 0}, {1, 3, 13, 11, 2, 7, 2, 3},
        {2, 5, 4, 6, 3, 1, 1, 0}, {1, 1, 3, 3, 1, 3, 1, 1}, {1, 2, 5, 5, 2, 5, 1, 0}, {1, 2, 6, 6, 2, 3, 1, 2},
    };
    for (size_t i = 0; i < sizeof convs / sizeof convs[0]; ++i)
        conv_case(convs[i][0], convs[i][1], convs[i][2], convs[i][3], convs[i][4], convs[i][5], convs[i][6], convs[i][7]);
    static const int pools[][7] = {
        {2, 3, 8, 6, 2, 2, 0}, {1, 2, 9, 7, 2, 2, 0}, {2, 2, 9, 8, 3, 2, 1}, {1, 3, 5, 5, 3, 1, 1}, {1, 1, 6, 7, 2, 2, 1},
        {1, 2, 7, 7, 3, 2, 0},
    };
    for (size_t i = 0; i < sizeof pools / sizeof pools[0]; ++i)
        pool_case(pools[i][0], pools[i][1], pools[i][2], pools[i][3], pools[i][4], pools[i][5], pools[i][6]);
    {   /* average pool incl. the global one and a ragged remainder that is dropped */
        static const int ap[][5] = {{2, 3, 6, 6, 3}, {1, 2, 7, 7, 7}, {1, 2, 7, 5, 2}};
        for (size_t i = 0; i < 3; ++i) {
            const int N = ap[i][0], C = ap[i][1], H = ap[i][2], W = ap[i][3], k = ap[i][4];
            const size_t nx = (size_t)N * C * H * W, ny = (size_t)N * C * (H / k) * (W / k);
            double *x = tensor(nx, 1), *y = tensor(ny, 0), *g = tensor(ny, 1), *dx = tensor(nx, 0);
            orc_avgpool_fwd(x, y, N, C, H, W, k, k);
            orc_avgpool_bwd(g, dx, N, C, H, W, k, k);
            close_to(dot(y, g, ny), dot(x, dx, nx), "avg-pool adjoint");
            free(x); free(y); free(g); free(dx);
        }
    }
    {   /* ReLU, bf16 rounding, SGD */
        const size_t n = 1001;
        double *x = tensor(n, 1), *y = tensor(n, 0), *g = tensor(n, 1), *dx = tensor(n, 0);
        orc_relu_fwd(x, y, n);
        orc_relu_bwd(y, g, dx, n);
        x[0] = 0.0; x[1] = -0.0; x[2] = 1e-45; x[3] = 3.4e38; x[4] = -3.4e38; x[5] = 1e300; x[6] = 1.0 + 1.0 / 256;
        orc_round_bf16(x, n);
        orc_sgd_step(x, g, 0.1, n);
        orc_round_bf16(x, 0);
        free(x); free(y); free(g); free(dx);
    }
    {   /* batch-norm */
        const int N = 3, C = 5, HW = 7;
        const size_t n = (size_t)N * C * HW;
        double *x = tensor(n, 1), *y = tensor(n, 0), *g = tensor(n, 1), *dx = tensor(n, 0);
        double *ga = tensor(C, 1), *be = tensor(C, 1), *mu = tensor(C, 0), *is = tensor(C, 0), *dga = tensor(C, 0), *dbe = tensor(C, 0);
        orc_bn_fwd(x, ga, be, 1e-5, y, mu, is, N, C, HW);
        orc_bn_bwd(x, g, ga, mu, is, dx, dga, dbe, N, C, HW);
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            for (int nn = 0; nn < N; ++nn)
                for (int p = 0; p < HW; ++p) s += dx[((size_t)nn * C + c) * HW + p];
            close_to(s, 0.0, "batch-norm sum dx");
        }
        free(x); free(y); free(g); free(dx); free(ga); free(be); free(mu); free(is); free(dga); free(dbe);
    }
    {   /* linear, softmax, cross-entropy */
        const int N = 4, In = 9, Out = 6;
        double *x = tensor((size_t)N * In, 1), *w = tensor((size_t)Out * In, 1), *b = tensor(Out, 0), *y = tensor((size_t)N * Out, 0);
        double *g = tensor((size_t)N * Out, 1), *dx = tensor((size_t)N * In, 0), *dw = tensor((size_t)Out * In, 0), *db = tensor(Out, 0);
        double *p = tensor((size_t)N * Out, 0), *dz = tensor((size_t)N * Out, 0);
        int32_t lab[4] = {0, 5, 2, 3};
        orc_linear_fwd(x, w, b, y, N, In, Out);
        orc_linear_dgrad(g, w, dx, N, In, Out);
        orc_linear_wgrad(x, g, dw, db, N, In, Out);
        orc_linear_wgrad(x, g, dw, NULL, N, In, Out);
        close_to(dot(y, g, (size_t)N * Out), dot(x, dx, (size_t)N * In), "linear adjoint");
        orc_softmax_fwd(y, p, N, Out);
        const double loss = orc_xent_bwd(y, lab, 0.25, dz, N, Out);
        if (!(loss > 0.0)) { fprintf(stderr, "loss %g\n", loss); ++failures; }
        free(x); free(w); free(b); free(y); free(g); free(dx); free(dw); free(db); free(p); free(dz);
    }
    for (int round16 = 0; round16 < 2; ++round16) {   /* LSTM, T = 1 and T > 1 */
        static const int ls[][4] = {{2, 3, 4, 1}, {3, 5, 2, 4}};
        for (size_t i = 0; i < 2; ++i) {
            const int N = ls[i][0], In = ls[i][1], Hd = ls[i][2], T = ls[i][3], G = 4 * Hd;
            double *x = tensor((size_t)N * T * In, 1), *w = tensor((size_t)G * (In + Hd), 1), *b = tensor(G, 1);
            double *y = tensor((size_t)N * T * Hd, 0), *gates = tensor((size_t)N * T * G, 0), *cells = tensor((size_t)N * T * Hd, 0);
            double *dy = tensor((size_t)N * T * Hd, 1), *dx = tensor((size_t)N * T * In, 0), *dw = tensor((size_t)G * (In + Hd), 0);
            double *db = tensor(G, 0), *D = tensor((size_t)N * T * G, 0);
            orc_lstm_fwd(x, w, b, y, gates, cells, N, In, Hd, T, round16);
            orc_lstm_bwd(x, y, w, gates, cells, dy, dx, dw, db, D, N, In, Hd, T, round16);
            free(x); free(w); free(b); free(y); free(gates); free(cells); free(dy); free(dx); free(dw); free(db); free(D);
        }
    }
    if (failures) return 1;
    puts("oracle sanitizer run clean");
    return 0;
}
