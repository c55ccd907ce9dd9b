/* Driver for the host-sanitizer build of the CPU oracle (compiled together with
 * oracle/rnn_oracle.c by tests/test_oracle_sanitizers.py with
 * -fsanitize=address,undefined).  It runs two of the oracle's pins on inputs with odd sizes, so
 * that an out-of-bounds index or an uninitialised read anywhere in forward, loss or BPTT (both
 * input kinds, both losses, initial state, incoming gradient) stops the program:
 *   pin 1  zero weights: the loss is ln(NV) and dc = (1/NV - onehot) / N exactly;
 *   pin 2  central finite differences of the loss for every parameter of a small tanh/MSE and a
 *          sigmoid/CE network agree with orc_bptt.
 * Exit status 0 and the line "ok" mean both held. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t in_dim, hidden, out_dim, seq_len, batch, input_kind, act, loss_kind;
} orc_dims;
int orc_forward(const orc_dims *d, const double *Wx, const double *Wh, const double *b, const void *x,
                const double *h0, double *h_all);
int orc_loss(const orc_dims *d, const double *V, const double *c, const double *h_all, const void *targets,
             double *loss, double *lse, double *Z);
int orc_bptt(const orc_dims *d, const double *Wx, const double *Wh, const double *V, const double *c,
             const void *x, const void *targets, const double *h_all, const double *dh_last, double *dWx,
             double *dWh, double *db, double *dV, double *dc, double *dh0, double *delta_out, double *g_out,
             double *dZ_out);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform(void)      /* splitmix64 -> (-0.5, 0.5) */
{
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (double)(z >> 11) / 9007199254740992.0 - 0.5;
}
static double *vec(size_t n, double scale)
{
    double *p = (double *)malloc(n * sizeof(double));     /* exact size: an overrun is an error */
    for (size_t i = 0; i < n; ++i) p[i] = scale * uniform();
    return p;
}

static int fail(const char *what, double got, double want)
{
    printf("FAILED %s: got %.12g, want %.12g\n", what, got, want);
    return 1;
}

static int pin_zero_weights(void)
{
    const orc_dims d = {7, 5, 7, 3, 2, 0, 0, 0};
    const int NV = 7, H = 5, T = 3, B = 2, N = T * B;
    double *Wx = vec((size_t)NV * H, 0), *Wh = vec((size_t)H * H, 0), *b = vec(H, 0);
    double *V = vec((size_t)H * NV, 0), *c = vec(NV, 0), *h_all = vec((size_t)(T + 1) * B * H, 1);
    int32_t x[6] = {0, 6, 3, 3, 1, 5}, y[6] = {6, 0, 2, 2, 4, 1};
    double loss = -1;
    if (orc_forward(&d, Wx, Wh, b, x, NULL, h_all) || orc_loss(&d, V, c, h_all, y, &loss, NULL, NULL)) return 1;
    if (fabs(loss - log((double)NV)) > 1e-14) return fail("zero-weight loss", loss, log((double)NV));
    double *dWx = vec((size_t)NV * H, 1), *dWh = vec((size_t)H * H, 1), *db = vec(H, 1);
    double *dV = vec((size_t)H * NV, 1), *dc = vec(NV, 1), *dh0 = vec((size_t)B * H, 1);
    if (orc_bptt(&d, Wx, Wh, V, c, x, y, h_all, NULL, dWx, dWh, db, dV, dc, dh0, NULL, NULL, NULL)) return 1;
    for (int k = 0; k < NV; ++k) {
        int hits = 0;
        for (int n = 0; n < N; ++n) hits += y[n] == k;
        const double want = ((double)N / NV - hits) / N;
        if (fabs(dc[k] - want) > 1e-14) return fail("zero-weight dc", dc[k], want);
    }
    free(Wx); free(Wh); free(b); free(V); free(c); free(h_all);
    free(dWx); free(dWh); free(db); free(dV); free(dc); free(dh0);
    return 0;
}

/* loss of the network as a function of all parameters (forward + loss) */
static double loss_of(const orc_dims *d, double **P, const void *x, const void *y, const double *h0)
{
    const size_t nh = (size_t)(d->seq_len + 1) * d->batch * d->hidden;
    double *h_all = (double *)malloc(nh * sizeof(double)), loss = 0;
    if (orc_forward(d, P[0], P[1], P[2], x, h0, h_all) || orc_loss(d, P[3], P[4], h_all, y, &loss, NULL, NULL)) {
        printf("FAILED forward/loss returned an error\n");
        exit(1);
    }
    free(h_all);
    return loss;
}

static int pin_finite_differences(int dense)
{
    /* dense: tanh + MSE on real inputs and targets; else sigmoid + softmax-CE on token ids */
    const orc_dims d = {dense ? 3 : 6, 5, dense ? 2 : 6, 4, 3, dense, dense, dense};
    const int D = d.in_dim, H = d.hidden, O = d.out_dim, T = d.seq_len, B = d.batch, N = T * B;
    const size_t sz[5] = {(size_t)D * H, (size_t)H * H, (size_t)H, (size_t)H * O, (size_t)O};
    const char *name[5] = {"dWx", "dWh", "db", "dV", "dc"};
    double *P[5], *G[5];
    for (int i = 0; i < 5; ++i) { P[i] = vec(sz[i], 1.0); G[i] = vec(sz[i], 1.0); }
    double *h0 = vec((size_t)B * H, 1.0);
    void *x, *y;
    if (dense) {
        x = vec((size_t)N * D, 2.0);
        y = vec((size_t)N * O, 2.0);
    } else {
        int32_t *xi = (int32_t *)malloc(N * sizeof(int32_t)), *yi = (int32_t *)malloc(N * sizeof(int32_t));
        for (int n = 0; n < N; ++n) { xi[n] = (int32_t)((uniform() + 0.5) * D) % D; yi[n] = (int32_t)((uniform() + 0.5) * O) % O; }
        x = xi; y = yi;
    }
    double *h_all = vec((size_t)(T + 1) * B * H, 1.0), *dh0 = vec((size_t)B * H, 1.0), loss;
    if (orc_forward(&d, P[0], P[1], P[2], x, h0, h_all) || orc_loss(&d, P[3], P[4], h_all, y, &loss, NULL, NULL) ||
        orc_bptt(&d, P[0], P[1], P[3], P[4], x, y, h_all, NULL, G[0], G[1], G[2], G[3], G[4], dh0, NULL, NULL, NULL))
        return 1;
    const double eps = 1e-6;
    for (int i = 0; i < 5; ++i)
        for (size_t k = 0; k < sz[i]; ++k) {
            const double keep = P[i][k];
            P[i][k] = keep + eps;
            const double up = loss_of(&d, P, x, y, h0);
            P[i][k] = keep - eps;
            const double dn = loss_of(&d, P, x, y, h0);
            P[i][k] = keep;
            const double fd = (up - dn) / (2 * eps);
            if (fabs(fd - G[i][k]) > 1e-8 + 1e-6 * fabs(fd)) return fail(name[i], G[i][k], fd);
        }
    for (size_t k = 0; k < (size_t)B * H; ++k) {        /* d loss / d initial state */
        const double keep = h0[k];
        h0[k] = keep + eps;
        const double up = loss_of(&d, P, x, y, h0);
        h0[k] = keep - eps;
        const double dn = loss_of(&d, P, x, y, h0);
        h0[k] = keep;
        const double fd = (up - dn) / (2 * eps);
        if (fabs(fd - dh0[k]) > 1e-8 + 1e-6 * fabs(fd)) return fail("dh0", dh0[k], fd);
    }
    for (int i = 0; i < 5; ++i) { free(P[i]); free(G[i]); }
    free(h0); free(x); free(y); free(h_all); free(dh0);
    return 0;
}

int main(void)
{
    if (pin_zero_weights() || pin_finite_differences(0) || pin_finite_differences(1)) return 1;
    printf("ok\n");
    return 0;
}
