/*
 * rnn_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision CPU definition of what the Elman-RNN training path
 * computes: forward recurrence, output layer + loss, and the gradients that
 * backpropagation through time yields.  It exists so that the GPU library can be
 * checked against something that can be verified by eye; nothing in the product
 * path may call, link or import it, and it shares no code with the GPU path.
 *
 * What the paper fixes: the loop is a scan over the leading (time) axis of its
 * sequences, and its gradient is backpropagation through time that keeps every
 * hidden state (Scan section, property 1); the benchmarked model is a simple
 * recurrent network whose input and output layers both have vocabulary size
 * (recurrent-network benchmark section).  The paper prints no equations for the
 * network; the Elman equations below are the textbook ones:
 *
 *   a_t = in_t + Wh h_{t-1} + b,  h_t = act(a_t)           act = sigmoid | tanh
 *   in_t = Wx[x_t,:]  (token input)  or  Wx x_t  (dense input)
 *   z_t = V^T h_t + c
 *   CE : loss = mean_n ( logsumexp(z_n) - z_n[y_n] )        natural log, n over T*B rows
 *   MSE: loss = mean_{n,k} (z_nk - Y_nk)^2                  no factor 1/2
 *
 * BPTT reaches exactly d loss / d parameter (it is not an approximation), so the
 * gradient functions are the chain rule written out, one row and one step at a time.
 *
 * All arrays are double, row-major, time-major ([T,B,.]).  Parallelism (OpenMP) is
 * only over independent units (batch rows, output rows); loop bodies stay plain.
 * Return value 0 = ok, -1 = bad argument.
 *
 * Pins (tests/test_oracle_*.py): central finite differences of the loss for every
 * parameter, closed forms at zero weights, softmax rows summing to one, column-sum
 * invariants, the no-recurrence special case against a separately written one-layer
 * routine, T=1, batch averaging, window chaining, a float64 autograd cross-check and a
 * hand-derived scalar case.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t in_dim;     /* NV (token input) or D (dense input) */
    int32_t hidden;     /* H */
    int32_t out_dim;    /* NV (softmax-CE) or O (linear-MSE) */
    int32_t seq_len;    /* T */
    int32_t batch;      /* B */
    int32_t input_kind; /* 0 token ids int32[T,B], 1 dense double[T,B,D] */
    int32_t act;        /* 0 sigmoid, 1 tanh */
    int32_t loss_kind;  /* 0 softmax cross-entropy, 1 linear + MSE */
} orc_dims;

static int dims_ok(const orc_dims *d)
{
    return d && d->in_dim > 0 && d->hidden > 0 && d->out_dim > 0 && d->seq_len > 0 &&
           d->batch > 0 && (d->input_kind == 0 || d->input_kind == 1) &&
           (d->act == 0 || d->act == 1) && (d->loss_kind == 0 || d->loss_kind == 1);
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- forward recurrence: h_all[0] = h0 (zeros if NULL), h_all[t+1] = h_t ---------- */
int orc_forward(const orc_dims *d, const double *Wx, const double *Wh, const double *b,
                const void *x, const double *h0, double *h_all)
{
    if (!dims_ok(d) || !Wx || !Wh || !b || !x || !h_all) return -1;
    const int H = d->hidden, T = d->seq_len, B = d->batch, D = d->in_dim;
    const int32_t *ids = (const int32_t *)x;
    const double *X = (const double *)x;

    for (int bb = 0; bb < B; ++bb)
        for (int j = 0; j < H; ++j)
            h_all[(size_t)bb * H + j] = h0 ? h0[(size_t)bb * H + j] : 0.0;

#pragma omp parallel for schedule(static)
    for (int bb = 0; bb < B; ++bb) {
        for (int t = 0; t < T; ++t) {
            const double *hp = h_all + ((size_t)t * B + bb) * H;
            double *hn = h_all + ((size_t)(t + 1) * B + bb) * H;
            for (int j = 0; j < H; ++j) {
                double a = b[j];
                if (d->input_kind == 0) {
                    int32_t v = ids[(size_t)t * B + bb];
                    a += Wx[(size_t)v * H + j];
                } else {
                    const double *xt = X + ((size_t)t * B + bb) * D;
                    for (int k = 0; k < D; ++k) a += Wx[(size_t)j * D + k] * xt[k];
                }
                for (int i = 0; i < H; ++i) a += Wh[(size_t)j * H + i] * hp[i];
                hn[j] = d->act == 0 ? 1.0 / (1.0 + exp(-a)) : tanh(a);
            }
        }
    }
    return 0;
}

/* logits of one row n: z[k] = sum_i h[i] V[i,k] + c[k] */
static void logits_row(const double *h, const double *V, const double *c, int H, int O, double *z)
{
    for (int k = 0; k < O; ++k) z[k] = c[k];
    for (int i = 0; i < H; ++i) {
        const double hi = h[i];
        const double *Vi = V + (size_t)i * O;
        for (int k = 0; k < O; ++k) z[k] += hi * Vi[k];
    }
}

/* ---- output layer + loss.  lse[N] and Z[N,O] are optional outputs ----------------- */
int orc_loss(const orc_dims *d, const double *V, const double *c, const double *h_all,
             const void *targets, double *loss, double *lse, double *Z)
{
    if (!dims_ok(d) || !V || !c || !h_all || !targets || !loss) return -1;
    const int H = d->hidden, O = d->out_dim;
    const long N = (long)d->seq_len * d->batch;
    const int32_t *y = (const int32_t *)targets;
    const double *Y = (const double *)targets;
    double total = 0.0;
    int bad = 0;

#pragma omp parallel for schedule(static) reduction(+ : total) reduction(| : bad)
    for (long n = 0; n < N; ++n) {
        double *z = Z ? Z + (size_t)n * O : (double *)malloc(sizeof(double) * O);
        const double *h = h_all + (size_t)(n + d->batch) * H; /* row n of h_all[1:] */
        logits_row(h, V, c, H, O, z);
        if (d->loss_kind == 0) {
            double m = z[0];
            for (int k = 1; k < O; ++k) if (z[k] > m) m = z[k];
            double s = 0.0;
            for (int k = 0; k < O; ++k) s += exp(z[k] - m);
            const double l = m + log(s);
            if (lse) lse[n] = l;
            if (y[n] < 0 || y[n] >= O) bad = 1; else total += l - z[y[n]];
        } else {
            double s = 0.0;
            for (int k = 0; k < O; ++k) {
                const double e = z[k] - Y[(size_t)n * O + k];
                s += e * e;
            }
            total += s;
        }
        if (!Z) free(z);
    }
    if (bad) return -1;
    *loss = d->loss_kind == 0 ? total / (double)N : total / ((double)N * O);
    return 0;
}

/* ---- gradients by backpropagation through time ------------------------------------
 * Outputs are overwritten.  dh_last (nullable, [B,H]) is d loss / d h_{T-1} arriving
 * from a later window; dh0 (nullable, [B,H]) receives d loss / d h_{-1}.
 * delta_out (nullable, [T,B,H]) receives d loss / d a_t; g_out (nullable, [T,B,H])
 * receives the output layer's contribution to d loss / d h_t; dZ_out (nullable,
 * [T*B,O]) receives d loss / d z.
 */
int orc_bptt(const orc_dims *d, const double *Wx, const double *Wh, const double *V,
             const double *c, const void *x, const void *targets, const double *h_all,
             const double *dh_last, double *dWx, double *dWh, double *db, double *dV,
             double *dc, double *dh0, double *delta_out, double *g_out, double *dZ_out)
{
    if (!dims_ok(d) || !Wx || !Wh || !V || !c || !x || !targets || !h_all || !dWx || !dWh ||
        !db || !dV || !dc)
        return -1;
    const int H = d->hidden, O = d->out_dim, T = d->seq_len, B = d->batch, D = d->in_dim;
    const long N = (long)T * B;
    const int32_t *ids = (const int32_t *)x;
    const double *X = (const double *)x;
    const int32_t *y = (const int32_t *)targets;
    const double *Y = (const double *)targets;
    const size_t wx_elems = d->input_kind == 0 ? (size_t)D * H : (size_t)H * D;

    if (d->loss_kind == 0)
        for (long n = 0; n < N; ++n)
            if (y[n] < 0 || y[n] >= O) return -1;

    double *dZ = dZ_out ? dZ_out : (double *)malloc(sizeof(double) * (size_t)N * O);
    double *g = g_out ? g_out : (double *)malloc(sizeof(double) * (size_t)N * H);
    double *delta = delta_out ? delta_out : (double *)malloc(sizeof(double) * (size_t)N * H);
    if (!dZ || !g || !delta) return -1;

    /* d loss / d z, row by row */
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n) {
        double *dz = dZ + (size_t)n * O;
        const double *h = h_all + (size_t)(n + B) * H;
        logits_row(h, V, c, H, O, dz); /* dz holds z for now */
        if (d->loss_kind == 0) {
            double m = dz[0];
            for (int k = 1; k < O; ++k) if (dz[k] > m) m = dz[k];
            double s = 0.0;
            for (int k = 0; k < O; ++k) s += exp(dz[k] - m);
            const double l = m + log(s);
            for (int k = 0; k < O; ++k) dz[k] = exp(dz[k] - l) / (double)N;
            dz[y[n]] -= 1.0 / (double)N;
        } else {
            for (int k = 0; k < O; ++k)
                dz[k] = 2.0 * (dz[k] - Y[(size_t)n * O + k]) / ((double)N * O);
        }
    }

    /* dc[k] = sum_n dz[n,k] */
    for (int k = 0; k < O; ++k) dc[k] = 0.0;
    for (long n = 0; n < N; ++n)
        for (int k = 0; k < O; ++k) dc[k] += dZ[(size_t)n * O + k];

    /* dV[i,k] = sum_n h[n,i] dz[n,k]   (each thread owns rows i) */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < H; ++i) {
        double *dVi = dV + (size_t)i * O;
        for (int k = 0; k < O; ++k) dVi[k] = 0.0;
        for (long n = 0; n < N; ++n) {
            const double hi = h_all[(size_t)(n + B) * H + i];
            const double *dz = dZ + (size_t)n * O;
            for (int k = 0; k < O; ++k) dVi[k] += hi * dz[k];
        }
    }

    /* g[n,i] = sum_k V[i,k] dz[n,k] */
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n) {
        const double *dz = dZ + (size_t)n * O;
        for (int i = 0; i < H; ++i) {
            const double *Vi = V + (size_t)i * O;
            double s = 0.0;
            for (int k = 0; k < O; ++k) s += Vi[k] * dz[k];
            g[(size_t)n * H + i] = s;
        }
    }

    /* reverse-time loop, independent per batch row */
#pragma omp parallel for schedule(static)
    for (int bb = 0; bb < B; ++bb) {
        double *carry = (double *)malloc(sizeof(double) * H); /* Wh^T delta_{t+1} */
        for (int i = 0; i < H; ++i) carry[i] = dh_last ? dh_last[(size_t)bb * H + i] : 0.0;
        for (int t = T - 1; t >= 0; --t) {
            const double *ht = h_all + ((size_t)(t + 1) * B + bb) * H;
            double *dl = delta + ((size_t)t * B + bb) * H;
            const double *gt = g + ((size_t)t * B + bb) * H;
            for (int j = 0; j < H; ++j) {
                const double dh = gt[j] + carry[j];
                const double dact = d->act == 0 ? ht[j] * (1.0 - ht[j]) : 1.0 - ht[j] * ht[j];
                dl[j] = dh * dact;
            }
            for (int i = 0; i < H; ++i) {
                double s = 0.0;
                for (int j = 0; j < H; ++j) s += Wh[(size_t)j * H + i] * dl[j];
                carry[i] = s;
            }
        }
        if (dh0)
            for (int i = 0; i < H; ++i) dh0[(size_t)bb * H + i] = carry[i];
        free(carry);
    }

    /* parameter gradients of the recurrent layer */
    for (int j = 0; j < H; ++j) db[j] = 0.0;
    for (long n = 0; n < N; ++n)
        for (int j = 0; j < H; ++j) db[j] += delta[(size_t)n * H + j];

#pragma omp parallel for schedule(static)
    for (int j = 0; j < H; ++j) {
        double *row = dWh + (size_t)j * H;
        for (int i = 0; i < H; ++i) row[i] = 0.0;
        for (long n = 0; n < N; ++n) { /* h_{t-1} of row n = (t,b) is h_all row n */
            const double dj = delta[(size_t)n * H + j];
            const double *hp = h_all + (size_t)n * H;
            for (int i = 0; i < H; ++i) row[i] += dj * hp[i];
        }
    }

    for (size_t e = 0; e < wx_elems; ++e) dWx[e] = 0.0;
    if (d->input_kind == 0) {
        for (long n = 0; n < N; ++n) {
            const int32_t v = ids[n];
            if (v < 0 || v >= D) return -1;
            for (int j = 0; j < H; ++j) dWx[(size_t)v * H + j] += delta[(size_t)n * H + j];
        }
    } else {
#pragma omp parallel for schedule(static)
        for (int j = 0; j < H; ++j)
            for (long n = 0; n < N; ++n) {
                const double dj = delta[(size_t)n * H + j];
                const double *xt = X + (size_t)n * D;
                for (int k = 0; k < D; ++k) dWx[(size_t)j * D + k] += dj * xt[k];
            }
    }

    if (!dZ_out) free(dZ);
    if (!g_out) free(g);
    if (!delta_out) free(delta);
    return 0;
}

/* ---- many windows of a token stream with plain stochastic gradient descent --------
 * The paper's function objects can repeat a compiled training function a given number
 * of times without returning to the interpreter (its section on repeated calls of one
 * function); its recurrent benchmark trains a language model that way, one truncated
 * window after the other.  The paper gives no update rule; the plain one is used:
 *
 *   for w = 0 .. n_windows-1:
 *       x = ids[w*T : w*T+T],  y = ids[w*T+1 : w*T+T+1]        (next-token targets)
 *       h_all  = forward(params, x, h)            h = state carried from window w-1
 *       loss_w = loss(params, h_all, y)
 *       grads  = bptt(params, x, y, h_all)        no gradient arrives from later windows
 *       params = params - lr * grads              all five tensors
 *       h      = h_all[T]                         computed with the weights before the update
 *
 * ids: int32 [(n_windows*T + 1), B]; params are updated in place; h [B,H] holds the
 * initial state on entry and the final state on return; losses [n_windows].
 * Token input and softmax cross-entropy only.  Each window simply calls the three
 * functions above.
 */
int orc_train_stream(const orc_dims *d, double *Wx, double *Wh, double *b, double *V, double *c,
                     const int32_t *ids, long n_windows, double lr, double *h, double *losses)
{
    if (!dims_ok(d) || d->input_kind != 0 || d->loss_kind != 0 || !Wx || !Wh || !b || !V || !c ||
        !ids || n_windows < 0 || !h || !losses)
        return -1;
    const int H = d->hidden, O = d->out_dim, T = d->seq_len, B = d->batch, NV = d->in_dim;
    const size_t nWx = (size_t)NV * H, nWh = (size_t)H * H, nV = (size_t)H * O;
    double *h_all = (double *)malloc(sizeof(double) * (size_t)(T + 1) * B * H);
    double *dWx = (double *)malloc(sizeof(double) * nWx);
    double *dWh = (double *)malloc(sizeof(double) * nWh);
    double *db = (double *)malloc(sizeof(double) * H);
    double *dV = (double *)malloc(sizeof(double) * nV);
    double *dc = (double *)malloc(sizeof(double) * O);
    int rc = (h_all && dWx && dWh && db && dV && dc) ? 0 : -1;
    for (long w = 0; w < n_windows && rc == 0; ++w) {
        const int32_t *x = ids + (size_t)w * T * B;
        const int32_t *y = x + B; /* the same stream one step later */
        rc = orc_forward(d, Wx, Wh, b, x, h, h_all);
        if (rc == 0) rc = orc_loss(d, V, c, h_all, y, &losses[w], NULL, NULL);
        if (rc == 0)
            rc = orc_bptt(d, Wx, Wh, V, c, x, y, h_all, NULL, dWx, dWh, db, dV, dc, NULL, NULL,
                          NULL, NULL);
        if (rc != 0) break;
        for (size_t e = 0; e < nWx; ++e) Wx[e] -= lr * dWx[e];
        for (size_t e = 0; e < nWh; ++e) Wh[e] -= lr * dWh[e];
        for (int j = 0; j < H; ++j) b[j] -= lr * db[j];
        for (size_t e = 0; e < nV; ++e) V[e] -= lr * dV[e];
        for (int k = 0; k < O; ++k) c[k] -= lr * dc[k];
        for (size_t e = 0; e < (size_t)B * H; ++e) h[e] = h_all[(size_t)T * B * H + e];
    }
    free(h_all); free(dWx); free(dWh); free(db); free(dV); free(dc);
    return rc;
}

/* ---- Gauss-Newton matrix times a vector, by the R-operator ---------------------------
 * The paper's section on the R-operator: the forward-mode directional derivative
 * R{f} = (df/dtheta) gamma, and, for a recurrent network, the Gauss-Newton
 * approximation of the Hessian times a vector as Lop(f, theta, Rop(f, theta, gamma)),
 * i.e. J^T (J gamma) with J the Jacobian of the network outputs, evaluated with one
 * forward sweep that carries (h_t, R h_t) and one reverse sweep.  With a loss on top
 * the Gauss-Newton matrix has the Hessian M of the loss with respect to the outputs in
 * the middle, G = J^T M J (the reference the paper cites for the method); metric = 0
 * uses M of this file's loss, metric = 1 uses M = I (the paper's literal expression).
 *
 *   f = z (all T*B rows of logits / linear outputs), theta = (Wx, Wh, b, V, c),
 *   gamma = (gWx, gWh, gb, gV, gc) a direction of the same shapes.
 *   forward:  R a_t = gin_t + gb + gWh h_{t-1} + Wh R h_{t-1},  gin_t = gWx[x_t,:] or gWx x_t
 *             R h_t = act'(h_t) * R a_t,   R h_{-1} = 0   (the initial state is a constant)
 *             R z_t = V^T R h_t + gV^T h_t + gc
 *   metric:   softmax-CE  u_n = (p_n * Rz_n - p_n (p_n . Rz_n)) / N,  p_n = softmax(z_n)
 *             linear-MSE  u_n = 2 Rz_n / (N O);      identity  u_n = Rz_n
 *   reverse:  ordinary backpropagation of u in place of d loss / d z.
 * h_all [T+1,B,H] as produced by orc_forward for the same parameters.  Rz_out (nullable,
 * [T*B,O]) receives R z.  Outputs G* have the shapes of the parameters.
 */
int orc_gauss_newton_vec(const orc_dims *d, int metric, const double *Wx, const double *Wh,
                         const double *V, const double *c, const double *gWx, const double *gWh,
                         const double *gb, const double *gV, const double *gc, const void *x,
                         const double *h_all, double *GWx, double *GWh, double *Gb, double *GV,
                         double *Gc, double *Rz_out)
{
    if (!dims_ok(d) || (metric != 0 && metric != 1) || !Wx || !Wh || !V || !c || !gWx || !gWh ||
        !gb || !gV || !gc || !x || !h_all || !GWx || !GWh || !Gb || !GV || !Gc)
        return -1;
    const int H = d->hidden, O = d->out_dim, T = d->seq_len, B = d->batch, D = d->in_dim;
    const long N = (long)T * B;
    const int32_t *ids = (const int32_t *)x;
    const double *X = (const double *)x;
    const size_t wx_elems = d->input_kind == 0 ? (size_t)D * H : (size_t)H * D;
    double *Rh = (double *)calloc((size_t)(T + 1) * B * H, sizeof(double)); /* Rh[0] = R h_{-1} = 0 */
    double *u = (double *)malloc(sizeof(double) * (size_t)N * O);
    double *g = (double *)malloc(sizeof(double) * (size_t)N * H);
    double *delta = (double *)malloc(sizeof(double) * (size_t)N * H);
    double *z = (double *)malloc(sizeof(double) * O);
    if (!Rh || !u || !g || !delta || !z) return -1;

    /* forward sweep of the R-operator */
    for (int t = 0; t < T; ++t)
        for (int bb = 0; bb < B; ++bb) {
            const double *hp = h_all + ((size_t)t * B + bb) * H;
            const double *ht = h_all + ((size_t)(t + 1) * B + bb) * H;
            const double *Rhp = Rh + ((size_t)t * B + bb) * H;
            double *Rht = Rh + ((size_t)(t + 1) * B + bb) * H;
            for (int j = 0; j < H; ++j) {
                double Ra = gb[j];
                if (d->input_kind == 0) {
                    const int32_t v = ids[(size_t)t * B + bb];
                    if (v < 0 || v >= D) return -1;
                    Ra += gWx[(size_t)v * H + j];
                } else {
                    const double *xt = X + ((size_t)t * B + bb) * D;
                    for (int k = 0; k < D; ++k) Ra += gWx[(size_t)j * D + k] * xt[k];
                }
                for (int i = 0; i < H; ++i)
                    Ra += gWh[(size_t)j * H + i] * hp[i] + Wh[(size_t)j * H + i] * Rhp[i];
                const double dact = d->act == 0 ? ht[j] * (1.0 - ht[j]) : 1.0 - ht[j] * ht[j];
                Rht[j] = dact * Ra;
            }
        }

    /* R z, then the loss metric, row by row */
    for (long n = 0; n < N; ++n) {
        const double *h = h_all + (size_t)(n + B) * H;
        const double *Rhn = Rh + (size_t)(n + B) * H;
        double *un = u + (size_t)n * O;
        for (int k = 0; k < O; ++k) {
            double s = gc[k];
            for (int i = 0; i < H; ++i) s += V[(size_t)i * O + k] * Rhn[i] + gV[(size_t)i * O + k] * h[i];
            un[k] = s;
        }
        if (Rz_out)
            for (int k = 0; k < O; ++k) Rz_out[(size_t)n * O + k] = un[k];
        if (metric == 1) continue;
        if (d->loss_kind == 0) {
            logits_row(h, V, c, H, O, z);
            double m = z[0];
            for (int k = 1; k < O; ++k) if (z[k] > m) m = z[k];
            double s = 0.0;
            for (int k = 0; k < O; ++k) s += exp(z[k] - m);
            double dot = 0.0;
            for (int k = 0; k < O; ++k) { z[k] = exp(z[k] - m) / s; dot += z[k] * un[k]; }
            for (int k = 0; k < O; ++k) un[k] = z[k] * (un[k] - dot) / (double)N;
        } else {
            for (int k = 0; k < O; ++k) un[k] = 2.0 * un[k] / ((double)N * O);
        }
    }

    /* reverse sweep: backpropagation of u */
    for (int k = 0; k < O; ++k) Gc[k] = 0.0;
    for (size_t e = 0; e < (size_t)H * O; ++e) GV[e] = 0.0;
    for (long n = 0; n < N; ++n) {
        const double *h = h_all + (size_t)(n + B) * H;
        const double *un = u + (size_t)n * O;
        for (int k = 0; k < O; ++k) Gc[k] += un[k];
        for (int i = 0; i < H; ++i) {
            double s = 0.0;
            for (int k = 0; k < O; ++k) {
                GV[(size_t)i * O + k] += h[i] * un[k];
                s += V[(size_t)i * O + k] * un[k];
            }
            g[(size_t)n * H + i] = s;
        }
    }
    for (int j = 0; j < H; ++j) Gb[j] = 0.0;
    for (size_t e = 0; e < (size_t)H * H; ++e) GWh[e] = 0.0;
    for (size_t e = 0; e < wx_elems; ++e) GWx[e] = 0.0;
    for (int bb = 0; bb < B; ++bb) {
        for (int t = T - 1; t >= 0; --t) {
            const size_t n = (size_t)t * B + bb;
            const double *ht = h_all + ((size_t)(t + 1) * B + bb) * H;
            const double *hp = h_all + ((size_t)t * B + bb) * H;
            double *dl = delta + n * H;
            for (int j = 0; j < H; ++j) {
                double dh = g[n * H + j];
                if (t + 1 < T) {
                    const double *dn = delta + ((size_t)(t + 1) * B + bb) * H;
                    for (int i = 0; i < H; ++i) dh += Wh[(size_t)i * H + j] * dn[i];
                }
                const double dact = d->act == 0 ? ht[j] * (1.0 - ht[j]) : 1.0 - ht[j] * ht[j];
                dl[j] = dh * dact;
            }
            for (int j = 0; j < H; ++j) {
                Gb[j] += dl[j];
                for (int i = 0; i < H; ++i) GWh[(size_t)j * H + i] += dl[j] * hp[i];
                if (d->input_kind == 0) {
                    GWx[(size_t)ids[n] * H + j] += dl[j];
                } else {
                    const double *xt = X + n * D;
                    for (int k = 0; k < D; ++k) GWx[(size_t)j * D + k] += dl[j] * xt[k];
                }
            }
        }
    }
    free(Rh); free(u); free(g); free(delta); free(z);
    return 0;
}
