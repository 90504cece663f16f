/*
 * CPU oracle for the Q-network arithmetic of the DQN hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, direct-from-the-definition double-precision loops: nothing here is blocked, fused
 * or reordered, so each function can be compared with the paper by eye.  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg may build or call this file; the GPU library shares
 * no code with it.
 *
 * What each function follows:
 *   conv/fc forward, greedy policy .... Section 2.1 (Q as a deep CNN, pi(s) = argmax_a Q(s,a));
 *                                        layer shapes are those of the setup the paper adopts
 *                                        (Section 5, "identical to" the Nature-DQN experiment setup)
 *   TD target / loss .................. Eq. 1, with error clipping (Huber, delta) and the terminal
 *                                        mask of the adopted setup
 *   backward .......................... Section 2.1, "first-order minimization with respect to theta"
 *   RMSProp ........................... Appendix B ("centered" RMSProp, both decays equal, constant
 *                                        added to the denominator)
 *
 * Layouts: activations [B, C, H, W]; conv weights [O, C, kh, kw]; fc weights [out, in]; the
 * parameter blob is conv_1.w, conv_1.b, ..., fc_1.w, fc_1.b, ...; ReLU after every layer but the last.
 *
 * Loops marked with an OpenMP pragma run over independent outputs only, so every output keeps its
 * own summation order and the result is bitwise identical for any thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define MAX_LAYERS 4

typedef struct {
    int32_t in_c, in_h, in_w;
    int32_t n_conv;
    int32_t conv_out[MAX_LAYERS], conv_k[MAX_LAYERS], conv_s[MAX_LAYERS];
    int32_t n_fc;
    int32_t fc_out[MAX_LAYERS];
} onet_desc;

static int conv_out_size(int in, int k, int s) { return (in - k) / s + 1; }

/* Per-layer geometry derived from the description. */
typedef struct {
    int n_layers;                 /* n_conv + n_fc */
    int is_conv[2 * MAX_LAYERS];
    int cin[2 * MAX_LAYERS], hin[2 * MAX_LAYERS], win[2 * MAX_LAYERS];
    int cout[2 * MAX_LAYERS], hout[2 * MAX_LAYERS], wout[2 * MAX_LAYERS];
    int k[2 * MAX_LAYERS], s[2 * MAX_LAYERS];
    size_t w_off[2 * MAX_LAYERS], b_off[2 * MAX_LAYERS]; /* offsets into the parameter blob */
    size_t act_off[2 * MAX_LAYERS];                       /* per-sample offset of the layer output */
    size_t act_per_sample;                                /* sum of all layer outputs per sample */
    size_t n_params;
} geom;

static void make_geom(const onet_desc *d, geom *g)
{
    int c = d->in_c, h = d->in_h, w = d->in_w;
    size_t p = 0, a = 0;
    int L = 0;
    for (int i = 0; i < d->n_conv; ++i, ++L) {
        g->is_conv[L] = 1;
        g->cin[L] = c; g->hin[L] = h; g->win[L] = w;
        g->k[L] = d->conv_k[i]; g->s[L] = d->conv_s[i];
        g->cout[L] = d->conv_out[i];
        g->hout[L] = conv_out_size(h, g->k[L], g->s[L]);
        g->wout[L] = conv_out_size(w, g->k[L], g->s[L]);
        g->w_off[L] = p; p += (size_t)g->cout[L] * c * g->k[L] * g->k[L];
        g->b_off[L] = p; p += (size_t)g->cout[L];
        g->act_off[L] = a; a += (size_t)g->cout[L] * g->hout[L] * g->wout[L];
        c = g->cout[L]; h = g->hout[L]; w = g->wout[L];
    }
    int feat = c * h * w;
    for (int i = 0; i < d->n_fc; ++i, ++L) {
        g->is_conv[L] = 0;
        g->cin[L] = feat; g->hin[L] = 1; g->win[L] = 1;
        g->k[L] = 1; g->s[L] = 1;
        g->cout[L] = d->fc_out[i]; g->hout[L] = 1; g->wout[L] = 1;
        g->w_off[L] = p; p += (size_t)g->cout[L] * feat;
        g->b_off[L] = p; p += (size_t)g->cout[L];
        g->act_off[L] = a; a += (size_t)g->cout[L];
        feat = g->cout[L];
    }
    g->n_layers = L;
    g->n_params = p;
    g->act_per_sample = a;
}

size_t onet_num_params(const onet_desc *d) { geom g; make_geom(d, &g); return g.n_params; }
size_t onet_acts_per_sample(const onet_desc *d) { geom g; make_geom(d, &g); return g.act_per_sample; }

/* y[o,i,j] = bias[o] + sum_{c,p,q} w[o,c,p,q] * x[c, i*s+p, j*s+q]   (cross-correlation, no padding) */
static void conv_forward_one(const double *x, const double *w, const double *bias, double *y,
                             int C, int H, int W, int O, int K, int S, int relu)
{
    int Ho = conv_out_size(H, K, S), Wo = conv_out_size(W, K, S);
    for (int o = 0; o < O; ++o)
        for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j) {
                double acc = bias[o];
                for (int c = 0; c < C; ++c)
                    for (int p = 0; p < K; ++p)
                        for (int q = 0; q < K; ++q)
                            acc += w[((o * C + c) * K + p) * K + q] *
                                   x[(c * H + (i * S + p)) * W + (j * S + q)];
                if (relu && acc < 0.0) acc = 0.0;
                y[(o * Ho + i) * Wo + j] = acc;
            }
}

/* y[o] = bias[o] + sum_f w[o,f] * x[f] */
static void fc_forward_one(const double *x, const double *w, const double *bias, double *y,
                           int F, int O, int relu)
{
    for (int o = 0; o < O; ++o) {
        double acc = bias[o];
        for (int f = 0; f < F; ++f) acc += w[(size_t)o * F + f] * x[f];
        if (relu && acc < 0.0) acc = 0.0;
        y[o] = acc;
    }
}

/*
 * Forward pass.  x: [B, in_c, in_h, in_w] (already scaled to [0,1]); theta: parameter blob;
 * acts: [B, acts_per_sample] workspace receiving every layer's post-activation output;
 * q: [B, A] (copy of the last layer's output).
 */
void onet_forward(const onet_desc *d, const double *theta, const double *x, int B,
                  double *acts, double *q)
{
    geom g; make_geom(d, &g);
    size_t in_sz = (size_t)d->in_c * d->in_h * d->in_w;
    int A = g.cout[g.n_layers - 1];
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        const double *in = x + b * in_sz;
        double *a = acts + b * g.act_per_sample;
        for (int L = 0; L < g.n_layers; ++L) {
            int relu = (L != g.n_layers - 1);
            double *out = a + g.act_off[L];
            if (g.is_conv[L])
                conv_forward_one(in, theta + g.w_off[L], theta + g.b_off[L], out,
                                 g.cin[L], g.hin[L], g.win[L], g.cout[L], g.k[L], g.s[L], relu);
            else
                fc_forward_one(in, theta + g.w_off[L], theta + g.b_off[L], out,
                               g.cin[L], g.cout[L], relu);
            in = out;
        }
        for (int k = 0; k < A; ++k) q[(size_t)b * A + k] = in[k];
    }
}

/*
 * Backward pass by the chain rule.  dq: [B, A] = dLoss/dQ.  grad: parameter-blob-shaped output
 * (overwritten).  ReLU'(z) = [z > 0], read off the stored post-activation output (max(z,0) > 0 iff z > 0).
 * dz_all: [B, acts_per_sample] workspace; receives dLoss/d(pre-activation) of every layer.
 */
void onet_backward(const onet_desc *d, const double *theta, const double *x, int B,
                   const double *acts, const double *dq, double *dz_all, double *grad)
{
    geom g; make_geom(d, &g);
    size_t in_sz = (size_t)d->in_c * d->in_h * d->in_w;
    int NL = g.n_layers;
    int A = g.cout[NL - 1];

    /* Pass 1 (per sample, independent): dz for every layer, last to first. */
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        const double *a = acts + b * g.act_per_sample;
        double *dz = dz_all + b * g.act_per_sample;
        for (int k = 0; k < A; ++k) dz[g.act_off[NL - 1] + k] = dq[(size_t)b * A + k];
        for (int L = NL - 1; L >= 1; --L) {
            /* gradient w.r.t. the input of layer L = output of layer L-1, then through ReLU */
            const double *w = theta + g.w_off[L];
            const double *dzo = dz + g.act_off[L];
            const double *ain = a + g.act_off[L - 1];
            double *dzi = dz + g.act_off[L - 1];
            size_t n_in = (size_t)g.cin[L] * g.hin[L] * g.win[L];
            if (g.is_conv[L]) {
                int C = g.cin[L], H = g.hin[L], W = g.win[L], O = g.cout[L], K = g.k[L], S = g.s[L];
                int Ho = g.hout[L], Wo = g.wout[L];
                for (size_t t = 0; t < n_in; ++t) dzi[t] = 0.0;
                for (int o = 0; o < O; ++o)
                    for (int i = 0; i < Ho; ++i)
                        for (int j = 0; j < Wo; ++j) {
                            double go = dzo[(o * Ho + i) * Wo + j];
                            for (int c = 0; c < C; ++c)
                                for (int p = 0; p < K; ++p)
                                    for (int q = 0; q < K; ++q)
                                        dzi[(c * H + (i * S + p)) * W + (j * S + q)] +=
                                            go * w[((o * C + c) * K + p) * K + q];
                        }
            } else {
                int F = g.cin[L], O = g.cout[L];
                for (int f = 0; f < F; ++f) {
                    double acc = 0.0;
                    for (int o = 0; o < O; ++o) acc += dzo[o] * w[(size_t)o * F + f];
                    dzi[f] = acc;
                }
            }
            for (size_t t = 0; t < n_in; ++t)
                if (!(ain[t] > 0.0)) dzi[t] = 0.0;
        }
    }

    /* Pass 2 (per output channel / unit, independent): weight and bias gradients, summed over b. */
    for (int L = 0; L < NL; ++L) {
        double *gw = grad + g.w_off[L];
        double *gb = grad + g.b_off[L];
        if (g.is_conv[L]) {
            int C = g.cin[L], H = g.hin[L], W = g.win[L], O = g.cout[L], K = g.k[L], S = g.s[L];
            int Ho = g.hout[L], Wo = g.wout[L];
#pragma omp parallel for schedule(static)
            for (int o = 0; o < O; ++o) {
                double accb = 0.0;
                for (int b = 0; b < B; ++b) {
                    const double *dzo = dz_all + b * g.act_per_sample + g.act_off[L];
                    for (int i = 0; i < Ho; ++i)
                        for (int j = 0; j < Wo; ++j) accb += dzo[(o * Ho + i) * Wo + j];
                }
                gb[o] = accb;
                for (int c = 0; c < C; ++c)
                    for (int p = 0; p < K; ++p)
                        for (int q = 0; q < K; ++q) {
                            double acc = 0.0;
                            for (int b = 0; b < B; ++b) {
                                const double *in = (L == 0) ? x + b * in_sz
                                    : acts + b * g.act_per_sample + g.act_off[L - 1];
                                const double *dzo = dz_all + b * g.act_per_sample + g.act_off[L];
                                for (int i = 0; i < Ho; ++i)
                                    for (int j = 0; j < Wo; ++j)
                                        acc += dzo[(o * Ho + i) * Wo + j] *
                                               in[(c * H + (i * S + p)) * W + (j * S + q)];
                            }
                            gw[((o * C + c) * K + p) * K + q] = acc;
                        }
            }
        } else {
            int F = g.cin[L], O = g.cout[L];
#pragma omp parallel for schedule(static)
            for (int o = 0; o < O; ++o) {
                double accb = 0.0;
                for (int b = 0; b < B; ++b)
                    accb += dz_all[b * g.act_per_sample + g.act_off[L] + o];
                gb[o] = accb;
                for (int f = 0; f < F; ++f) {
                    double acc = 0.0;
                    for (int b = 0; b < B; ++b) {
                        const double *in = (L == 0) ? x + b * in_sz
                            : acts + b * g.act_per_sample + g.act_off[L - 1];
                        acc += dz_all[b * g.act_per_sample + g.act_off[L] + o] * in[f];
                    }
                    gw[(size_t)o * F + f] = acc;
                }
            }
        }
    }
}

/* Lowest-index argmax of a row (inputs are finite). */
static int argmax_row(const double *row, int A)
{
    int best = 0;
    for (int k = 1; k < A; ++k)
        if (row[k] > row[best]) best = k;
    return best;
}

void greedy_actions(const double *q, int B, int A, int32_t *out)
{
    for (int b = 0; b < B; ++b) out[b] = argmax_row(q + (size_t)b * A, A);
}

/*
 * TD target, clipped (Huber) loss and dLoss/dQ for a minibatch (Eq. 1 with the terminal mask).
 *   q_sa      [B, A]  Q(s, . ; theta)
 *   q_next_t  [B, A]  Q(s', . ; theta^-)
 *   q_next_o  [B, A] or NULL.  NULL: y = r + gamma (1-done) max_a' q_next_t.
 *             non-NULL (Double-DQN): a* = lowest-index argmax_a q_next_o; y = r + gamma (1-done) q_next_t[a*].
 *   delta_b = Q(s_b, a_b) - y_b;  loss = (1/B) sum_b huber(delta_b);  dq[b, a_b] = clip(delta_b, -h, h)/B.
 * Outputs y[B], td[B], dq[B, A]; returns the batch-mean loss.  No gradient flows into y.
 */
double td_loss(const double *q_sa, const double *q_next_t, const double *q_next_o,
               const int32_t *a, const double *r, const double *done,
               double gamma, double huber, int B, int A,
               double *y, double *td, double *dq)
{
    double loss = 0.0;
    for (int b = 0; b < B; ++b) {
        const double *qt = q_next_t + (size_t)b * A;
        double boot;
        if (q_next_o) boot = qt[argmax_row(q_next_o + (size_t)b * A, A)];
        else          boot = qt[argmax_row(qt, A)];
        y[b] = r[b] + gamma * (1.0 - done[b]) * boot;
        double dl = q_sa[(size_t)b * A + a[b]] - y[b];
        td[b] = dl;
        double ad = fabs(dl);
        loss += (ad <= huber) ? 0.5 * dl * dl : huber * (ad - 0.5 * huber);
        double clipped = dl > huber ? huber : (dl < -huber ? -huber : dl);
        for (int k = 0; k < A; ++k) dq[(size_t)b * A + k] = 0.0;
        dq[(size_t)b * A + a[b]] = clipped / (double)B;
    }
    return loss / (double)B;
}

/*
 * RMSProp (Appendix B).  centered: m <- alpha m + (1-alpha) g;  v <- alpha v + (1-alpha) g^2;
 * theta <- theta - lr * g / (sqrt(max(v - m^2, 0)) + eps).  Not centered: the m terms are dropped.
 */
void rmsprop_step(double *theta, const double *g, double *v, double *m, size_t n,
                  double lr, double alpha, double eps, int centered)
{
    for (size_t i = 0; i < n; ++i) {
        v[i] = alpha * v[i] + (1.0 - alpha) * g[i] * g[i];
        double var = v[i];
        if (centered) {
            m[i] = alpha * m[i] + (1.0 - alpha) * g[i];
            var = v[i] - m[i] * m[i];
            if (var < 0.0) var = 0.0;
        }
        theta[i] -= lr * g[i] / (sqrt(var) + eps);
    }
}

/* Number of threads the OpenMP loops above will use (reported by the benchmark's CPU leg). */
#ifdef _OPENMP
#include <omp.h>
int oracle_max_threads(void) { return omp_get_max_threads(); }
/* Thread count of the loops above from now on (n >= 1); results do not depend on it.  Returns the previous count. */
int oracle_set_threads(int n) { int old = omp_get_max_threads(); if (n >= 1) omp_set_num_threads(n); return old; }
#else
int oracle_max_threads(void) { return 1; }
int oracle_set_threads(int n) { (void)n; return 1; }
#endif
