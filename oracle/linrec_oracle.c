/*
 * linrec_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain sequential fp64 evaluation of the diagonal linear recurrence of
 * arXiv 1709.04057 and of its gradients.  It exists so that the GPU library
 * can be checked against something obviously correct; only the tests, the
 * smoke check and the cpu_baseline leg of the benchmark may call it.  It
 * shares no source, header, table or helper with the GPU path.
 *
 * Storage convention used by every function here
 *   - tensors are row-major [T, C]: element (t, c) at t*C + c, C = B*n
 *     independent columns (the layout of Section 3.1.1: T vectors of B*n elements);
 *   - 0-based row t holds the paper's lambda_{t+1}, x_{t+1}, h_{t+1};
 *     h0 is the paper's h_0 and is an input, never an output row
 *     (the SCAN definition in Section 1 returns n outputs for n inputs);
 *   - inputs are fp32 and are widened exactly to fp64; all arithmetic and
 *     all outputs are fp64 (round-to-nearest; build with -ffp-contract=off).
 *
 * Every function works on the column range [c0, c1) and the row slab
 * [t0, t1) of the full tensors, carrying the recurrence state in a caller
 * supplied fp64 vector, so that big problems can be streamed through in
 * slabs and columns can be handed to several host threads.  Rows are never
 * split across threads: time is always walked sequentially.
 *
 * Pins (tests/test_oracle_pins.py): exact rational closed form by brute
 * force (T <= 64), lambda==0, lambda==1 vs numpy.cumsum, geometric series,
 * scipy.signal.lfilter, backward closed form by brute force, reversed
 * cumprod, finite differences, adjoint identity, row perturbation, slab and
 * column split invariance.  The gated (GILR) form further down is pinned by
 * the exact dyadic case g_pre == 0, the moving-average closed form, the
 * convex-hull invariant, reduction to the plain recurrence above through
 * scipy.special.expit / numpy.tanh, and central finite differences of its own
 * forward pass for every gradient.  The LSTM-cell form at the end is pinned
 * the same way (exact dyadic case, closed forms, finite differences, reduction
 * to the plain recurrence, planted mistakes; tests/test_lstm_oracle_pins.py).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/*
 * Forward recurrence (Section 2: each state is the elementwise product of lambda_t
 * with the previous state, plus x_t; Algorithm 1 fixes the initial value: C_{-1} = h_0).
 *
 *   state[c]      on entry: h at row t0-1 (h0 when t0 == 0), fp64
 *                 on exit : h at row t1-1
 *   href          fp64 [T, C] (full-size array); rows [t0,t1), columns
 *                 [c0,c1) are written
 */
void linrec_oracle_forward(const float *lambda, const float *x,
                           double *state, double *href,
                           int64_t T, int64_t C,
                           int64_t t0, int64_t t1, int64_t c0, int64_t c1)
{
    (void)T;
    for (int64_t t = t0; t < t1; ++t) {
        const float *lt = lambda + (size_t)t * (size_t)C;
        const float *xt = x + (size_t)t * (size_t)C;
        double *ht = href + (size_t)t * (size_t)C;
        for (int64_t c = c0; c < c1; ++c) {
            double s = (double)lt[c] * state[c] + (double)xt[c];
            state[c] = s;
            ht[c] = s;
        }
    }
}

/*
 * Backward pass (Section 2.2).  With e = dL/dh (the direct
 * upstream gradient) and g_t the accumulated gradient nabla_{h_t} L:
 *
 *   g_{T-1} = e_{T-1}                                   (last row: no successor)
 *   g_t     = lambda_{t+1} * g_{t+1} + e_t
 *   grad_x_t      = g_t
 *   grad_lambda_t = h_{t-1} * g_t          (h_{-1} = h0, zero if h0 == NULL)
 *   grad_h0       = lambda_0 * g_0
 *
 * Rows are walked from t1-1 down to t0.
 *
 *   gstate[c]     on entry: g at row t1 (ignored when t1 == T: row T of
 *                 lambda does not exist and is never read)
 *                 on exit : g at row t0
 *   h             fp32 [T, C]: the forward output handed to the backward pass
 *   gx, glam      fp64 [T, C] full-size; rows [t0,t1), columns [c0,c1) written
 *   gh0           fp64 [C]; written only when t0 == 0
 */
void linrec_oracle_backward(const float *lambda, const float *h,
                            const float *h0, const float *e,
                            double *gstate,
                            double *gx, double *glam, double *gh0,
                            int64_t T, int64_t C,
                            int64_t t0, int64_t t1, int64_t c0, int64_t c1)
{
    for (int64_t t = t1 - 1; t >= t0; --t) {
        const float *et = e + (size_t)t * (size_t)C;
        const float *lnext = (t + 1 < T) ? lambda + (size_t)(t + 1) * (size_t)C : NULL;
        const float *hprev = (t > 0) ? h + (size_t)(t - 1) * (size_t)C : h0;
        double *gxt = gx + (size_t)t * (size_t)C;
        double *glt = glam + (size_t)t * (size_t)C;
        for (int64_t c = c0; c < c1; ++c) {
            double g = (double)et[c];
            if (lnext)
                g += (double)lnext[c] * gstate[c];
            gstate[c] = g;
            gxt[c] = g;
            glt[c] = g * (hprev ? (double)hprev[c] : 0.0);
        }
    }
    if (t0 == 0 && t1 > 0) {
        for (int64_t c = c0; c < c1; ++c)
            gh0[c] = (double)lambda[c] * gstate[c];
    }
}

/*
 * Gated impulse linear recurrent layer (Section 3.1), the part after the two matrix products: from the
 * pre-activations g_pre = U x_t + b_g and i_pre = V x_t + b_z,
 *
 *   g_t = sigmoid(g_pre_t)        i_t = tau(i_pre_t)
 *   h_t = g_t * h_{t-1} + (1 - g_t) * i_t
 *
 * tau is tanh (tau != 0) or the identity (tau == 0); the paper leaves tau open.
 * Same storage, slab and state conventions as linrec_oracle_forward.
 */
static double sigmoid_f64(double z) { return 1.0 / (1.0 + exp(-z)); }

void linrec_oracle_gilr_forward(const float *g_pre, const float *i_pre, int tau,
                                double *state, double *href,
                                int64_t T, int64_t C,
                                int64_t t0, int64_t t1, int64_t c0, int64_t c1)
{
    (void)T;
    for (int64_t t = t0; t < t1; ++t) {
        const float *gt = g_pre + (size_t)t * (size_t)C;
        const float *it = i_pre + (size_t)t * (size_t)C;
        double *ht = href + (size_t)t * (size_t)C;
        for (int64_t c = c0; c < c1; ++c) {
            double g = sigmoid_f64((double)gt[c]);
            double i = tau ? tanh((double)it[c]) : (double)it[c];
            double s = g * state[c] + (1.0 - g) * i;
            state[c] = s;
            ht[c] = s;
        }
    }
}

/*
 * Gradients of the layer above with respect to its pre-activations (chain
 * rule through Section 2.2's backward recurrence).  With e = dL/dh (direct)
 * and d_t the accumulated gradient nabla_{h_t} L:
 *
 *   d_{T-1} = e_{T-1},   d_t = g_{t+1} * d_{t+1} + e_t
 *   dL/dg_t = d_t * (h_{t-1} - i_t)          (g_t also scales the impulse)
 *   dL/di_t = d_t * (1 - g_t)
 *   grad_g_pre_t = dL/dg_t * g_t * (1 - g_t)                 (sigmoid')
 *   grad_i_pre_t = dL/di_t * (1 - i_t^2)   (tanh')   or  dL/di_t  (identity)
 *   grad_h0      = g_0 * d_0
 *
 * h is the fp32 forward output handed to the backward pass; rows are walked
 * from t1-1 down to t0; dstate carries d in and out like gstate above.
 */
void linrec_oracle_gilr_backward(const float *g_pre, const float *i_pre, int tau,
                                 const float *h, const float *h0, const float *e,
                                 double *dstate,
                                 double *gg, double *gi, double *gh0,
                                 int64_t T, int64_t C,
                                 int64_t t0, int64_t t1, int64_t c0, int64_t c1)
{
    for (int64_t t = t1 - 1; t >= t0; --t) {
        const float *et = e + (size_t)t * (size_t)C;
        const float *gt = g_pre + (size_t)t * (size_t)C;
        const float *it = i_pre + (size_t)t * (size_t)C;
        const float *gnext = (t + 1 < T) ? g_pre + (size_t)(t + 1) * (size_t)C : NULL;
        const float *hprev = (t > 0) ? h + (size_t)(t - 1) * (size_t)C : h0;
        double *ggt = gg + (size_t)t * (size_t)C;
        double *git = gi + (size_t)t * (size_t)C;
        for (int64_t c = c0; c < c1; ++c) {
            double d = (double)et[c];
            if (gnext)
                d += sigmoid_f64((double)gnext[c]) * dstate[c];
            dstate[c] = d;
            double g = sigmoid_f64((double)gt[c]);
            double i = tau ? tanh((double)it[c]) : (double)it[c];
            double hp = hprev ? (double)hprev[c] : 0.0;
            ggt[c] = d * (hp - i) * (g * (1.0 - g));
            git[c] = d * (1.0 - g) * (tau ? (1.0 - i * i) : 1.0);
        }
    }
    if (t0 == 0 && t1 > 0) {
        for (int64_t c = c0; c < c1; ++c)
            gh0[c] = sigmoid_f64((double)g_pre[c]) * dstate[c];
    }
}

/*
 * Cell of the GILR-LSTM (Section 3.2: the LSTM equations with the
 * gates computed from the surrogate state), the part after the matrix products.  From the
 * pre-activations of the forget, input and output gates and of the candidate,
 *
 *   f_t = sigmoid(f_pre_t)   i_t = sigmoid(i_pre_t)   o_t = sigmoid(o_pre_t)   z_t = tanh(z_pre_t)
 *   c_t = f_t * c_{t-1} + i_t * z_t                   h_t = o_t * c_t
 *
 * state[] carries c (c_0 on entry when t0 == 0).  cref, href: fp64 [T, C], rows [t0,t1) written.
 */
void linrec_oracle_lstm_forward(const float *f_pre, const float *i_pre, const float *z_pre,
                                const float *o_pre, double *state, double *cref, double *href,
                                int64_t T, int64_t C,
                                int64_t t0, int64_t t1, int64_t c0, int64_t c1)
{
    (void)T;
    for (int64_t t = t0; t < t1; ++t) {
        const size_t row = (size_t)t * (size_t)C;
        for (int64_t c = c0; c < c1; ++c) {
            double f = sigmoid_f64((double)f_pre[row + c]);
            double i = sigmoid_f64((double)i_pre[row + c]);
            double o = sigmoid_f64((double)o_pre[row + c]);
            double z = tanh((double)z_pre[row + c]);
            double s = f * state[c] + i * z;
            state[c] = s;
            cref[row + c] = s;
            href[row + c] = o * s;
        }
    }
}

/*
 * Gradients of the cell with respect to its four pre-activations and c_0, for an upstream
 * gradient e = dL/dh (c_t reaches the loss only through h_t and c_{t+1}).  With d_t the
 * accumulated gradient nabla_{c_t} L (Section 2.2's reverse recurrence on the cell state):
 *
 *   d_t = e_t * o_t + f_{t+1} * d_{t+1}                    (no second term for t = T-1)
 *   grad_o_pre_t = e_t * c_t * o_t (1 - o_t)
 *   grad_f_pre_t = d_t * c_{t-1} * f_t (1 - f_t)           (c_{-1} = c0, zero if NULL)
 *   grad_i_pre_t = d_t * z_t * i_t (1 - i_t)
 *   grad_z_pre_t = d_t * i_t * (1 - z_t^2)
 *   grad_c0      = f_0 * d_0
 *
 * cst is the fp32 cell state the forward pass stored; rows walked from t1-1 down to t0.
 */
void linrec_oracle_lstm_backward(const float *f_pre, const float *i_pre, const float *z_pre,
                                 const float *o_pre, const float *cst, const float *c0v,
                                 const float *e, double *dstate,
                                 double *gf, double *gi, double *gz, double *go, double *gc0,
                                 int64_t T, int64_t C,
                                 int64_t t0, int64_t t1, int64_t c0, int64_t c1)
{
    for (int64_t t = t1 - 1; t >= t0; --t) {
        const size_t row = (size_t)t * (size_t)C;
        const float *fnext = (t + 1 < T) ? f_pre + (size_t)(t + 1) * (size_t)C : NULL;
        const float *cprev = (t > 0) ? cst + (size_t)(t - 1) * (size_t)C : c0v;
        for (int64_t c = c0; c < c1; ++c) {
            double f = sigmoid_f64((double)f_pre[row + c]);
            double i = sigmoid_f64((double)i_pre[row + c]);
            double o = sigmoid_f64((double)o_pre[row + c]);
            double z = tanh((double)z_pre[row + c]);
            double d = (double)e[row + c] * o;
            if (fnext)
                d += sigmoid_f64((double)fnext[c]) * dstate[c];
            dstate[c] = d;
            go[row + c] = (double)e[row + c] * (double)cst[row + c] * (o * (1.0 - o));
            gf[row + c] = d * (cprev ? (double)cprev[c] : 0.0) * (f * (1.0 - f));
            gi[row + c] = d * z * (i * (1.0 - i));
            gz[row + c] = d * i * (1.0 - z * z);
        }
    }
    if (t0 == 0 && t1 > 0) {
        for (int64_t c = c0; c < c1; ++c)
            gc0[c] = sigmoid_f64((double)f_pre[c]) * dstate[c];
    }
}

int linrec_oracle_version(void) { return 3; }
