/*
 * CPU oracle for the dense part of the DLRM train step (bottom MLP, pairwise-dot
 * interaction, top MLP, sigmoid + mean binary cross-entropy, backward, SGD).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: plain loops in double precision,
 * written so that they can be checked by eye.  Only the tests, the smoke check
 * and the benchmark's baseline leg may call it; it shares nothing with the GPU
 * library.
 *
 * What the paper fixes (model-architecture table, Fig. 1(a)): the DLRM layout --
 * a bottom MLP over the dense features, 26 embedding tables, a feature
 * interaction, a top MLP producing a click probability -- and the layer widths
 * (Kaggle: 13-512-256-64-16 and 512-256-1 on top of the 367-wide interaction).
 * What it leaves open, and the reading taken: ReLU after every bottom layer and
 * after every top layer but the last; the interaction is DLRM's pairwise dot
 * product of the V = T+1 vectors [bottom output, table 0..T-1], strictly lower
 * triangle in row-major order (i = 1..V-1, j = 0..i-1), appended after the bottom
 * output; loss = mean binary cross-entropy with log arguments clamped at 1e-12;
 * plain SGD, the gradients being those of the weights before the step.
 *
 * Parity pin (tests/test_oracle_dense_pins.py): the same network written with
 * torch (float64 CPU tensors, autograd) -- loss, gradient w.r.t. the pooled
 * embeddings and the updated parameters agree to 1e-12.
 *
 * The quantised variants of the dense part (distributed-training section and the
 * model-quantisation appendix of the paper):
 *   oracle_mlp_fake_quant     channel-wise (one scale per output row) INT4 / INT8
 *                             fake quantisation of a linear layer's weights; the
 *                             forward and the input gradients use the quantised
 *                             weights, the step goes to the fp32 weights
 *                             (straight-through), activations stay unquantised;
 *   oracle_mlp_grad_quant_ec  per-tensor INT8 quantisation of an MLP gradient with
 *                             error compensation.  The paper only cites the scheme
 *                             (error feedback); the reading taken: the residual of
 *                             the previous step is added before quantising,
 *                             g' = g + e;  q = Q(g');  e <- g' - s*q;  the step uses s*q.
 * Both decide integer codes, so they compute in binary32 (one rounding per
 * operation), like the embedding oracle.  Pins: tests/test_oracle_mlp_quant_pins.py
 * (the scalar quantiser and the table-wise routines of the embedding oracle on the
 * same numbers, closed-form invariants, the telescoping sum of error feedback, hand
 * examples under tests/golden/, torch autograd with a straight-through weight).
 *
 * Build: gcc -O2 -ffp-contract=off -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* y[b][o] = act(sum_i x[b][i] * W[o][i] + bias[o]) */
static void linear_fwd(const double *x, const double *W, const double *bias, double *y, int B, int in, int out,
                       int relu)
{
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < out; ++o) {
            double s = bias[o];
            for (int i = 0; i < in; ++i) s += x[(size_t)b * in + i] * W[(size_t)o * in + i];
            y[(size_t)b * out + o] = (relu && s < 0.0) ? 0.0 : s;
        }
}

/* given dz (gradient w.r.t. the layer's pre-activation): dx through the weights Wf the forward used, the
 * gradients gw / gb (stored if the pointers are given), and -- if asked -- the SGD step on W and bias */
static void linear_bwd(const double *dz, const double *x, const double *Wf, double *W, double *bias, double *dx, int B,
                       int in, int out, double lr, int apply_sgd, double *gw_out, double *gb_out)
{
    if (dx)
        for (int b = 0; b < B; ++b)
            for (int i = 0; i < in; ++i) {
                double s = 0.0;
                for (int o = 0; o < out; ++o) s += dz[(size_t)b * out + o] * Wf[(size_t)o * in + i];
                dx[(size_t)b * in + i] = s;
            }
    for (int o = 0; o < out; ++o) {
        double gb = 0.0;
        for (int b = 0; b < B; ++b) gb += dz[(size_t)b * out + o];
        for (int i = 0; i < in; ++i) {
            double gw = 0.0;
            for (int b = 0; b < B; ++b) gw += dz[(size_t)b * out + o] * x[(size_t)b * in + i];
            if (gw_out) gw_out[(size_t)o * in + i] = gw;
            if (apply_sgd) W[(size_t)o * in + i] -= lr * gw;
        }
        if (gb_out) gb_out[o] = gb;
        if (apply_sgd) bias[o] -= lr * gb;
    }
}

/*
 * All matrices row-major.  bot_w / top_w: arrays of pointers to double matrices
 * [dims[l+1]][dims[l]] (updated in place); bot_b / top_b likewise.
 * Returns the loss; grad_emb [B][T][D] receives d loss / d emb.
 *
 * The general form.  bot_wf / top_wf: the weights the forward and the input gradients use (NULL: the
 * master weights bot_w / top_w; otherwise e.g. their fake-quantised copies).  apply_sgd: whether the master
 * weights and biases take the step.  bot_gw / bot_gb / top_gw / top_gb: arrays of pointers that receive the
 * gradients (NULL: not wanted).
 */
double oracle_dense_step_ex(int B, int num_dense, int T, int D, int bot_layers, const int32_t *bot_dims,
                            double **bot_w, double **bot_b, int top_layers, const int32_t *top_dims, double **top_w,
                            double **top_b, const double *dense_x, const double *emb, const double *labels, double lr,
                            double *grad_emb, double **bot_wf, double **top_wf, int apply_sgd, double **bot_gw,
                            double **bot_gb, double **top_gw, double **top_gb)
{
    if (!bot_wf) bot_wf = bot_w;
    if (!top_wf) top_wf = top_w;
    const int V = T + 1, P = V * (V - 1) / 2, RW = D + P;
    (void)num_dense;
    /* ---- forward */
    double **ba = (double **)calloc((size_t)bot_layers + 1, sizeof(double *));
    double **ta = (double **)calloc((size_t)top_layers + 1, sizeof(double *));
    ba[0] = (double *)dense_x;
    for (int l = 0; l < bot_layers; ++l) {
        ba[l + 1] = (double *)malloc(sizeof(double) * (size_t)B * bot_dims[l + 1]);
        linear_fwd(ba[l], bot_wf[l], bot_b[l], ba[l + 1], B, bot_dims[l], bot_dims[l + 1], 1);
    }
    double *Z = (double *)malloc(sizeof(double) * (size_t)B * V * D); /* [B][V][D] */
    double *R = (double *)malloc(sizeof(double) * (size_t)B * RW);
    for (int b = 0; b < B; ++b) {
        double *z = Z + (size_t)b * V * D;
        for (int d = 0; d < D; ++d) z[d] = ba[bot_layers][(size_t)b * D + d];
        for (int t = 0; t < T; ++t)
            for (int d = 0; d < D; ++d) z[(t + 1) * D + d] = emb[((size_t)b * T + t) * D + d];
        double *r = R + (size_t)b * RW;
        for (int d = 0; d < D; ++d) r[d] = z[d];
        int p = 0;
        for (int i = 1; i < V; ++i)
            for (int j = 0; j < i; ++j) {
                double s = 0.0;
                for (int d = 0; d < D; ++d) s += z[i * D + d] * z[j * D + d];
                r[D + p++] = s;
            }
    }
    ta[0] = R;
    for (int l = 0; l < top_layers; ++l) {
        ta[l + 1] = (double *)malloc(sizeof(double) * (size_t)B * top_dims[l + 1]);
        linear_fwd(ta[l], top_wf[l], top_b[l], ta[l + 1], B, top_dims[l], top_dims[l + 1], l + 1 < top_layers);
    }
    /* ---- loss and its gradient w.r.t. the logit */
    double loss = 0.0;
    double *dz = (double *)malloc(sizeof(double) * (size_t)B);
    for (int b = 0; b < B; ++b) {
        double p = 1.0 / (1.0 + exp(-ta[top_layers][b]));
        double y = labels[b];
        double lp = log(p > 1e-12 ? p : 1e-12), lq = log(1.0 - p > 1e-12 ? 1.0 - p : 1e-12);
        loss += -(y * lp + (1.0 - y) * lq);
        dz[b] = (p - y) / (double)B;
    }
    loss /= (double)B;
    /* ---- backward through the top MLP */
    double *g = dz; /* gradient w.r.t. the pre-activation of the current layer */
    for (int l = top_layers - 1; l >= 0; --l) {
        double *dx = (double *)malloc(sizeof(double) * (size_t)B * top_dims[l]);
        linear_bwd(g, ta[l], top_wf[l], top_w[l], top_b[l], dx, B, top_dims[l], top_dims[l + 1], lr, apply_sgd,
                   top_gw ? top_gw[l] : NULL, top_gb ? top_gb[l] : NULL);
        if (l > 0) /* ta[l] is a ReLU output */
            for (size_t e = 0; e < (size_t)B * top_dims[l]; ++e)
                if (!(ta[l][e] > 0.0)) dx[e] = 0.0;
        free(g);
        g = dx;
    }
    /* ---- backward through the interaction: g = dR [B][RW] */
    double *dbot = (double *)malloc(sizeof(double) * (size_t)B * D);
    for (int b = 0; b < B; ++b) {
        const double *z = Z + (size_t)b * V * D;
        const double *dr = g + (size_t)b * RW;
        double *dZ = (double *)calloc((size_t)V * D, sizeof(double));
        for (int d = 0; d < D; ++d) dZ[d] += dr[d];
        int p = 0;
        for (int i = 1; i < V; ++i)
            for (int j = 0; j < i; ++j) {
                for (int d = 0; d < D; ++d) {
                    dZ[i * D + d] += dr[D + p] * z[j * D + d];
                    dZ[j * D + d] += dr[D + p] * z[i * D + d];
                }
                ++p;
            }
        for (int d = 0; d < D; ++d) /* the bottom output is a ReLU output */
            dbot[(size_t)b * D + d] = ba[bot_layers][(size_t)b * D + d] > 0.0 ? dZ[d] : 0.0;
        for (int t = 0; t < T; ++t)
            for (int d = 0; d < D; ++d) grad_emb[((size_t)b * T + t) * D + d] = dZ[(t + 1) * D + d];
        free(dZ);
    }
    free(g);
    /* ---- backward through the bottom MLP */
    g = dbot;
    for (int l = bot_layers - 1; l >= 0; --l) {
        double *dx = l > 0 ? (double *)malloc(sizeof(double) * (size_t)B * bot_dims[l]) : NULL;
        linear_bwd(g, ba[l], bot_wf[l], bot_w[l], bot_b[l], dx, B, bot_dims[l], bot_dims[l + 1], lr, apply_sgd,
                   bot_gw ? bot_gw[l] : NULL, bot_gb ? bot_gb[l] : NULL);
        if (l > 0)
            for (size_t e = 0; e < (size_t)B * bot_dims[l]; ++e)
                if (!(ba[l][e] > 0.0)) dx[e] = 0.0;
        free(g);
        g = dx;
    }
    for (int l = 1; l <= bot_layers; ++l) free(ba[l]);
    for (int l = 1; l <= top_layers; ++l) free(ta[l]);
    free(ba);
    free(ta);
    free(Z);
    free(R);
    return loss;
}

/* the plain fp32-weight train step */
double oracle_dense_step(int B, int num_dense, int T, int D, int bot_layers, const int32_t *bot_dims, double **bot_w,
                         double **bot_b, int top_layers, const int32_t *top_dims, double **top_w, double **top_b,
                         const double *dense_x, const double *emb, const double *labels, double lr, double *grad_emb)
{
    return oracle_dense_step_ex(B, num_dense, T, D, bot_layers, bot_dims, bot_w, bot_b, top_layers, top_dims, top_w,
                                top_b, dense_x, emb, labels, lr, grad_emb, NULL, NULL, 1, NULL, NULL, NULL, NULL);
}

/* ---- channel-wise fake quantisation of a linear layer's weights (binary32) ----
 * W [out][in] row-major.  Per output row o:  a = max_i |W[o][i]|,  s_o = max(a / qmax, 1e-8) with
 * qmax = 2^(bits-1) - 1;  code = clamp(rint(W / s_o), -2^(bits-1), qmax);  Wq = s_o * code.
 * row_scale [out] and codes [out][in] are optional outputs. */
void oracle_mlp_fake_quant(const float *W, int out, int in, int bits, float *Wq, float *row_scale, int8_t *codes)
{
    const float qmax = (float)((1 << (bits - 1)) - 1), qmin = -(float)(1 << (bits - 1));
    for (int o = 0; o < out; ++o) {
        float a = 0.0f;
        for (int i = 0; i < in; ++i) {
            const float m = fabsf(W[(size_t)o * in + i]);
            if (m > a) a = m;
        }
        float s = a / qmax;
        if (s < 1e-8f) s = 1e-8f;
        if (row_scale) row_scale[o] = s;
        for (int i = 0; i < in; ++i) {
            float q = rintf(W[(size_t)o * in + i] / s);
            if (q < qmin) q = qmin;
            if (q > qmax) q = qmax;
            if (codes) codes[(size_t)o * in + i] = (int8_t)q;
            Wq[(size_t)o * in + i] = s * q;
        }
    }
}

/* ---- INT8 quantisation of one parameter tensor's gradient with error compensation (binary32) ----
 * g [n] the gradient, err [n] the residual carried from the previous step (NULL: none is kept),
 * param [n] the parameter.  g' = g + err;  s = max(max|g'| / 127, 1e-8);  code = clamp(rint(g' / s), -128, 127);
 * err <- g' - s * code;  param <- param - lr * (s * code).  Returns s. */
float oracle_mlp_grad_quant_ec(int64_t n, const float *g, float *err, float *param, float lr, int8_t *codes)
{
    float a = 0.0f;
    for (int64_t k = 0; k < n; ++k) {
        const float gp = err ? g[k] + err[k] : g[k];
        const float m = fabsf(gp);
        if (m > a) a = m;
    }
    float s = a / 127.0f;
    if (s < 1e-8f) s = 1e-8f;
    for (int64_t k = 0; k < n; ++k) {
        const float gp = err ? g[k] + err[k] : g[k];
        float q = rintf(gp / s);
        if (q < -128.0f) q = -128.0f;
        if (q > 127.0f) q = 127.0f;
        const int8_t c = (int8_t)q;
        if (codes) codes[k] = c;
        const float deq = s * (float)c;
        if (err) err[k] = gp - deq;
        const float step = lr * deq;
        param[k] = param[k] - step;
    }
    return s;
}
