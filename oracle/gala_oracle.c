/*
 * gala_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision CPU statement of what one GALA-A2C round
 * computes (Algorithm 1 of "Gossip-based Actor-Learner Architectures for Deep
 * Reinforcement Learning"): per-agent n-step returns and advantages, the A2C
 * loss (TD loss Eq. (1) + batched policy gradient with entropy Eq. (4)), its
 * gradient through the 3-conv / 1-hidden / two-head network of App. C.2, global
 * gradient-norm clipping and RMSprop (Table 2), and the gossip mixing step
 * x_i <- (x_i + sum_j m_j) / (1 + |N_in_i|) (Algorithm 1, Sec. 2 "Gossip
 * algorithms", Eq. (6) for delayed messages).
 *
 * Nothing here is shared with the GPU library: no headers, helpers, tables or
 * constants.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  Every loop is the textbook definition; the only concession to
 * run time is "omp parallel for" over independent frames / output rows, which
 * does not change any summation order.
 *
 * Where the paper is silent the following readings are used (both sides of a
 * parity test follow them):
 *   - inputs are bytes scaled by 1/255; convolutions are unpadded
 *     cross-correlations followed by ReLU; the hidden layer is followed by ReLU;
 *     the flatten order is channel, row, column;
 *   - every sample of a T-step rollout bootstraps from the single state reached
 *     after the last action, and a terminal transition cuts the return;
 *   - returns and advantages are constants for differentiation (theta_t in
 *     Eq. (1), (2));
 *   - the three loss terms are means over all T*B samples; the entropy enters
 *     as a bonus (loss = pg + c_v * td - eta * H), following the text of Sec. 2
 *     ("prevents premature convergence to deterministic policies");
 *   - clip scale = min(1, c / (norm + 1e-6)); RMSprop keeps v <- a v + (1-a) g^2
 *     and steps x <- x - lr g / (sqrt(v) + eps), no momentum (Table 2).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_CONV 4

typedef struct {
    int in_c, in_h, in_w;
    int n_conv;
    int conv_out[ORC_MAX_CONV];
    int conv_k[ORC_MAX_CONV];
    int conv_stride[ORC_MAX_CONV];
    int fc;
    int n_actions;
} orc_net;

typedef struct {
    int T, B;
    double gamma, vf_coef, ent_coef;
    double lr, rms_alpha, rms_eps, max_grad_norm;
} orc_hparams;

/* ---- shapes ------------------------------------------------------------ */

typedef struct {
    int c[ORC_MAX_CONV + 1], h[ORC_MAX_CONV + 1], w[ORC_MAX_CONV + 1]; /* [0] = input */
    long act_off[ORC_MAX_CONV + 2]; /* offsets of conv outputs and hidden inside a frame's record */
    long act_size;                  /* doubles per frame: input + conv outputs + hidden */
    long in_size;
    long flat;                      /* inputs of the hidden layer */
    long w_off[ORC_MAX_CONV], b_off[ORC_MAX_CONV];
    long fcw_off, fcb_off, piw_off, pib_off, vw_off, vb_off;
    long d;
} orc_shape;

static void shape_of(const orc_net *n, orc_shape *s)
{
    s->c[0] = n->in_c; s->h[0] = n->in_h; s->w[0] = n->in_w;
    long off = 0;
    for (int l = 0; l < n->n_conv; ++l) {
        s->c[l + 1] = n->conv_out[l];
        s->h[l + 1] = (s->h[l] - n->conv_k[l]) / n->conv_stride[l] + 1;
        s->w[l + 1] = (s->w[l] - n->conv_k[l]) / n->conv_stride[l] + 1;
        s->w_off[l] = off; off += (long)n->conv_out[l] * s->c[l] * n->conv_k[l] * n->conv_k[l];
        s->b_off[l] = off; off += n->conv_out[l];
    }
    int L = n->n_conv;
    s->flat = (long)s->c[L] * s->h[L] * s->w[L];
    s->fcw_off = off; off += (long)n->fc * s->flat;
    s->fcb_off = off; off += n->fc;
    s->piw_off = off; off += (long)n->n_actions * n->fc;
    s->pib_off = off; off += n->n_actions;
    s->vw_off = off;  off += n->fc;
    s->vb_off = off;  off += 1;
    s->d = off;
    s->in_size = (long)s->c[0] * s->h[0] * s->w[0];
    long a = s->in_size;
    for (int l = 1; l <= L; ++l) { s->act_off[l] = a; a += (long)s->c[l] * s->h[l] * s->w[l]; }
    s->act_off[L + 1] = a; a += n->fc;
    s->act_size = a;
}

long orc_param_count(const orc_net *n) { orc_shape s; shape_of(n, &s); return s.d; }
long orc_act_size(const orc_net *n) { orc_shape s; shape_of(n, &s); return s.act_size; }

/* ---- network, one frame ------------------------------------------------- */

/* Forward pass of one frame.  rec receives: scaled input, every conv output
 * (after ReLU), hidden (after ReLU).  pre (may be NULL) receives, at the same
 * offsets, the values before each ReLU.  logits[A], *value. */
static void forward_frame(const orc_net *n, const orc_shape *s, const double *x,
                          const uint8_t *obs, double *rec, double *pre, double *logits, double *value)
{
    for (long i = 0; i < s->in_size; ++i) rec[i] = (double)obs[i] / 255.0;

    const double *in = rec;
    for (int l = 0; l < n->n_conv; ++l) {
        const int C = s->c[l], H = s->h[l], W = s->w[l];
        const int O = s->c[l + 1], OH = s->h[l + 1], OW = s->w[l + 1];
        const int K = n->conv_k[l], S = n->conv_stride[l];
        const double *w = x + s->w_off[l], *b = x + s->b_off[l];
        double *out = rec + s->act_off[l + 1];
        for (int o = 0; o < O; ++o)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = b[o];
                    for (int c = 0; c < C; ++c)
                        for (int ky = 0; ky < K; ++ky)
                            for (int kx = 0; kx < K; ++kx)
                                acc += w[(((long)o * C + c) * K + ky) * K + kx] *
                                       in[((long)c * H + (oy * S + ky)) * W + (ox * S + kx)];
                    out[((long)o * OH + oy) * OW + ox] = acc > 0.0 ? acc : 0.0;
                    if (pre) pre[s->act_off[l + 1] + ((long)o * OH + oy) * OW + ox] = acc;
                }
        in = out;
        (void)H;
    }

    const int L = n->n_conv;
    double *hid = rec + s->act_off[L + 1];
    const double *fw = x + s->fcw_off, *fb = x + s->fcb_off;
    for (int j = 0; j < n->fc; ++j) {
        double acc = fb[j];
        for (long k = 0; k < s->flat; ++k) acc += fw[(long)j * s->flat + k] * in[k];
        hid[j] = acc > 0.0 ? acc : 0.0;
        if (pre) pre[s->act_off[L + 1] + j] = acc;
    }
    const double *pw = x + s->piw_off, *pb = x + s->pib_off;
    for (int a = 0; a < n->n_actions; ++a) {
        double acc = pb[a];
        for (int j = 0; j < n->fc; ++j) acc += pw[(long)a * n->fc + j] * hid[j];
        logits[a] = acc;
    }
    double acc = x[s->vb_off];
    for (int j = 0; j < n->fc; ++j) acc += x[s->vw_off + j] * hid[j];
    *value = acc;
}

/* Whether a ReLU unit passes gradient.  The unit's own sign decides, unless the
 * caller marks it (gate 1 = pass, 2 = block).  Tests use the marks only for units
 * whose pre-activation lies within single-precision rounding of zero, where the
 * derivative of max(z, 0) is decided by rounding and both answers are valid. */
static int relu_open(double act, const uint8_t *gate, long i)
{
    if (gate && gate[i] == 1) return 1;
    if (gate && gate[i] == 2) return 0;
    return act > 0.0;
}

/* Reverse pass of one frame down to the pre-activation gradients of every
 * layer.  dz receives, at the same offsets as the activations in rec, the loss
 * gradient w.r.t. the value *before* each ReLU (conv outputs and hidden).
 * The input needs no gradient.  gate: NULL or act_size bytes, see relu_open. */
static void backward_frame(const orc_net *n, const orc_shape *s, const double *x,
                           const double *rec, const double *dlogits, double dvalue, double *dz,
                           const uint8_t *gate)
{
    const int L = n->n_conv;
    const double *hid = rec + s->act_off[L + 1];
    double *dzh = dz + s->act_off[L + 1];
    const double *pw = x + s->piw_off;
    for (int j = 0; j < n->fc; ++j) {
        double g = x[s->vw_off + j] * dvalue;
        for (int a = 0; a < n->n_actions; ++a) g += pw[(long)a * n->fc + j] * dlogits[a];
        dzh[j] = relu_open(hid[j], gate, s->act_off[L + 1] + j) ? g : 0.0;
    }
    /* hidden layer -> flattened last conv output */
    {
        const double *act = rec + s->act_off[L];
        double *dzl = dz + s->act_off[L];
        const double *fw = x + s->fcw_off;
        for (long k = 0; k < s->flat; ++k) {
            double g = 0.0;
            for (int j = 0; j < n->fc; ++j) g += fw[(long)j * s->flat + k] * dzh[j];
            dzl[k] = relu_open(act[k], gate, s->act_off[L] + k) ? g : 0.0;
        }
    }
    /* conv l (1-based l+1) output gradient -> conv l-1 output gradient */
    for (int l = L - 1; l >= 1; --l) {
        const int C = s->c[l], H = s->h[l], W = s->w[l];
        const int O = s->c[l + 1], OH = s->h[l + 1], OW = s->w[l + 1];
        const int K = n->conv_k[l], S = n->conv_stride[l];
        const double *w = x + s->w_off[l];
        const double *dout = dz + s->act_off[l + 1];
        const double *act = rec + s->act_off[l];
        double *din = dz + s->act_off[l];
        for (long i = 0; i < (long)C * H * W; ++i) din[i] = 0.0;
        for (int o = 0; o < O; ++o)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    const double g = dout[((long)o * OH + oy) * OW + ox];
                    if (g == 0.0) continue;
                    for (int c = 0; c < C; ++c)
                        for (int ky = 0; ky < K; ++ky)
                            for (int kx = 0; kx < K; ++kx)
                                din[((long)c * H + (oy * S + ky)) * W + (ox * S + kx)] +=
                                    w[(((long)o * C + c) * K + ky) * K + kx] * g;
                }
        for (long i = 0; i < (long)C * H * W; ++i) if (!relu_open(act[i], gate, s->act_off[l] + i)) din[i] = 0.0;
    }
}

/* Parameter gradients from the stored activations and pre-activation
 * gradients of F frames: every entry is the sum over frames (and positions) in
 * increasing frame order. */
static void param_gradients(const orc_net *n, const orc_shape *s, int F,
                            const double *recs, const double *dzs,
                            const double *dlogits, const double *dvalues, double *g)
{
    const int L = n->n_conv;
    for (int l = 0; l < L; ++l) {
        const int C = s->c[l], H = s->h[l], W = s->w[l];
        const int O = s->c[l + 1], OH = s->h[l + 1], OW = s->w[l + 1];
        const int K = n->conv_k[l], S = n->conv_stride[l];
        double *gw = g + s->w_off[l], *gb = g + s->b_off[l];
        const long in_off = (l == 0) ? 0 : s->act_off[l];
        #pragma omp parallel for schedule(static)
        for (int o = 0; o < O; ++o) {
            double sb = 0.0;
            for (int f = 0; f < F; ++f) {
                const double *dout = dzs + (long)f * s->act_size + s->act_off[l + 1];
                for (int p = 0; p < OH * OW; ++p) sb += dout[(long)o * OH * OW + p];
            }
            gb[o] = sb;
            for (int c = 0; c < C; ++c)
                for (int ky = 0; ky < K; ++ky)
                    for (int kx = 0; kx < K; ++kx) {
                        double acc = 0.0;
                        for (int f = 0; f < F; ++f) {
                            const double *dout = dzs + (long)f * s->act_size + s->act_off[l + 1];
                            const double *in = recs + (long)f * s->act_size + in_off;
                            for (int oy = 0; oy < OH; ++oy)
                                for (int ox = 0; ox < OW; ++ox)
                                    acc += dout[((long)o * OH + oy) * OW + ox] *
                                           in[((long)c * H + (oy * S + ky)) * W + (ox * S + kx)];
                        }
                        gw[(((long)o * C + c) * K + ky) * K + kx] = acc;
                    }
        }
    }
    #pragma omp parallel for schedule(static)
    for (int j = 0; j < n->fc; ++j) {
        double sb = 0.0;
        for (int f = 0; f < F; ++f) sb += dzs[(long)f * s->act_size + s->act_off[L + 1] + j];
        g[s->fcb_off + j] = sb;
        for (long k = 0; k < s->flat; ++k) {
            double acc = 0.0;
            for (int f = 0; f < F; ++f)
                acc += dzs[(long)f * s->act_size + s->act_off[L + 1] + j] *
                       recs[(long)f * s->act_size + s->act_off[L] + k];
            g[s->fcw_off + (long)j * s->flat + k] = acc;
        }
    }
    for (int a = 0; a < n->n_actions; ++a) {
        double sb = 0.0;
        for (int f = 0; f < F; ++f) sb += dlogits[(long)f * n->n_actions + a];
        g[s->pib_off + a] = sb;
        for (int j = 0; j < n->fc; ++j) {
            double acc = 0.0;
            for (int f = 0; f < F; ++f)
                acc += dlogits[(long)f * n->n_actions + a] *
                       recs[(long)f * s->act_size + s->act_off[L + 1] + j];
            g[s->piw_off + (long)a * n->fc + j] = acc;
        }
    }
    {
        double sb = 0.0;
        for (int f = 0; f < F; ++f) sb += dvalues[f];
        g[s->vb_off] = sb;
        for (int j = 0; j < n->fc; ++j) {
            double acc = 0.0;
            for (int f = 0; f < F; ++f)
                acc += dvalues[f] * recs[(long)f * s->act_size + s->act_off[L + 1] + j];
            g[s->vw_off + j] = acc;
        }
    }
}

/* ---- exported pieces ---------------------------------------------------- */

/* Forward pass of F frames (obs: F consecutive C*H*W byte frames).
 * acts may be NULL; otherwise it receives F records of orc_act_size doubles
 * (scaled input, conv outputs after ReLU, hidden after ReLU).  pre may be NULL;
 * otherwise it receives the values before each ReLU at the same offsets. */
void orc_forward(const orc_net *n, const double *x, const uint8_t *obs, int F,
                 double *logits, double *values, double *acts, double *pre)
{
    orc_shape s; shape_of(n, &s);
    double *own = NULL;
    if (!acts) { own = (double *)malloc(sizeof(double) * s.act_size * (size_t)F); acts = own; }
    #pragma omp parallel for schedule(dynamic, 1)
    for (int f = 0; f < F; ++f)
        forward_frame(n, &s, x, obs + (long)f * s.in_size, acts + (long)f * s.act_size,
                      pre ? pre + (long)f * s.act_size : NULL, logits + (long)f * n->n_actions, values + f);
    free(own);
}

/* n-step returns over a T-step rollout of B environments (Sec. 2:
 * G_t = sum_{i<n} gamma^i r_{t+i} + gamma^n V(s_{t+n}), n = T - t), written as
 * the backward recursion G_t = r_t + gamma (1 - done_t) G_{t+1}, G_T = V(s_T),
 * and advantages A_t = G_t - V(s_t).  Arrays are [T][B]; v_boot is [B]. */
void orc_nstep_returns(int T, int B, double gamma, const double *rewards, const uint8_t *dones,
                       const double *v_boot, const double *values, double *G, double *Adv)
{
    for (int b = 0; b < B; ++b) {
        double next = v_boot[b];
        for (int t = T - 1; t >= 0; --t) {
            const double keep = dones[t * B + b] ? 0.0 : 1.0;
            next = rewards[t * B + b] + gamma * keep * next;
            G[t * B + b] = next;
            Adv[t * B + b] = next - values[t * B + b];
        }
    }
}

/* A2C loss over M samples with A actions and its gradient w.r.t. the network
 * outputs.  terms[0] = mean(-log pi(a) Adv), terms[1] = mean((G - V)^2),
 * terms[2] = mean(entropy); loss = terms[0] + vf_coef terms[1] - ent_coef terms[2].
 * G and Adv are treated as constants. */
void orc_a2c_loss(int M, int A, const double *logits, const double *values, const int32_t *actions,
                  const double *G, const double *Adv, double vf_coef, double ent_coef,
                  double *terms, double *dlogits, double *dvalues)
{
    double pg = 0.0, td = 0.0, ent = 0.0;
    double *logp = (double *)malloc(sizeof(double) * (size_t)A);
    for (int m = 0; m < M; ++m) {
        const double *z = logits + (long)m * A;
        double zmax = z[0];
        for (int a = 1; a < A; ++a) if (z[a] > zmax) zmax = z[a];
        double se = 0.0;
        for (int a = 0; a < A; ++a) se += exp(z[a] - zmax);
        const double lse = zmax + log(se);
        double H = 0.0;
        for (int a = 0; a < A; ++a) { logp[a] = z[a] - lse; H -= exp(logp[a]) * logp[a]; }
        pg += -logp[actions[m]] * Adv[m];
        td += (G[m] - values[m]) * (G[m] - values[m]);
        ent += H;
        if (dlogits)
            for (int a = 0; a < A; ++a) {
                const double p = exp(logp[a]);
                const double dpg = Adv[m] * (p - (a == actions[m] ? 1.0 : 0.0));
                const double dent = p * (logp[a] + H);      /* d(-H)/dz_a */
                dlogits[(long)m * A + a] = (dpg + ent_coef * dent) / M;
            }
        if (dvalues) dvalues[m] = -2.0 * vf_coef * (G[m] - values[m]) / M;
    }
    free(logp);
    terms[0] = pg / M; terms[1] = td / M; terms[2] = ent / M;
}

/* Gradient of one agent's A2C loss w.r.t. all of its parameters.
 * obs [T][B][C][H][W] bytes, boot_obs [B][C][H][W], actions/rewards/dones [T][B].
 * grads[d]; terms[3] as in orc_a2c_loss.  Optional outputs (may be NULL):
 * out_G, out_Adv [T*B]; out_logits [T*B][A]; out_values [T*B + B] (rollout then bootstrap).
 * gate: NULL, or [T*B][orc_act_size] bytes of ReLU-derivative marks (see relu_open). */
void orc_agent_gradient(const orc_net *n, const orc_hparams *hp, const double *x,
                        const uint8_t *obs, const int32_t *actions, const double *rewards,
                        const uint8_t *dones, const uint8_t *boot_obs,
                        double *grads, double *terms,
                        double *out_G, double *out_Adv, double *out_logits, double *out_values,
                        const uint8_t *gate)
{
    orc_shape s; shape_of(n, &s);
    const int M = hp->T * hp->B, Bn = hp->B, A = n->n_actions;
    double *recs = (double *)malloc(sizeof(double) * s.act_size * (size_t)(M + Bn));
    double *dzs = (double *)malloc(sizeof(double) * s.act_size * (size_t)M);
    double *logits = (double *)malloc(sizeof(double) * (size_t)(M + Bn) * A);
    double *values = (double *)malloc(sizeof(double) * (size_t)(M + Bn));
    double *G = (double *)malloc(sizeof(double) * M), *Adv = (double *)malloc(sizeof(double) * M);
    double *dlogits = (double *)malloc(sizeof(double) * (size_t)M * A);
    double *dvalues = (double *)malloc(sizeof(double) * M);

    /* values of the rollout states and of the state after the last action, all
     * under the current parameters */
    #pragma omp parallel for schedule(dynamic, 1)
    for (int f = 0; f < M + Bn; ++f) {
        const uint8_t *frame = f < M ? obs + (long)f * s.in_size : boot_obs + (long)(f - M) * s.in_size;
        forward_frame(n, &s, x, frame, recs + (long)f * s.act_size, NULL, logits + (long)f * A, values + f);
    }
    orc_nstep_returns(hp->T, hp->B, hp->gamma, rewards, dones, values + M, values, G, Adv);
    orc_a2c_loss(M, A, logits, values, actions, G, Adv, hp->vf_coef, hp->ent_coef, terms, dlogits, dvalues);

    #pragma omp parallel for schedule(dynamic, 1)
    for (int f = 0; f < M; ++f)
        backward_frame(n, &s, x, recs + (long)f * s.act_size, dlogits + (long)f * A, dvalues[f],
                       dzs + (long)f * s.act_size, gate ? gate + (long)f * s.act_size : NULL);
    param_gradients(n, &s, M, recs, dzs, dlogits, dvalues, grads);

    if (out_G) memcpy(out_G, G, sizeof(double) * M);
    if (out_Adv) memcpy(out_Adv, Adv, sizeof(double) * M);
    if (out_logits) memcpy(out_logits, logits, sizeof(double) * (size_t)M * A);
    if (out_values) memcpy(out_values, values, sizeof(double) * (size_t)(M + Bn));
    free(recs); free(dzs); free(logits); free(values); free(G); free(Adv); free(dlogits); free(dvalues);
}

/* Loss value only (used by finite-difference checks): the three terms for
 * given parameters, with returns/advantages either recomputed from these
 * parameters (fixed_G == NULL) or held at the supplied constants. */
void orc_agent_loss(const orc_net *n, const orc_hparams *hp, const double *x,
                    const uint8_t *obs, const int32_t *actions, const double *rewards,
                    const uint8_t *dones, const uint8_t *boot_obs,
                    const double *fixed_G, const double *fixed_Adv, double *terms)
{
    orc_shape s; shape_of(n, &s);
    const int M = hp->T * hp->B, Bn = hp->B, A = n->n_actions;
    double *rec = (double *)malloc(sizeof(double) * s.act_size);
    double *logits = (double *)malloc(sizeof(double) * (size_t)(M + Bn) * A);
    double *values = (double *)malloc(sizeof(double) * (size_t)(M + Bn));
    double *G = (double *)malloc(sizeof(double) * M), *Adv = (double *)malloc(sizeof(double) * M);
    for (int f = 0; f < M + Bn; ++f) {
        const uint8_t *frame = f < M ? obs + (long)f * s.in_size : boot_obs + (long)(f - M) * s.in_size;
        forward_frame(n, &s, x, frame, rec, NULL, logits + (long)f * A, values + f);
    }
    if (fixed_G) { memcpy(G, fixed_G, sizeof(double) * M); memcpy(Adv, fixed_Adv, sizeof(double) * M); }
    else orc_nstep_returns(hp->T, hp->B, hp->gamma, rewards, dones, values + M, values, G, Adv);
    orc_a2c_loss(M, A, logits, values, actions, G, Adv, hp->vf_coef, hp->ent_coef, terms, NULL, NULL);
    free(rec); free(logits); free(values); free(G); free(Adv);
}

/* Global-norm clipping of one agent's gradient (Table 2: "clip global gradient
 * norm 0.5").  Returns the pre-clip 2-norm; *scale receives the factor applied. */
double orc_clip_grad_norm(double *g, long d, double max_norm, double *scale)
{
    double ss = 0.0;
    for (long i = 0; i < d; ++i) ss += g[i] * g[i];
    const double norm = sqrt(ss);
    double c = max_norm / (norm + 1e-6);
    if (c > 1.0) c = 1.0;
    if (c < 1.0) for (long i = 0; i < d; ++i) g[i] *= c;
    if (scale) *scale = c;
    return norm;
}

/* RMSprop without momentum (Table 2): v <- a v + (1 - a) g^2; x <- x - lr g / (sqrt(v) + eps). */
void orc_rmsprop(double *x, double *v, const double *g, long d, double lr, double alpha, double eps)
{
    for (long i = 0; i < d; ++i) {
        v[i] = alpha * v[i] + (1.0 - alpha) * g[i] * g[i];
        x[i] -= lr * g[i] / (sqrt(v[i]) + eps);
    }
}

/* One learner step of N independent agents (Algorithm 1: returns, then the A2C
 * optimisation step).  X, V: [N][d] parameters and RMSprop state, updated in
 * place.  grads_out [N][d] (pre-clip, may be NULL); stats [N][5] =
 * pg, td, entropy, pre-clip norm, clip scale.  gates: NULL, or
 * [N][T*B][orc_act_size] ReLU-derivative marks (see relu_open). */
void orc_learner_step(const orc_net *n, const orc_hparams *hp, int N, double *X, double *V,
                      const uint8_t *obs, const int32_t *actions, const float *rewards,
                      const uint8_t *dones, const uint8_t *boot_obs,
                      double *grads_out, double *stats, const uint8_t *gates)
{
    orc_shape s; shape_of(n, &s);
    const int M = hp->T * hp->B;
    double *g = (double *)malloc(sizeof(double) * s.d);
    double *r = (double *)malloc(sizeof(double) * M);
    for (int i = 0; i < N; ++i) {
        for (int m = 0; m < M; ++m) r[m] = (double)rewards[(long)i * M + m];
        double terms[3], scale;
        orc_agent_gradient(n, hp, X + (long)i * s.d, obs + (long)i * M * s.in_size,
                           actions + (long)i * M, r, dones + (long)i * M,
                           boot_obs + (long)i * hp->B * s.in_size, g, terms, NULL, NULL, NULL, NULL,
                           gates ? gates + (long)i * M * s.act_size : NULL);
        if (grads_out) memcpy(grads_out + (long)i * s.d, g, sizeof(double) * s.d);
        const double norm = orc_clip_grad_norm(g, s.d, hp->max_grad_norm, &scale);
        orc_rmsprop(X + (long)i * s.d, V + (long)i * s.d, g, s.d, hp->lr, hp->rms_alpha, hp->rms_eps);
        if (stats) {
            stats[i * 5 + 0] = terms[0]; stats[i * 5 + 1] = terms[1]; stats[i * 5 + 2] = terms[2];
            stats[i * 5 + 3] = norm; stats[i * 5 + 4] = scale;
        }
    }
    free(g); free(r);
}

/* Synchronous A2C with gradient averaging across agents (Sec. 5 "Experimental
 * setup": individual A2C agents average their gradients with AllReduce before
 * each update; Eq. (5) is the batched update this equals for identical
 * replicas).  Every agent computes its own gradient at its own parameters,
 * gbar = (1/N) sum_i g_i is clipped once, and every agent applies RMSprop with
 * gbar to its own X and V rows.  grads_out [N][d]: the agents' own pre-average
 * gradients; gbar_out [d] pre-clip average (either may be NULL); stats [N][5] as
 * in orc_learner_step with the norm and clip scale of gbar in every row. */
void orc_a2c_allreduce_step(const orc_net *n, const orc_hparams *hp, int N, double *X, double *V,
                            const uint8_t *obs, const int32_t *actions, const float *rewards,
                            const uint8_t *dones, const uint8_t *boot_obs,
                            double *grads_out, double *gbar_out, double *stats, const uint8_t *gates)
{
    orc_shape s; shape_of(n, &s);
    const int M = hp->T * hp->B;
    double *g = (double *)malloc(sizeof(double) * s.d);
    double *gbar = (double *)calloc(s.d, sizeof(double));
    double *r = (double *)malloc(sizeof(double) * M);
    for (int i = 0; i < N; ++i) {
        for (int m = 0; m < M; ++m) r[m] = (double)rewards[(long)i * M + m];
        double terms[3];
        orc_agent_gradient(n, hp, X + (long)i * s.d, obs + (long)i * M * s.in_size,
                           actions + (long)i * M, r, dones + (long)i * M,
                           boot_obs + (long)i * hp->B * s.in_size, g, terms, NULL, NULL, NULL, NULL,
                           gates ? gates + (long)i * M * s.act_size : NULL);
        if (grads_out) memcpy(grads_out + (long)i * s.d, g, sizeof(double) * s.d);
        for (long k = 0; k < s.d; ++k) gbar[k] += g[k];
        if (stats) { stats[i * 5 + 0] = terms[0]; stats[i * 5 + 1] = terms[1]; stats[i * 5 + 2] = terms[2]; }
    }
    for (long k = 0; k < s.d; ++k) gbar[k] /= (double)N;
    if (gbar_out) memcpy(gbar_out, gbar, sizeof(double) * s.d);
    double scale;
    const double norm = orc_clip_grad_norm(gbar, s.d, hp->max_grad_norm, &scale);
    for (int i = 0; i < N; ++i) {
        orc_rmsprop(X + (long)i * s.d, V + (long)i * s.d, gbar, s.d, hp->lr, hp->rms_alpha, hp->rms_eps);
        if (stats) { stats[i * 5 + 3] = norm; stats[i * 5 + 4] = scale; }
    }
    free(g); free(gbar); free(r);
}

/* ---- gossip -------------------------------------------------------------- */

/* The single in-peer of agent i at a given round (integer table).
 * kind 0: directed ring v_1 -> v_2 -> ... -> v_n -> v_1 (Fig. 5): agent i
 *         receives from i-1.
 * kind 1: one-peer exponential graph: agent i mixes with (i + 2^k) mod N,
 *         k = round mod log2(N).
 * kind 2: the same graph with every edge reversed: agent i mixes with
 *         (i - 2^k) mod N (the transposed, equally doubly stochastic matrix). */
int orc_in_peer(int kind, int N, long round, int i)
{
    if (kind == 0) return (i + N - 1) % N;
    int m = 0;
    while ((1 << (m + 1)) <= N) ++m;      /* log2 N for a power of two */
    if (m == 0) return i;
    const int k = (int)(round % m);
    const int hop = (1 << k) % N;
    return kind == 1 ? (i + hop) % N : (i + N - hop) % N;
}

int orc_n_phases(int kind, int N)
{
    if (kind == 0) return 1;
    int m = 0;
    while ((1 << (m + 1)) <= N) ++m;
    return m > 0 ? m : 1;
}

static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Fixed delay (in rounds) of the edge into agent i during phase k: one
 * splitmix64 draw keyed by seed + k*N + i, reduced modulo max_delay + 1. */
int orc_edge_delay(uint64_t seed, int N, int phase, int i, int max_delay)
{
    if (max_delay <= 0) return 0;
    return (int)(mix64(seed + (uint64_t)phase * (uint64_t)N + (uint64_t)i) % (uint64_t)(max_delay + 1));
}

/* ---- acting (Algorithm 1: "take actions according to pi") ------------------- */

/* Uniform variate in [0, 1) with 24 random bits: the top 24 bits of the
 * splitmix64 output for the state seed + counter (counter-based, so any draw can
 * be made on its own).  2^-24 spacing makes it exact in single precision too. */
double orc_uniform24(uint64_t seed, uint64_t counter)
{
    return (double)(mix64(seed + counter) >> 40) * (1.0 / 16777216.0);
}

/* One draw from the categorical distribution pi = softmax(logits) by inverting
 * its distribution function: the smallest a with pi_0 + ... + pi_a > u (the last
 * action if rounding leaves the total below u).  logp_out: log pi(a); cdf_out [A]:
 * the running sums (either may be NULL). */
int orc_categorical_sample(int A, const double *logits, double u, double *logp_out, double *cdf_out)
{
    double zmax = logits[0];
    for (int k = 1; k < A; ++k) if (logits[k] > zmax) zmax = logits[k];
    double se = 0.0;
    for (int k = 0; k < A; ++k) se += exp(logits[k] - zmax);
    const double lse = zmax + log(se);
    double run = 0.0;
    int a = -1;
    for (int k = 0; k < A; ++k) {
        run += exp(logits[k] - lse);
        if (cdf_out) cdf_out[k] = run;
        if (a < 0 && run > u) a = k;
    }
    if (a < 0) a = A - 1;
    if (logp_out) *logp_out = logits[a] - lse;
    return a;
}

/* The mixing step of Algorithm 1 for one agent with uniform weights:
 * out = (x + sum_j msgs[j]) / (1 + n_msgs). */
void orc_mix_uniform(const double *x, const double *const *msgs, int n_msgs, long d, double *out)
{
    for (long e = 0; e < d; ++e) {
        double acc = x[e];
        for (int j = 0; j < n_msgs; ++j) acc += msgs[j][e];
        out[e] = acc / (double)(1 + n_msgs);
    }
}

/* General row of a mixing matrix: out = w_self x + sum_j w[j] msgs[j]  (x_i = sum_j p_ij x_j). */
void orc_mix_weighted(const double *x, double w_self, const double *const *msgs, const double *w,
                      int n_msgs, long d, double *out)
{
    for (long e = 0; e < d; ++e) {
        double acc = w_self * x[e];
        for (int j = 0; j < n_msgs; ++j) acc += w[j] * msgs[j][e];
        out[e] = acc;
    }
}

/* Distance from consensus (Prop. 1): mean row xbar = (1/N) sum_i x_i;
 * *max_row = max_i ||x_i - xbar||_2, *frob = ||X - 1 xbar^T||_F. */
void orc_consensus_distance(const double *X, int N, long d, double *max_row, double *frob)
{
    double *mean = (double *)calloc((size_t)d, sizeof(double));
    for (int i = 0; i < N; ++i) for (long e = 0; e < d; ++e) mean[e] += X[(long)i * d + e];
    for (long e = 0; e < d; ++e) mean[e] /= (double)N;
    double mx = 0.0, tot = 0.0;
    for (int i = 0; i < N; ++i) {
        double ss = 0.0;
        for (long e = 0; e < d; ++e) { const double t = X[(long)i * d + e] - mean[e]; ss += t * t; }
        tot += ss;
        if (sqrt(ss) > mx) mx = sqrt(ss);
    }
    free(mean);
    *max_row = mx; *frob = sqrt(tot);
}

/* ---- diagnostics of Sec. 5 "Effects of gossip" ---------------------------------- */

/* Pair-wise cosine similarity of the agents' gradients (Fig. 2b):
 * out[i][j] = <g_i, g_j> / (||g_i|| ||g_j||); a zero gradient gives 0. */
void orc_cosine_matrix(const double *G, int N, long d, double *out)
{
    double *nrm = (double *)malloc(sizeof(double) * (size_t)N);
    for (int i = 0; i < N; ++i) {
        double ss = 0.0;
        for (long e = 0; e < d; ++e) ss += G[(long)i * d + e] * G[(long)i * d + e];
        nrm[i] = sqrt(ss);
    }
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j) {
            double dot = 0.0;
            for (long e = 0; e < d; ++e) dot += G[(long)i * d + e] * G[(long)j * d + e];
            out[(long)i * N + j] = (nrm[i] > 0.0 && nrm[j] > 0.0) ? dot / (nrm[i] * nrm[j]) : 0.0;
        }
    free(nrm);
}

/* Size of one round's local updates in the notation of Prop. 1: the update matrix
 * alpha G^(k) has rows x_i(before the optimiser step) - x_i(after it, before
 * mixing).  row_norms[i] = ||alpha g_i||_2 (may be NULL); returns ||alpha G||_F. */
double orc_update_norm(const double *X_before, const double *X_after, int N, long d, double *row_norms)
{
    double tot = 0.0;
    for (int i = 0; i < N; ++i) {
        double ss = 0.0;
        for (long e = 0; e < d; ++e) {
            const double t = X_before[(long)i * d + e] - X_after[(long)i * d + e];
            ss += t * t;
        }
        if (row_norms) row_norms[i] = sqrt(ss);
        tot += ss;
    }
    return sqrt(tot);
}

/* Right-hand side of Prop. 1 after k + 1 rounds for agents that started from
 * identical parameters: sum_{s=0..k} beta^(k+1-s) ||alpha G^(s)||, with
 * update_norms[s] = ||alpha G^(s)|| (n = k + 1 entries). */
double orc_prop1_bound(double beta, const double *update_norms, int n)
{
    double acc = 0.0;
    for (int s = 0; s < n; ++s) acc += pow(beta, (double)(n - s)) * update_norms[s];
    return acc;
}
