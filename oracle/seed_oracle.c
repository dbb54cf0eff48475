/*
 * seed_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, direct-loop CPU statement of what SEED RL's central
 * inference step computes for one gathered batch of actor observations
 * (Section 3, "Detailed Learner architecture": the inference thread takes a
 * batch of observations, rewards and recurrent states, runs the agent
 * network, and gets back sampled actions and new recurrent states).
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may load this
 * file's library.  It shares no code, header, table or helper with the HIP
 * library; the HIP library never calls it.
 *
 * Arithmetic: activations and outputs are stored as `real` (float unless the
 * file is compiled with -DORACLE_F64, then double); every dot product is
 * accumulated in double and rounded once to `real`.  Nothing is blocked,
 * fused or reordered: each function is the textbook definition of its layer.
 *
 * Network families (Appendix A.3.1 for the R2D2 net; Section 4.1 names the
 * "ResNet from IMPALA"; Section 4.2 names the Football model; the exact layer
 * lists of the latter two are fixed by the benchmark configurations, the
 * paper gives only their names):
 *   torso 0: conv(k,stride,VALID)+ReLU repeated, flatten, dense, ReLU
 *   torso 1: sections of [conv3x3 SAME, maxpool 3x3/2 SAME, 2 residual blocks
 *            x + conv(ReLU(conv(ReLU(x))))], ReLU, flatten, dense, ReLU
 *   core   : optional LSTM fed [features, one-hot previous action, previous
 *            reward] (Appendix A.3.1)
 *   heads  : policy logits + value, or dueling value/advantage streams
 *            (Section 3.2 cites the dueling architecture)
 *   select : greedy argmax, or Gumbel-max sampling from caller uniforms
 *
 * Parity pins: every exported function below is pinned by tests/test_oracle_*.py
 * against brute force, closed forms, hand-worked cells or torch CPU fp64
 * library routines.  The end-to-end value of oracle_forward on a whole
 * network is pinned only through the composition of those unit pins plus a
 * torch-CPU fp64 re-composition ("parity unpinned" by the paper itself: it
 * prints no forward-pass numbers).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifdef ORACLE_F64
typedef double real;
#define R_EXP exp
#define R_LOG log
#define R_TANH tanh
#else
typedef float real;
#define R_EXP expf
#define R_LOG logf
#define R_TANH tanhf
#endif

typedef struct {
    int32_t obs_h, obs_w, obs_c;
    int32_t torso;              /* 0 = VALID conv stack, 1 = deep ResNet */
    int32_t n_conv;
    int32_t conv_ch[4], conv_k[4], conv_stride[4];
    int32_t n_sections;
    int32_t section_ch[4];
    int32_t fc_units;
    int32_t lstm_units;         /* 0 = no recurrent core */
    int32_t num_actions;
    int32_t head;               /* 0 = policy + value, 1 = dueling Q */
    int32_t head_hidden;
    int32_t select;             /* 0 = greedy, 1 = Gumbel-max */
} oracle_arch;

int oracle_sizeof_real(void) { return (int)sizeof(real); }

/* threads oracle_forward spreads batch rows over (1 without OpenMP) */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- layers */

/* Observation bytes to the unit interval: x = obs / 255.  The paper never
 * states the input scaling; this is the reading fixed for the build. */
void oracle_normalise(const uint8_t *obs, int64_t n, real *x)
{
    for (int64_t i = 0; i < n; ++i) x[i] = (real)obs[i] / (real)255;
}

/* Output extent of a convolution or pooling window along one axis.
 * VALID: floor((n-k)/s)+1.  SAME: ceil(n/s). */
int oracle_out_size(int n, int k, int stride, int same)
{
    if (same) return (n + stride - 1) / stride;
    if (n < k) return 0;
    return (n - k) / stride + 1;
}

/* Leading padding of a SAME window (the trailing side takes the odd cell):
 * total = max((out-1)*s + k - n, 0), before = floor(total/2). */
static int same_pad_before(int n, int k, int stride)
{
    int out = (n + stride - 1) / stride;
    int total = (out - 1) * stride + k - n;
    if (total < 0) total = 0;
    return total / 2;
}

/* 2-D cross-correlation (no kernel flip), NHWC activations, HWIO weights:
 *   y[oh,ow,co] = b[co] + sum_{kh,kw,ci} x[oh*s+kh-pt, ow*s+kw-pl, ci] * W[kh,kw,ci,co]
 * with taps outside the image contributing zero.  Appendix A.3.1 gives the
 * R2D2 stack's kernel sizes, strides and "valid" padding; the 3x3 ResNet
 * convolutions are SAME because the residual sum needs equal shapes. */
void oracle_conv2d(const real *x, int H, int W, int Cin,
                   const real *wt, const real *bias,
                   int k, int stride, int same, int Cout, real *y)
{
    int OH = oracle_out_size(H, k, stride, same);
    int OW = oracle_out_size(W, k, stride, same);
    int pt = same ? same_pad_before(H, k, stride) : 0;
    int pl = same ? same_pad_before(W, k, stride) : 0;
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int co = 0; co < Cout; ++co) {
                double acc = bias ? (double)bias[co] : 0.0;
                for (int kh = 0; kh < k; ++kh) {
                    int ih = oh * stride + kh - pt;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < k; ++kw) {
                        int iw = ow * stride + kw - pl;
                        if (iw < 0 || iw >= W) continue;
                        const real *xp = x + ((int64_t)ih * W + iw) * Cin;
                        const real *wp = wt + (((int64_t)kh * k + kw) * Cin) * Cout + co;
                        for (int ci = 0; ci < Cin; ++ci)
                            acc += (double)xp[ci] * (double)wp[(int64_t)ci * Cout];
                    }
                }
                y[((int64_t)oh * OW + ow) * Cout + co] = (real)acc;
            }
}

/* 3x3 max-pool, stride 2, SAME: the maximum over the in-range cells of each
 * window; cells outside the image never take part. */
void oracle_maxpool_3x3_s2(const real *x, int H, int W, int C, real *y)
{
    int OH = oracle_out_size(H, 3, 2, 1), OW = oracle_out_size(W, 3, 2, 1);
    int pt = same_pad_before(H, 3, 2), pl = same_pad_before(W, 3, 2);
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int c = 0; c < C; ++c) {
                int have = 0;
                real m = 0;
                for (int i = 0; i < 3; ++i) {
                    int ih = oh * 2 + i - pt;
                    if (ih < 0 || ih >= H) continue;
                    for (int j = 0; j < 3; ++j) {
                        int iw = ow * 2 + j - pl;
                        if (iw < 0 || iw >= W) continue;
                        real v = x[((int64_t)ih * W + iw) * C + c];
                        if (!have || v > m) { m = v; have = 1; }
                    }
                }
                y[((int64_t)oh * OW + ow) * C + c] = m;
            }
}

void oracle_relu(const real *x, int64_t n, real *y)
{
    for (int64_t i = 0; i < n; ++i) y[i] = x[i] > 0 ? x[i] : 0;
}

/* Dense layer y[o] = b[o] + sum_i x[i] * W[i,o], W row-major [n_in][n_out]. */
void oracle_dense(const real *x, int n_in, const real *wt, const real *bias,
                  int n_out, real *y)
{
    for (int o = 0; o < n_out; ++o) {
        double acc = bias ? (double)bias[o] : 0.0;
        for (int i = 0; i < n_in; ++i)
            acc += (double)x[i] * (double)wt[(int64_t)i * n_out + o];
        y[o] = (real)acc;
    }
}

/* One residual block of the deep ResNet torso on a C-channel map:
 *   y = x + conv_b(ReLU(conv_a(ReLU(x)))),  both 3x3 SAME, C -> C.
 * w points at [Wa (9*C*C), ba (C), Wb (9*C*C), bb (C)]. */
void oracle_residual_block(const real *x, int H, int W, int C, const real *w, real *y)
{
    int64_t n = (int64_t)H * W * C;
    int64_t wsz = (int64_t)9 * C * C;
    real *t0 = (real *)malloc(sizeof(real) * n);
    real *t1 = (real *)malloc(sizeof(real) * n);
    oracle_relu(x, n, t0);
    oracle_conv2d(t0, H, W, C, w, w + wsz, 3, 1, 1, C, t1);
    oracle_relu(t1, n, t0);
    oracle_conv2d(t0, H, W, C, w + wsz + C, w + 2 * wsz + C, 3, 1, 1, C, t1);
    for (int64_t i = 0; i < n; ++i) y[i] = x[i] + t1[i];
    free(t0);
    free(t1);
}

static double sigmoid_d(double v) { return 1.0 / (1.0 + exp(-v)); }

/* One LSTM step (Appendix A.3.1: the core also takes the one-hot previous
 * action and the previous reward).  z = [feat(F), onehot_A(prev_action),
 * prev_reward]; W has rows [z rows | h rows] and column blocks [i|f|g|o]:
 *   gates = z W_z + h_in W_h + b
 *   c' = sigma(f) c + sigma(i) tanh(g),   h' = sigma(o) tanh(c')
 * A previous action outside [0,A) gives an all-zero one-hot. */
void oracle_lstm_cell(const real *feat, int F, int prev_action, int A, real prev_reward,
                      const real *h_in, const real *c_in, int H,
                      const real *wt, const real *bias, real *h_out, real *c_out)
{
    int Z = F + A + 1;
    int G = 4 * H;
    real *z = (real *)calloc((size_t)Z, sizeof(real));
    real *gates = (real *)malloc(sizeof(real) * (size_t)G);
    memcpy(z, feat, sizeof(real) * (size_t)F);
    if (prev_action >= 0 && prev_action < A) z[F + prev_action] = 1;
    z[F + A] = prev_reward;
    for (int g = 0; g < G; ++g) {
        double acc = (double)bias[g];
        for (int i = 0; i < Z; ++i)
            acc += (double)z[i] * (double)wt[(int64_t)i * G + g];
        for (int i = 0; i < H; ++i)
            acc += (double)h_in[i] * (double)wt[(int64_t)(Z + i) * G + g];
        gates[g] = (real)acc;
    }
    for (int j = 0; j < H; ++j) {
        double gi = gates[j], gf = gates[H + j], gg = gates[2 * H + j], go = gates[3 * H + j];
        double cn = sigmoid_d(gf) * (double)c_in[j] + sigmoid_d(gi) * tanh(gg);
        real cr = (real)cn;
        c_out[j] = cr;
        h_out[j] = (real)(sigmoid_d(go) * tanh((double)cr));
    }
    free(z);
    free(gates);
}

/* Policy logits and scalar value from the core output. w = [Wp (n*A), bp (A),
 * Wv (n), bv (1)]. */
void oracle_head_policy_value(const real *core, int n, int A, const real *w,
                              real *logits, real *value)
{
    const real *wp = w, *bp = wp + (int64_t)n * A, *wv = bp + A, *bv = wv + n;
    oracle_dense(core, n, wp, bp, A, logits);
    oracle_dense(core, n, wv, bv, 1, value);
}

/* Dueling streams (Section 3.2 / Appendix A.3.1: "dueling heads with 512
 * hidden units"): V = ReLU(core W1v + b1v) W2v + b2v, Adv likewise, and
 * Q = V + Adv - mean_a Adv.  w = [W1v, b1v, W2v, b2v, W1a, b1a, W2a, b2a]. */
void oracle_head_dueling(const real *core, int n, int hid, int A, const real *w,
                         real *q, real *value)
{
    const real *w1v = w, *b1v = w1v + (int64_t)n * hid, *w2v = b1v + hid, *b2v = w2v + hid;
    const real *w1a = b2v + 1, *b1a = w1a + (int64_t)n * hid, *w2a = b1a + hid;
    const real *b2a = w2a + (int64_t)hid * A;
    real *hv = (real *)malloc(sizeof(real) * (size_t)hid);
    real *ha = (real *)malloc(sizeof(real) * (size_t)hid);
    real *adv = (real *)malloc(sizeof(real) * (size_t)A);
    oracle_dense(core, n, w1v, b1v, hid, hv);
    oracle_relu(hv, hid, hv);
    oracle_dense(hv, hid, w2v, b2v, 1, value);
    oracle_dense(core, n, w1a, b1a, hid, ha);
    oracle_relu(ha, hid, ha);
    oracle_dense(ha, hid, w2a, b2a, A, adv);
    double mean = 0.0;
    for (int a = 0; a < A; ++a) mean += (double)adv[a];
    mean /= (double)A;
    for (int a = 0; a < A; ++a) q[a] = (real)((double)value[0] + (double)adv[a] - mean);
    free(hv);
    free(ha);
    free(adv);
}

/* softmax with the row maximum subtracted first */
void oracle_softmax(const real *logits, int A, real *probs)
{
    real m = logits[0];
    for (int a = 1; a < A; ++a) if (logits[a] > m) m = logits[a];
    double s = 0.0;
    for (int a = 0; a < A; ++a) s += exp((double)logits[a] - (double)m);
    for (int a = 0; a < A; ++a) probs[a] = (real)(exp((double)logits[a] - (double)m) / s);
}

/* argmax with ties to the lowest index; *margin = top1 - top2 (0 if A==1) */
static int argmax_margin(const real *v, int A, real *margin)
{
    int best = 0;
    for (int a = 1; a < A; ++a) if (v[a] > v[best]) best = a;
    if (margin) {
        int have = 0;
        real second = 0;
        for (int a = 0; a < A; ++a) {
            if (a == best) continue;
            if (!have || v[a] > second) { second = v[a]; have = 1; }
        }
        *margin = have ? v[best] - second : 0;
    }
    return best;
}

int oracle_select_greedy(const real *logits, int A, real *margin)
{
    return argmax_margin(logits, A, margin);
}

/* Gumbel-max sampling: a = argmax_j (logit_j + G_j), G_j = -log(-log u_j),
 * u clamped into [FLT_MIN, 1 - 2^-24] so both logarithms are finite.  The
 * action is then distributed as softmax(logits).  perturbed (may be NULL)
 * receives logit_j + G_j. */
int oracle_select_gumbel(const real *logits, const real *u, int A, real *perturbed, real *margin)
{
    real *p = (real *)malloc(sizeof(real) * (size_t)A);
    const real lo = (real)FLT_MIN, hi = (real)(1.0 - 1.0 / 16777216.0);
    for (int a = 0; a < A; ++a) {
        real uu = u[a];
        if (uu < lo) uu = lo;
        if (uu > hi) uu = hi;
        p[a] = logits[a] - R_LOG(-R_LOG(uu));
    }
    int best = argmax_margin(p, A, margin);
    if (perturbed) memcpy(perturbed, p, sizeof(real) * (size_t)A);
    free(p);
    return best;
}

/* ------------------------------------------------------- weight offsets */

/* Canonical flat weight order (row-major fp values): per conv W[kh][kw][cin][cout]
 * then b[cout], layers in forward order (ResNet section: conv0, block1.a,
 * block1.b, block2.a, block2.b); dense W[in][out], b; LSTM W[(F+A+1)+H][4H], b[4H];
 * heads as documented on the two head functions above. */
static int torso_out_dims(const oracle_arch *a, int *h, int *w, int *c)
{
    int H = a->obs_h, W = a->obs_w, C = a->obs_c;
    if (a->torso == 0) {
        for (int l = 0; l < a->n_conv; ++l) {
            H = oracle_out_size(H, a->conv_k[l], a->conv_stride[l], 0);
            W = oracle_out_size(W, a->conv_k[l], a->conv_stride[l], 0);
            C = a->conv_ch[l];
            if (H <= 0 || W <= 0) return -1;
        }
    } else {
        for (int s = 0; s < a->n_sections; ++s) {
            H = oracle_out_size(H, 3, 2, 1);
            W = oracle_out_size(W, 3, 2, 1);
            C = a->section_ch[s];
        }
    }
    *h = H; *w = W; *c = C;
    return 0;
}

int64_t oracle_weight_count(const oracle_arch *a)
{
    int64_t n = 0;
    int C = a->obs_c, H, W, Co;
    if (torso_out_dims(a, &H, &W, &Co)) return 0;
    if (a->torso == 0) {
        for (int l = 0; l < a->n_conv; ++l) {
            n += (int64_t)a->conv_k[l] * a->conv_k[l] * C * a->conv_ch[l] + a->conv_ch[l];
            C = a->conv_ch[l];
        }
    } else {
        for (int s = 0; s < a->n_sections; ++s) {
            int ch = a->section_ch[s];
            n += (int64_t)9 * C * ch + ch;
            n += 4 * ((int64_t)9 * ch * ch + ch);
            C = ch;
        }
    }
    int64_t flat = (int64_t)H * W * Co;
    n += flat * a->fc_units + a->fc_units;
    int core = a->fc_units;
    if (a->lstm_units > 0) {
        int Z = a->fc_units + a->num_actions + 1;
        n += (int64_t)(Z + a->lstm_units) * 4 * a->lstm_units + 4 * a->lstm_units;
        core = a->lstm_units;
    }
    if (a->head == 0) {
        n += (int64_t)core * a->num_actions + a->num_actions + core + 1;
    } else {
        n += 2 * ((int64_t)core * a->head_hidden + a->head_hidden);
        n += a->head_hidden + 1;
        n += (int64_t)a->head_hidden * a->num_actions + a->num_actions;
    }
    return n;
}

int64_t oracle_torso_features(const oracle_arch *a)
{
    int H, W, C;
    if (torso_out_dims(a, &H, &W, &C)) return 0;
    return (int64_t)H * W * C;
}

/* ------------------------------------------- episode boundary, exploration */

/* Episode termination flags reach the inference thread together with the
 * observations (Section 3, "Detailed Learner architecture"): a row whose flag
 * is set starts a new episode, so its recurrent core runs from the zero state
 * instead of the stored one.  Writes the state the core must use. */
void oracle_episode_state(int done, const real *h_in, const real *c_in, int Hn, real *h0, real *c0)
{
    for (int i = 0; i < Hn; ++i) {
        h0[i] = done ? (real)0 : h_in[i];
        c0[i] = done ? (real)0 : c_in[i];
    }
}

/* epsilon-greedy exploration (Appendix A.3.1: actor i of N acts epsilon-greedily
 * with epsilon_i = 0.4^(1 + 7 i / (N - 1))): with probability eps the action is
 * drawn uniformly from the A actions, otherwise the selected action is kept.
 * Both draws are caller uniforms in [0, 1): explore iff u0 < eps; the random
 * action is floor(u1 * A), clamped to A - 1. */
int oracle_epsilon_greedy(int selected, int A, real eps, real u0, real u1)
{
    if (!(u0 < eps)) return selected;
    int r = (int)floor((double)u1 * (double)A);
    if (r < 0) r = 0;
    if (r > A - 1) r = A - 1;
    return r;
}

/* -------------------------------------------------------------- forward */

static void forward_row(const oracle_arch *a, const real *w, const uint8_t *obs,
                        int prev_action, real prev_reward,
                        const real *h_in, const real *c_in, const real *u,
                        int32_t *action, real *logits, real *value,
                        real *h_out, real *c_out, real *probs, real *margin,
                        real *torso_feat, real *fc_act)
{
    int H = a->obs_h, W = a->obs_w, C = a->obs_c;
    int64_t n = (int64_t)H * W * C;
    real *x = (real *)malloc(sizeof(real) * (size_t)n);
    oracle_normalise(obs, n, x);

    if (a->torso == 0) {
        for (int l = 0; l < a->n_conv; ++l) {
            int k = a->conv_k[l], s = a->conv_stride[l], co = a->conv_ch[l];
            int OH = oracle_out_size(H, k, s, 0), OW = oracle_out_size(W, k, s, 0);
            int64_t wsz = (int64_t)k * k * C * co;
            real *y = (real *)malloc(sizeof(real) * (size_t)OH * OW * co);
            oracle_conv2d(x, H, W, C, w, w + wsz, k, s, 0, co, y);
            oracle_relu(y, (int64_t)OH * OW * co, y);
            w += wsz + co;
            free(x);
            x = y; H = OH; W = OW; C = co;
        }
    } else {
        for (int sct = 0; sct < a->n_sections; ++sct) {
            int co = a->section_ch[sct];
            int64_t wsz = (int64_t)9 * C * co;
            real *y = (real *)malloc(sizeof(real) * (size_t)H * W * co);
            oracle_conv2d(x, H, W, C, w, w + wsz, 3, 1, 1, co, y);
            w += wsz + co;
            free(x);
            int PH = oracle_out_size(H, 3, 2, 1), PW = oracle_out_size(W, 3, 2, 1);
            real *p = (real *)malloc(sizeof(real) * (size_t)PH * PW * co);
            oracle_maxpool_3x3_s2(y, H, W, co, p);
            free(y);
            H = PH; W = PW; C = co;
            int64_t bsz = 2 * ((int64_t)9 * C * C + C);
            for (int blk = 0; blk < 2; ++blk) {
                real *q = (real *)malloc(sizeof(real) * (size_t)H * W * C);
                oracle_residual_block(p, H, W, C, w, q);
                w += bsz;
                free(p);
                p = q;
            }
            x = p;
        }
        oracle_relu(x, (int64_t)H * W * C, x);
    }

    /* flatten in (h, w, c) order, dense, ReLU */
    int flat = H * W * C;
    if (torso_feat) memcpy(torso_feat, x, sizeof(real) * (size_t)flat);
    int F = a->fc_units;
    real *fc = (real *)malloc(sizeof(real) * (size_t)F);
    oracle_dense(x, flat, w, w + (int64_t)flat * F, F, fc);
    oracle_relu(fc, F, fc);
    w += (int64_t)flat * F + F;
    free(x);
    if (fc_act) memcpy(fc_act, fc, sizeof(real) * (size_t)F);

    const real *core = fc;
    int ncore = F;
    if (a->lstm_units > 0) {
        int Hn = a->lstm_units, Z = F + a->num_actions + 1;
        const real *lw = w, *lb = w + (int64_t)(Z + Hn) * 4 * Hn;
        oracle_lstm_cell(fc, F, prev_action, a->num_actions, prev_reward, h_in, c_in, Hn,
                         lw, lb, h_out, c_out);
        w = lb + 4 * Hn;
        core = h_out;
        ncore = Hn;
    }

    if (a->head == 0)
        oracle_head_policy_value(core, ncore, a->num_actions, w, logits, value);
    else
        oracle_head_dueling(core, ncore, a->head_hidden, a->num_actions, w, logits, value);

    if (a->select == 0)
        *action = oracle_select_greedy(logits, a->num_actions, margin);
    else
        *action = oracle_select_gumbel(logits, u, a->num_actions, NULL, margin);
    if (probs) oracle_softmax(logits, a->num_actions, probs);
    free(fc);
}

/* Whole step on a batch; rows are independent (OpenMP over rows only).
 * Optional outputs (may be NULL): probs [B,A], margin [B] (top1 - top2 of
 * what the selection compared), torso_feat [B, H*W*C] (ReLU'd, flattened
 * torso output), fc_act [B, fc_units].  Returns 0, or -1 on a bad arch. */
int oracle_forward_ext(const oracle_arch *a, const real *weights, int B,
                       const uint8_t *obs, const int32_t *prev_action, const real *prev_reward,
                       const real *h_in, const real *c_in, const real *uniforms,
                       const uint8_t *done, const real *epsilon, const real *explore_u,
                       int32_t *action, real *logits, real *value, real *h_out, real *c_out,
                       real *probs, real *margin, real *torso_feat, real *fc_act);

int oracle_forward(const oracle_arch *a, const real *weights, int B,
                   const uint8_t *obs, const int32_t *prev_action, const real *prev_reward,
                   const real *h_in, const real *c_in, const real *uniforms,
                   int32_t *action, real *logits, real *value, real *h_out, real *c_out,
                   real *probs, real *margin, real *torso_feat, real *fc_act)
{
    return oracle_forward_ext(a, weights, B, obs, prev_action, prev_reward, h_in, c_in, uniforms, NULL, NULL, NULL,
                              action, logits, value, h_out, c_out, probs, margin, torso_feat, fc_act);
}

/* The step with episode flags and epsilon-greedy exploration (each optional):
 * done [B] uint8 (non-zero: the row's core starts from the zero state),
 * epsilon [B] and explore_u [B,2] (see oracle_epsilon_greedy; applied after
 * the greedy / Gumbel-max selection, logits and values are unaffected). */
int oracle_forward_ext(const oracle_arch *a, const real *weights, int B,
                       const uint8_t *obs, const int32_t *prev_action, const real *prev_reward,
                       const real *h_in, const real *c_in, const real *uniforms,
                       const uint8_t *done, const real *epsilon, const real *explore_u,
                       int32_t *action, real *logits, real *value, real *h_out, real *c_out,
                       real *probs, real *margin, real *torso_feat, real *fc_act)
{
    int64_t flat = oracle_torso_features(a);
    if (flat <= 0 || oracle_weight_count(a) <= 0) return -1;
    int64_t frame = (int64_t)a->obs_h * a->obs_w * a->obs_c;
    int A = a->num_actions, Hn = a->lstm_units;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        real m = 0;
        real *h0 = NULL, *c0 = NULL;
        if (Hn > 0) {
            h0 = (real *)malloc(sizeof(real) * (size_t)Hn);
            c0 = (real *)malloc(sizeof(real) * (size_t)Hn);
            oracle_episode_state(done ? done[b] : 0, h_in + (int64_t)Hn * b, c_in + (int64_t)Hn * b, Hn, h0, c0);
        }
        forward_row(a, weights, obs + frame * b,
                    Hn > 0 ? prev_action[b] : 0, Hn > 0 ? prev_reward[b] : (real)0,
                    h0, c0,
                    a->select ? uniforms + (int64_t)A * b : NULL,
                    action + b, logits + (int64_t)A * b, value + b,
                    Hn > 0 ? h_out + (int64_t)Hn * b : NULL,
                    Hn > 0 ? c_out + (int64_t)Hn * b : NULL,
                    probs ? probs + (int64_t)A * b : NULL, &m,
                    torso_feat ? torso_feat + flat * b : NULL,
                    fc_act ? fc_act + (int64_t)a->fc_units * b : NULL);
        if (epsilon) action[b] = oracle_epsilon_greedy(action[b], A, epsilon[b], explore_u[2 * b], explore_u[2 * b + 1]);
        if (margin) margin[b] = m;
        free(h0);
        free(c0);
    }
    return 0;
}
