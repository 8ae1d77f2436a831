/*
 * CAWN Resonance-Layer hot path -- reference oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain fp64 statement of what the
 * path computes.  Only the test-suite, the smoke check and the benchmark's CPU-baseline
 * leg may build or call it; the GPU library shares no code, header, table or constant
 * with it and never calls it.
 *
 * What is computed (paper sections):
 *   - Temporal Syntax Cache (Sec. 3.2): causal depth-wise conv over time, hard clamp,
 *     SiLU.
 *   - Gated phasor push (Sec. 3.3 hard-threshold gate with straight-through estimator;
 *     Sec. 3.4 gated-push equations): p = g * a * (cos phi, sin phi).
 *   - gate_mode 1, the input valve as Sec. 3.3 states it ("Hard-Threshold Gating"): one logit
 *     v per (token, head); beta_sig = sigmoid(v - 3); beta_hard = beta_sig if beta_sig >= eps
 *     else 0; forward p = beta_hard * a * (cos phi, sin phi) (Sec. 3.4 gated-push equations);
 *     backward through beta = beta_hard - sg(beta_sig) + beta_sig, i.e. d beta / d v =
 *     beta_sig (1 - beta_sig) whatever the threshold did.  No per-lane threshold in this mode.
 *   - Causal phase accumulation (Sec. 3.4 accumulation equations, real form):
 *       S_r[t] = p_r[t] + gamma (S_r[t-1] cos th - S_i[t-1] sin th)
 *       S_i[t] = p_i[t] + gamma (S_r[t-1] sin th + S_i[t-1] cos th),  S[-1] = state_in or 0.
 *   - ret_mode 1, the retention gate as Sec. 3.3 item 4 and "Frequency-Dependent Retention" state
 *     it: one logit r per (token, head) (the per-head projection, its own bias included) plus a
 *     static per-harmonic bias b_k; gamma[t][h][k] = sigmoid(r[t][h] + b_k) takes the place of the
 *     constant gamma_j in the accumulation equations, which are printed with gamma_{t,j}: the
 *     retention of token t multiplies the rotated state of token t-1.  Backward: the adjoint of
 *     token t reaches token t-1 through gamma[t]; d gamma[t] = Re(conj(G[t]) e^{i th} S[t-1]) per
 *     lane (clamped like every returned per-element gradient), chained through the sigmoid and
 *     summed over the harmonics of a head into d r[t][h].  b_k is static: no gradient.
 *   - Output clamp (Sec. 3.4 clamp equation), Concat layout (Sec. 3.5).
 *   - Depth-wise harmonic convolution of the output along the harmonics of each head
 *     (Sec. 3.6), as functions of their own: oracle_harmonic_conv and its adjoint
 *     oracle_harmonic_conv_bwd.
 *   - State passing (Sec. 3.7 / Sec. 5 chunked prefill): the phase state plus the last
 *     conv_k-1 pre-conv rows.
 *   - Backward (Sec. 3.4 last paragraph, Sec. 3.5): reverse-time adjoint; clamp passes the
 *     gradient; returned per-element gradients clamped.
 *
 * Readings taken where the paper is silent (each is also listed in the design notes):
 *   - conv is a cross-correlation, last tap on the current token, optional bias;
 *   - the gate thresholds the per-lane amplitude |a| >= tau (keep when >=);
 *   - the output clamp is NOT fed back into the recurrence unless clamp_feedback=1
 *     (forward only, for quantifying the difference);
 *   - the gate DECISION is taken in fp32 (the kernel's precision): with the conv
 *     front-end the fp32 pre-activation z32 = fmaf-chain(bias, taps in order) is formed,
 *     and the decision is |A(SiLU(clamp(z32)))| >= tau evaluated in fp64 on that fp32
 *     value; without the conv it is evaluated on the fp32 input itself.  Everything else
 *     is fp64;
 *   - grad clamp applies to the returned per-element dp (= adjoint G_t) before the chain
 *     to d(amplitude), d(phase), and to each per-(b,t) term of dgamma / dtheta before the
 *     sum; the carried adjoint is not clamped.
 *
 * All arrays are dense, lane index j = h*F + k fastest.  Inputs are the same fp32 arrays the
 * GPU receives, widened to double.
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
    int32_t B, L, H, F;
    int32_t conv_k;          /* 0 = no conv front-end: inputs are already magnitude/angle */
    int32_t amp_mode;        /* 0: a = m;  1: a = min(softplus(m), 10) (Sec. 3.3 item 1)   */
    int32_t clamp_feedback;  /* 0: clamp only what is emitted; 1: carry the clamped value  */
    int32_t nthreads;        /* <=0: leave the OpenMP default                              */
    int32_t gate_mode;       /* 0: per-lane threshold on |a|;  1: per-head valve (Sec. 3.3) */
    float gate_tau;          /* threshold, same fp32 value the GPU gets; 0 = open           */
    float valve_eps;         /* gate_mode 1: the valve closes below this (paper: 0.001)     */
    int32_t ret_mode;        /* 0: constant gamma[j];  1: sigmoid(ret[t][h] + ret_bias[k])  */
    int32_t dz_f64;          /* backward: dz_re / dz_im point at doubles (an upstream gradient that another
                                oracle function produced, e.g. oracle_harmonic_conv_bwd) instead of floats */
    double conv_clamp;       /* 50 in the paper; +inf disables                              */
    double out_clamp;        /* 100; +inf disables                                          */
    double grad_clamp;       /* 100; +inf disables                                          */
} oracle_cfg;

static double clampd(double v, double c) { return v < -c ? -c : (v > c ? c : v); }
static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }
static double silu(double v) { return v / (1.0 + exp(-v)); }
static double dsilu(double v)
{
    double s = sigmoid(v);
    return s * (1.0 + v * (1.0 - s));
}
static double softplus(double v) { return v > 30.0 ? v + log1p(exp(-v)) : log1p(exp(v)); }
static double amp(int mode, double m) { return mode == 1 ? fmin(softplus(m), 10.0) : m; }
static double damp(int mode, double m)
{
    if (mode != 1) return 1.0;
    return softplus(m) < 10.0 ? sigmoid(m) : 0.0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Pre-conv input of stream s (0 magnitude, 1 angle) at time t (may be negative: history). */
static double u_at(const float *x, const float *tail_in, int L, int J, int Kc, int b, int s,
                   int j, int t)
{
    if (t >= 0) return (double)x[((size_t)b * L + t) * J + j];
    if (!tail_in) return 0.0;
    int row = t + (Kc - 1); /* oldest row first */
    return (double)tail_in[(((size_t)b * (Kc - 1) + row) * 2 + s) * J + j];
}
static float u_at_f(const float *x, const float *tail_in, int L, int J, int Kc, int b, int s,
                    int j, int t)
{
    if (t >= 0) return x[((size_t)b * L + t) * J + j];
    if (!tail_in) return 0.0f;
    int row = t + (Kc - 1);
    return tail_in[(((size_t)b * (Kc - 1) + row) * 2 + s) * J + j];
}

/*
 * Stand-alone Temporal Syntax Cache on C channels (Sec. 3.2).
 *   x [B][L][C] fp32, w [C][Kc], bias [C] or NULL, hist_in [B][Kc-1][C] or NULL (zeros),
 *   y [B][L][C] fp64, hist_out [B][Kc-1][C] fp32 or NULL.
 */
int oracle_syntax_conv(int B, int L, int C, int Kc, double conv_clamp, const float *x,
                       const float *w, const float *bias, const float *hist_in, double *y,
                       float *hist_out)
{
    if (B <= 0 || L < 0 || C <= 0 || Kc < 1) return -1;
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < L; ++t)
            for (int c = 0; c < C; ++c) {
                double z = bias ? (double)bias[c] : 0.0;
                for (int i = 0; i < Kc; ++i) {
                    int tt = t - (Kc - 1) + i;
                    double u;
                    if (tt >= 0)
                        u = (double)x[((size_t)b * L + tt) * C + c];
                    else if (hist_in)
                        u = (double)hist_in[((size_t)b * (Kc - 1) + (tt + Kc - 1)) * C + c];
                    else
                        u = 0.0;
                    z += (double)w[(size_t)c * Kc + i] * u;
                }
                y[((size_t)b * L + t) * C + c] = silu(clampd(z, conv_clamp));
            }
    if (hist_out)
        for (int b = 0; b < B; ++b)
            for (int r = 0; r < Kc - 1; ++r)
                for (int c = 0; c < C; ++c) {
                    int tt = L - (Kc - 1) + r;
                    float v;
                    if (tt >= 0)
                        v = x[((size_t)b * L + tt) * C + c];
                    else if (hist_in)
                        v = hist_in[((size_t)b * (Kc - 1) + (tt + Kc - 1)) * C + c];
                    else
                        v = 0.0f;
                    hist_out[((size_t)b * (Kc - 1) + r) * C + c] = v;
                }
    return 0;
}

/*
 * Depth-wise harmonic convolution on the path's output (Sec. 3.6, "Convolutional SwiGLU Ear", the
 * step before the dense projection): the concatenated state of a token is read as 2 H channels
 * (plane p = real / imaginary, head h) of F positions (the harmonics k of the head), and each
 * channel is convolved along k with its own Kh taps and bias.
 *   out[b][t][p][h][k] = bias[p][h] + sum_{i < Kh} w[p][h][i] * Z[b][t][p][h][k + i - (Kh-1)/2],
 *   positions outside 0 .. F-1 read as zero.
 * Readings where the paper is silent: Kh is odd and the padding symmetric ("same": every harmonic
 * keeps a position, harmonics are not a causal axis); taps are applied as deep-learning
 * libraries apply a conv1d (tap i multiplies position k + i - pad, no flip); one bias per channel.
 *   z_re, z_im [B][L][H*F] fp64; w [2][H][Kh], bias [2][H] fp32 (bias NULL: zeros);
 *   o_re, o_im [B][L][H*F] fp64.
 */
int oracle_harmonic_conv(int B, int L, int H, int F, int Kh, const double *z_re, const double *z_im,
                         const float *w, const float *bias, double *o_re, double *o_im)
{
    if (B <= 0 || L < 0 || H <= 0 || F <= 0 || Kh < 1 || Kh % 2 == 0) return -1;
    const int pad = (Kh - 1) / 2;
    const size_t J = (size_t)H * F;
    for (int p = 0; p < 2; ++p) {
        const double *z = p == 0 ? z_re : z_im;
        double *o = p == 0 ? o_re : o_im;
        for (int b = 0; b < B; ++b)
            for (int t = 0; t < L; ++t)
                for (int h = 0; h < H; ++h)
                    for (int k = 0; k < F; ++k) {
                        double acc = bias ? (double)bias[(size_t)p * H + h] : 0.0;
                        for (int i = 0; i < Kh; ++i) {
                            const int kk = k + i - pad;
                            if (kk < 0 || kk >= F) continue;
                            acc += (double)w[((size_t)p * H + h) * Kh + i] *
                                   z[((size_t)b * L + t) * J + (size_t)h * F + kk];
                        }
                        o[((size_t)b * L + t) * J + (size_t)h * F + k] = acc;
                    }
    }
    return 0;
}

/*
 * Backward of the depth-wise harmonic convolution (Sec. 3.6; the paper trains through it like through
 * any layer of the block, Sec. 4): the adjoint of oracle_harmonic_conv, term by term.  Every product
 * w[p][h][i] * Z[..][kk] that the forward adds into out[..][k] hands do[..][k] * w[p][h][i] back to
 * dZ[..][kk] and do[..][k] * Z[..][kk] to dw[p][h][i]; the bias receives the sum of do over its channel.
 *   z_re, z_im  [B][L][H*F] fp64: what the forward convolved (the path's clamped output);
 *   do_re, do_im [B][L][H*F] fp64: upstream gradient of the convolution's output;
 *   dz_re, dz_im [B][L][H*F] fp64 (written); dw [2][H][Kh], dbias [2][H] fp64 (written; either may be NULL).
 */
int oracle_harmonic_conv_bwd(int B, int L, int H, int F, int Kh, const double *z_re, const double *z_im,
                             const float *w, const double *do_re, const double *do_im, double *dz_re,
                             double *dz_im, double *dw, double *dbias)
{
    if (B <= 0 || L < 0 || H <= 0 || F <= 0 || Kh < 1 || Kh % 2 == 0) return -1;
    const int pad = (Kh - 1) / 2;
    const size_t J = (size_t)H * F;
    if (dw) memset(dw, 0, sizeof(double) * 2 * H * Kh);
    if (dbias) memset(dbias, 0, sizeof(double) * 2 * H);
    for (int p = 0; p < 2; ++p) {
        const double *z = p == 0 ? z_re : z_im;
        const double *up = p == 0 ? do_re : do_im;
        double *dz = p == 0 ? dz_re : dz_im;
        memset(dz, 0, sizeof(double) * (size_t)B * L * J);
        for (int b = 0; b < B; ++b)
            for (int t = 0; t < L; ++t)
                for (int h = 0; h < H; ++h)
                    for (int k = 0; k < F; ++k) {
                        const size_t row = ((size_t)b * L + t) * J + (size_t)h * F;
                        const double g = up[row + k];
                        if (dbias) dbias[(size_t)p * H + h] += g;
                        for (int i = 0; i < Kh; ++i) {
                            const int kk = k + i - pad;
                            if (kk < 0 || kk >= F) continue;
                            dz[row + kk] += (double)w[((size_t)p * H + h) * Kh + i] * g;
                            if (dw) dw[((size_t)p * H + h) * Kh + i] += g * z[row + kk];
                        }
                    }
    }
    return 0;
}

/* Everything the front-end produces for one (b, t, j). */
typedef struct {
    double zm, za;   /* conv pre-activations (fp64); the raw inputs when conv_k = 0 */
    double m, phi;   /* magnitude-stream and angle-stream values after the front-end */
    double a;        /* amplitude */
    int g;           /* gate (gate_mode 1: the valve is open) */
    double scale;    /* what multiplies a e^{i phi} in the forward: g, or beta_hard */
    double bsig;     /* gate_mode 1: sigmoid(v - 3) */
} front_t;

static front_t front_end(const oracle_cfg *c, const float *mag, const float *ang,
                         const float *valve, const float *conv_w, const float *conv_b,
                         const float *tail_in, int b, int t, int j)
{
    const int J = c->H * c->F, L = c->L, Kc = c->conv_k;
    front_t f;
    double gate_arg; /* fp32-representable quantity the gate decision is taken on */
    if (Kc > 0) {
        double z[2];
        float z32 = 0.0f;
        for (int s = 0; s < 2; ++s) {
            const float *x = s ? ang : mag;
            const float *w = conv_w + ((size_t)s * J + j) * Kc;
            double acc = conv_b ? (double)conv_b[(size_t)s * J + j] : 0.0;
            float acc32 = conv_b ? conv_b[(size_t)s * J + j] : 0.0f;
            for (int i = 0; i < Kc; ++i) {
                int tt = t - (Kc - 1) + i;
                acc += (double)w[i] * u_at(x, tail_in, L, J, Kc, b, s, j, tt);
                if (s == 0) acc32 = fmaf(w[i], u_at_f(x, tail_in, L, J, Kc, b, s, j, tt), acc32);
            }
            z[s] = acc;
            if (s == 0) z32 = acc32;
        }
        f.zm = z[0];
        f.za = z[1];
        f.m = silu(clampd(f.zm, c->conv_clamp));
        f.phi = silu(clampd(f.za, c->conv_clamp));
        gate_arg = silu(clampd((double)z32, c->conv_clamp));
    } else {
        f.zm = (double)mag[((size_t)b * L + t) * J + j];
        f.za = (double)ang[((size_t)b * L + t) * J + j];
        f.m = f.zm;
        f.phi = f.za;
        gate_arg = f.zm;
    }
    f.a = amp(c->amp_mode, f.m);
    if (c->gate_mode == 1) {
        /* the decision is taken on the fp32 logit, evaluated in fp64 */
        const double v = (double)valve[((size_t)b * L + t) * c->H + j / c->F];
        f.bsig = sigmoid(v - 3.0);
        f.g = f.bsig >= (double)c->valve_eps ? 1 : 0;
        f.scale = f.g ? f.bsig : 0.0;
    } else {
        f.g = fabs(amp(c->amp_mode, gate_arg)) >= (double)c->gate_tau ? 1 : 0;
        f.scale = (double)f.g;
        f.bsig = 0.0;
    }
    return f;
}

/* Retention of token t on lane j = h F + k (Sec. 3.3 item 4): what multiplies the rotated S[t-1]. */
static double retention(const oracle_cfg *c, const float *ret, const float *ret_bias,
                        const float *gamma, int b, int t, int j)
{
    if (c->ret_mode != 1) return (double)gamma[j];
    return sigmoid((double)ret[((size_t)b * c->L + t) * c->H + j / c->F] + (double)ret_bias[j % c->F]);
}

/*
 * Forward: front-end, gate, phasor, accumulation, clamp.
 *   mag, ang   [B][L][J] fp32          gamma, theta [J] fp32
 *   valve      [B][L][H] fp32 (gate_mode 1)
 *   ret        [B][L][H] fp32, ret_bias [F] fp32 (ret_mode 1; gamma is then unused)
 *   conv_w     [2][J][Kc] fp32         conv_b [2][J] fp32 or NULL   (unused when conv_k = 0)
 *   scan_in    [B][2][J] fp64 or NULL  tail_in [B][Kc-1][2][J] fp32 or NULL
 *   z_re, z_im [B][L][J] fp64          scan_out [B][2][J] fp64 or NULL (unclamped S[L-1])
 *   tail_out   [B][Kc-1][2][J] fp32 or NULL      gate [B][L][J] bytes (0/1) or NULL
 */
int oracle_phase_fwd(const oracle_cfg *c, const float *mag, const float *ang, const float *valve,
                     const float *ret, const float *ret_bias,
                     const float *gamma, const float *theta, const float *conv_w, const float *conv_b,
                     const double *scan_in, const float *tail_in, double *z_re, double *z_im,
                     double *scan_out, float *tail_out, uint8_t *gate)
{
    if (!c || c->B <= 0 || c->L < 0 || c->H <= 0 || c->F <= 0 || c->conv_k < 0) return -1;
    if (c->gate_mode == 1 && !valve) return -1;
    if (c->ret_mode == 1 ? (!ret || !ret_bias) : !gamma) return -1;
    const int B = c->B, L = c->L, J = c->H * c->F, Kc = c->conv_k;
#ifdef _OPENMP
    if (c->nthreads > 0) omp_set_num_threads(c->nthreads);
#endif
#pragma omp parallel for schedule(static)
    for (int bj = 0; bj < B * J; ++bj) {
        const int b = bj / J, j = bj % J;
        const double ct = cos((double)theta[j]), st = sin((double)theta[j]);
        double Sr = scan_in ? scan_in[((size_t)b * 2 + 0) * J + j] : 0.0;
        double Si = scan_in ? scan_in[((size_t)b * 2 + 1) * J + j] : 0.0;
        for (int t = 0; t < L; ++t) {
            front_t f = front_end(c, mag, ang, valve, conv_w, conv_b, tail_in, b, t, j);
            double pr = f.g ? f.scale * f.a * cos(f.phi) : 0.0;
            double pi = f.g ? f.scale * f.a * sin(f.phi) : 0.0;
            const double ga = retention(c, ret, ret_bias, gamma, b, t, j);
            double nr = pr + ga * (Sr * ct - Si * st);
            double ni = pi + ga * (Sr * st + Si * ct);
            double zr = clampd(nr, c->out_clamp), zi = clampd(ni, c->out_clamp);
            if (c->clamp_feedback) {
                nr = zr;
                ni = zi;
            }
            Sr = nr;
            Si = ni;
            size_t o = ((size_t)b * L + t) * J + j;
            z_re[o] = zr;
            z_im[o] = zi;
            if (gate) gate[o] = (uint8_t)f.g;
        }
        if (scan_out) {
            scan_out[((size_t)b * 2 + 0) * J + j] = Sr;
            scan_out[((size_t)b * 2 + 1) * J + j] = Si;
        }
        if (tail_out && Kc > 1)
            for (int r = 0; r < Kc - 1; ++r)
                for (int s = 0; s < 2; ++s)
                    tail_out[(((size_t)b * (Kc - 1) + r) * 2 + s) * J + j] =
                        u_at_f(s ? ang : mag, tail_in, L, J, Kc, b, s, j, L - (Kc - 1) + r);
    }
    return 0;
}

/*
 * Backward of oracle_phase_fwd (clamp_feedback must be 0).
 *   dz_re, dz_im [B][L][J] upstream gradients of the emitted (clamped) outputs: fp32, or fp64 when
 *              cfg.dz_f64 is set
 *   dscan_out    [B][2][J] fp64 or NULL     gradient w.r.t. scan_out
 *   dtail_out    [B][Kc-1][2][J] fp64 or NULL gradient w.r.t. tail_out
 * Outputs (fp64, any may be NULL except dmag, dang):
 *   dmag, dang [B][L][J]; dgamma, dtheta [J]; dconv_w [2][J][Kc]; dconv_b [2][J];
 *   dscan_in [B][2][J]; dtail_in [B][Kc-1][2][J]; gate_mode 1: dvalve [B][L][H] (needs
 *   valve_term, scratch of [B][L][J] doubles: the per-lane terms, summed per head afterwards);
 *   ret_mode 1: dret [B][L][H] (needs ret_term, the same kind of scratch); dgamma is not written.
 * Parameter gradients are overwritten (summed over b and t).
 */
int oracle_phase_bwd(const oracle_cfg *c, const float *mag, const float *ang, const float *valve,
                     const float *ret, const float *ret_bias,
                     const float *gamma, const float *theta, const float *conv_w, const float *conv_b,
                     const double *scan_in, const float *tail_in, const void *dz_re,
                     const void *dz_im, const double *dscan_out, const double *dtail_out,
                     double *dmag, double *dang, double *dgamma, double *dtheta, double *dconv_w,
                     double *dconv_b, double *dscan_in, double *dtail_in, double *dvalve,
                     double *valve_term, double *dret, double *ret_term)
{
    if (!c || c->B <= 0 || c->L < 0 || c->H <= 0 || c->F <= 0 || c->conv_k < 0 || c->conv_k > 16)
        return -1;
    if (c->clamp_feedback) return -2;
    if (c->gate_mode == 1 && (!valve || (dvalve && !valve_term))) return -1;
    if (c->ret_mode == 1 ? (!ret || !ret_bias || (dret && !ret_term)) : !gamma) return -1;
    const int B = c->B, L = c->L, J = c->H * c->F, Kc = c->conv_k;
    const double gc = c->grad_clamp;
#ifdef _OPENMP
    if (c->nthreads > 0) omp_set_num_threads(c->nthreads);
#endif
#pragma omp parallel for schedule(static)
    for (int j = 0; j < J; ++j) {
        const double ct = cos((double)theta[j]), st = sin((double)theta[j]);
        double acc_g = 0.0, acc_t = 0.0;
        double acc_w[2][16], acc_b[2] = {0.0, 0.0};
        for (int s = 0; s < 2; ++s)
            for (int i = 0; i < 16; ++i) acc_w[s][i] = 0.0;
        /* per-sequence scratch */
        double *Sr = (double *)malloc(sizeof(double) * (size_t)(L + 1) * 2);
        double *Si = Sr + (L + 1);
        front_t *fr = (front_t *)malloc(sizeof(front_t) * (size_t)(L > 0 ? L : 1));
        double *dzc = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * 2);
        for (int b = 0; b < B; ++b) {
            /* forward recompute; Sr[t+1] holds S[t], Sr[0] holds S[-1] */
            Sr[0] = scan_in ? scan_in[((size_t)b * 2 + 0) * J + j] : 0.0;
            Si[0] = scan_in ? scan_in[((size_t)b * 2 + 1) * J + j] : 0.0;
            for (int t = 0; t < L; ++t) {
                fr[t] = front_end(c, mag, ang, valve, conv_w, conv_b, tail_in, b, t, j);
                double pr = fr[t].g ? fr[t].scale * fr[t].a * cos(fr[t].phi) : 0.0;
                double pi = fr[t].g ? fr[t].scale * fr[t].a * sin(fr[t].phi) : 0.0;
                const double ga = retention(c, ret, ret_bias, gamma, b, t, j);
                Sr[t + 1] = pr + ga * (Sr[t] * ct - Si[t] * st);
                Si[t + 1] = pi + ga * (Sr[t] * st + Si[t] * ct);
            }
            /* reverse-time adjoint */
            double Gr = 0.0, Gi = 0.0;
            double Mr = 0.0, Mi = 0.0; /* what token t+1 hands back: gamma[t+1] conj(e^{i th}) G[t+1] */
            for (int t = L - 1; t >= 0; --t) {
                const double ga = retention(c, ret, ret_bias, gamma, b, t, j);
                size_t o = ((size_t)b * L + t) * J + j;
                /* the output clamp passes the gradient */
                double dSr = c->dz_f64 ? ((const double *)dz_re)[o] : (double)((const float *)dz_re)[o];
                double dSi = c->dz_f64 ? ((const double *)dz_im)[o] : (double)((const float *)dz_im)[o];
                if (t == L - 1 && dscan_out) {
                    dSr += dscan_out[((size_t)b * 2 + 0) * J + j];
                    dSi += dscan_out[((size_t)b * 2 + 1) * J + j];
                }
                /* G[t] = dS[t] + gamma[t+1] conj(e^{i th}) G[t+1] */
                Gr = dSr + Mr;
                Gi = dSi + Mi;
                Mr = ga * (Gr * ct + Gi * st);
                Mi = ga * (-Gr * st + Gi * ct);
                /* parameter terms use S[t-1] and the unclamped adjoint */
                double rr = Sr[t] * ct - Si[t] * st, ri = Sr[t] * st + Si[t] * ct; /* e^{i th} S[t-1] */
                acc_g += clampd(Gr * rr + Gi * ri, gc);
                acc_t += clampd(ga * (Gr * (-ri) + Gi * rr), gc);
                /* d gamma[t] on this lane, chained through the sigmoid */
                if (c->ret_mode == 1 && dret) ret_term[o] = clampd(Gr * rr + Gi * ri, gc) * ga * (1.0 - ga);
                /* returned dp, clamped, then chained to amplitude and phase */
                double hr = clampd(Gr, gc), hi = clampd(Gi, gc);
                double cph = cos(fr[t].phi), sph = sin(fr[t].phi);
                double da = hr * cph + hi * sph;                 /* straight-through: no gate */
                double dphi = fr[t].g ? fr[t].scale * fr[t].a * (-hr * sph + hi * cph) : 0.0;
                if (c->gate_mode == 1) {
                    /* p = beta a e^{i phi}: the valve's value multiplies d/da; its own gradient is
                       a Re(conj(dp) e^{i phi}), whatever the threshold did (straight-through) */
                    if (dvalve) valve_term[o] = fr[t].a * da;
                    da *= fr[t].scale;
                }
                double dm = da * damp(c->amp_mode, fr[t].m);
                if (Kc > 0) {
                    double km = fabs(fr[t].zm) <= c->conv_clamp ? dsilu(fr[t].zm) : 0.0;
                    double ka = fabs(fr[t].za) <= c->conv_clamp ? dsilu(fr[t].za) : 0.0;
                    dzc[t] = dm * km;
                    dzc[L + t] = dphi * ka;
                } else {
                    dmag[o] = dm;
                    dang[o] = dphi;
                }
            }
            if (dscan_in) {
                dscan_in[((size_t)b * 2 + 0) * J + j] = Mr;
                dscan_in[((size_t)b * 2 + 1) * J + j] = Mi;
            }
            if (Kc > 0) {
                /* transposed conv, weight and bias gradients, history gradient */
                for (int s = 0; s < 2; ++s) {
                    const float *x = s ? ang : mag;
                    double *dx = s ? dang : dmag;
                    const float *w = conv_w + ((size_t)s * J + j) * Kc;
                    for (int t = 0; t < L; ++t) dx[((size_t)b * L + t) * J + j] = 0.0;
                    if (dtail_in)
                        for (int r = 0; r < Kc - 1; ++r)
                            dtail_in[(((size_t)b * (Kc - 1) + r) * 2 + s) * J + j] = 0.0;
                    for (int t = 0; t < L; ++t) {
                        double d = dzc[(size_t)s * L + t];
                        acc_b[s] += d;
                        for (int i = 0; i < Kc; ++i) {
                            int tt = t - (Kc - 1) + i;
                            acc_w[s][i] += d * u_at(x, tail_in, L, J, Kc, b, s, j, tt);
                            if (tt >= 0)
                                dx[((size_t)b * L + tt) * J + j] += (double)w[i] * d;
                            else if (dtail_in)
                                dtail_in[(((size_t)b * (Kc - 1) + (tt + Kc - 1)) * 2 + s) * J + j] +=
                                    (double)w[i] * d;
                        }
                    }
                    /* tail_out rows are copies of input rows (or of tail_in rows when L < Kc-1) */
                    if (dtail_out)
                        for (int r = 0; r < Kc - 1; ++r) {
                            int tt = L - (Kc - 1) + r;
                            double d = dtail_out[(((size_t)b * (Kc - 1) + r) * 2 + s) * J + j];
                            if (tt >= 0)
                                dx[((size_t)b * L + tt) * J + j] += d;
                            else if (dtail_in)
                                dtail_in[(((size_t)b * (Kc - 1) + (tt + Kc - 1)) * 2 + s) * J + j] += d;
                        }
                }
            }
        }
        if (dgamma && c->ret_mode != 1) dgamma[j] = acc_g;
        if (dtheta) dtheta[j] = acc_t;
        if (Kc > 0) {
            for (int s = 0; s < 2; ++s) {
                if (dconv_b) dconv_b[(size_t)s * J + j] = acc_b[s];
                if (dconv_w)
                    for (int i = 0; i < Kc; ++i) dconv_w[((size_t)s * J + j) * Kc + i] = acc_w[s][i];
            }
        }
        free(Sr);
        free(fr);
        free(dzc);
    }
    if (c->gate_mode == 1 && dvalve)
        for (int b = 0; b < B; ++b)
            for (int t = 0; t < L; ++t)
                for (int h = 0; h < c->H; ++h) {
                    double sum = 0.0;
                    for (int k = 0; k < c->F; ++k) sum += valve_term[((size_t)b * L + t) * J + h * c->F + k];
                    const double bs = sigmoid((double)valve[((size_t)b * L + t) * c->H + h] - 3.0);
                    dvalve[((size_t)b * L + t) * c->H + h] = bs * (1.0 - bs) * sum;
                }
    if (c->ret_mode == 1 && dret)
        for (int b = 0; b < B; ++b)
            for (int t = 0; t < L; ++t)
                for (int h = 0; h < c->H; ++h) {
                    double sum = 0.0;
                    for (int k = 0; k < c->F; ++k) sum += ret_term[((size_t)b * L + t) * J + h * c->F + k];
                    dret[((size_t)b * L + t) * c->H + h] = sum;
                }
    return 0;
}
