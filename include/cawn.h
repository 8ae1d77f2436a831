/*
 * libcawn -- the hot path of CAWN's Resonance Layer on one AMD MI355X (gfx950), C ABI.
 *
 * Operation (paper: Sec. 3.2 Temporal Syntax Cache, Sec. 3.3 hard-threshold gate with
 * straight-through estimator, Sec. 3.4 causal phase accumulation and its clamp, Sec. 3.5 Concat
 * output and clamped returned gradients, Sec. 3.7 / Sec. 5 O(1) state passing):
 *
 *   per batch row b, token t, lane j = h*F + k (H heads x F frequencies, j fastest in memory)
 *     z_s   = bias_s[j] + sum_{i<conv_k} w_s[j][i] * u_s[t-(conv_k-1)+i][j]      s in {mag, ang}
 *     x_s   = SiLU(clamp(z_s, +-conv_clamp))            (conv_k = 0: x_s = u_s, no conv, no SiLU)
 *     a     = x_mag (amp_mode 0)  |  min(softplus(x_mag), 10) (amp_mode 1);   phi = x_ang
 *     g     = [ |a| >= gate_tau ]                        (forward only; backward ignores g for a)
 *     p     = g * a * (cos phi, sin phi)
 *   gate_mode 1 (the *_valve_* entry points; Sec. 3.3 "Hard-Threshold Gating"): one logit v per
 *   (token, head) replaces g:
 *     beta  = sigmoid(v - 3) if sigmoid(v - 3) >= valve_eps else 0
 *     p     = beta * a * (cos phi, sin phi);  backward: d beta / d v = sig (1 - sig) always
 *     S[t]  = p + gamma[j] * e^{i theta[j]} * S[t-1]     (complex, written out in real fp32
 *                                                         arithmetic), S[-1] = state_in or 0
 *     Z[t]  = clamp(S[t], +-out_clamp)                   (the carried S is not clamped)
 *
 * Every pointer below is DEVICE memory owned by the caller unless it says "host".  All tensors
 * are fp32.  The library allocates nothing, frees nothing and never synchronises: each call
 * enqueues its kernels on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 * and returns.  Calls that share a workspace must be ordered on one stream.
 *
 * Return value: CAWN_OK (0) or a negative cawn_status.  Nothing is written to stdout/stderr.
 */
#ifndef CAWN_H_
#define CAWN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cawn_status {
    CAWN_OK = 0,
    CAWN_EINVAL = -1,       /* null required pointer, non-positive size, bad stride            */
    CAWN_EUNSUPPORTED = -2, /* valid request this build does not implement                     */
    CAWN_EWORKSPACE = -3,   /* workspace too small or misaligned (needs 256-byte alignment)    */
    CAWN_ELAUNCH = -4,      /* the HIP runtime refused a launch or copy                        */
    CAWN_ETIMEOUT = -5      /* (cawn_workspace_status only) a tile gave up waiting for a carry */
} cawn_status;

typedef struct cawn_desc {
    int32_t B, L, H, F;   /* L = tokens in THIS call (0 allowed: state is passed through).
                             One call spans at most 2^18 tiles: B * ceil(L/256) * ceil(H*F/32)
                             forward, B * ceil(L/128) * ceil(H*F/32) backward; beyond that
                             CAWN_EUNSUPPORTED (pass the sequence in chunks: state_in/state_out) */
    int32_t conv_k;       /* 0 = no conv front-end; 1..4 taps (paper: 3; benchmark configs: 4)  */
    int32_t amp_mode;     /* 0 amplitude = magnitude stream; 1 = min(softplus(.), 10), Sec. 3.3 */
    int32_t gate_mode;    /* 0 per-lane threshold on |a| (cawn_phase_accumulate_fwd/_bwd);
                             1 per-head input valve (cawn_phase_accumulate_valve_fwd/_bwd; needs
                             F % 32 == 0, F == 16 or F == 8, CAWN_EUNSUPPORTED otherwise); any other
                             value, or a mode passed to an entry point that is not its own:
                             CAWN_EINVAL                                                         */
    float gate_tau;       /* gate_mode 0: keep when |a| >= gate_tau; 0 = gate open              */
    float conv_clamp;     /* 50 in the paper; +inf disables                                     */
    float out_clamp;      /* 100; +inf disables                                                 */
    float grad_clamp;     /* 100; +inf disables (backward only)                                 */
    int32_t accumulate_param_grads; /* backward: 0 overwrite, 1 add into dgamma/dtheta/dconv_*  */
    int32_t lane_consts_cached;     /* 1: gamma (ret_mode 1: ret_bias), theta, conv_w, conv_b
                                       are unchanged since the last call on this workspace with
                                       the same H, F, conv_k, ret_mode that had this flag 0 --
                                       skip rebuilding the lane table                           */
    float valve_eps;      /* gate_mode 1: the valve closes below this (paper: 0.001)            */
    int32_t ret_mode;     /* 0 constant per-lane retention gamma[j]; 1 data-dependent retention
                             sigmoid(ret[t][h] + ret_bias[k]) (cawn_phase_accumulate_ret_fwd/_bwd; same
                             head widths as gate_mode 1)                                        */
    int32_t hconv_k;      /* 0: none; 3: the depth-wise harmonic convolution is applied to the output
                             before it is stored (cawn_phase_accumulate_hconv_fwd / _hconv_bwd only;
                             every other call wants 0, CAWN_EINVAL otherwise)                    */
    int64_t in_stride_b, in_stride_t;   /* element strides of mag/ang/dmag/dang; 0 = dense
                                           (t stride J, b stride L*J); lane stride is always 1;
                                           t strides above 2^21 elements: CAWN_EUNSUPPORTED     */
    int64_t out_stride_b, out_stride_t; /* element strides of z_re/z_im/dz_re/dz_im; 0 = dense  */
} cawn_desc;

/* State blob (Sec. 3.7 and Sec. 5.1: the fixed-size phase state that chunked prefill and decoding
 * carry; Sec. 5.2: the two-step history of the Temporal Syntax Cache beside it):
 * [B][2][J] scan state (re, im of S at the last token, unclamped) followed by
 * [B][conv_k-1][2][J] conv history (last conv_k-1 PRE-conv rows, oldest first, mag then ang).
 * J = H*F.  The same layout is used for the gradient blobs dstate_out / dstate_in.
 * Returns 0 for an invalid descriptor. */
size_t cawn_state_bytes(const cawn_desc *d);

/* Scratch the kernels need to evaluate the recurrence of Sec. 3.4 tile-parallel: the carries that
 * the time tiles of one lane publish to each other, the per-lane constants (powers of
 * gamma e^{i theta}, conv taps), and the per-tile partial sums of the parameter gradients (Sec. 3.5).
 * Must be 256-byte aligned and must have been passed ONCE to cawn_workspace_init before its first
 * use; calls leave it ready for the next call, with any descriptor.  Returns 0 for an invalid
 * descriptor. */
size_t cawn_workspace_bytes(const cawn_desc *d);

/* Forward checkpoints the backward consumes (the gradients of the retention and of the rotation
 * angle, Sec. 3.5, need the state S[t-1] of Sec. 3.4; it is rebuilt from these instead of being
 * stored per token): the unclamped scan state before every cawn_tile_len()-th token,
 * [B][ceil(L / cawn_tile_len())][2][J].  Returns 0 for an invalid descriptor. */
size_t cawn_ckpt_bytes(const cawn_desc *d);

/* Tokens between checkpoints (the run of tokens one backward thread owns). */
int32_t cawn_tile_len(void);

const char *cawn_status_string(int status);

/* Zero the control words of a freshly allocated workspace (enqueues a fill kernel). */
int cawn_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Synchronises `stream`, then reports CAWN_ETIMEOUT if any tile of an earlier call on this
 * workspace gave up waiting for its predecessor (its outputs are then invalid), else CAWN_OK.
 * Clears the condition.  Diagnostic only; the compute calls never wait on the host. */
int cawn_workspace_status(void *workspace, void *stream);

/* Number of polls a tile spends waiting for its predecessor's carry before it gives up
 * (default 1<<20, about a second; every wave exits either way).  Host-side setting, applies to later calls. */
void cawn_set_spin_limit(uint32_t polls);

/* Rotation angles as the paper initialises them (Sec. 3.4): theta_j = 10000^(-2j/(H*F)).
 * theta_host: HOST buffer of H*F floats. */
int cawn_theta_init(int32_t H, int32_t F, float *theta_host);

/*
 * Temporal Syntax Cache alone (Sec. 3.2) on C independent channels:
 *   y[b][t][c] = SiLU(clamp(bias[c] + sum_i w[c][i] * x[b][t-(conv_k-1)+i][c], +-conv_clamp)).
 * Uses d->B, d->L, d->conv_k (1..4), d->conv_clamp, d->in_stride_* for x, d->out_stride_* for y.
 *   x [B][L][C]; w [C][conv_k]; bias [C] or NULL; conv_state_in [B][conv_k-1][C] or NULL (zeros);
 *   y [B][L][C]; conv_state_out [B][conv_k-1][C] or NULL.  conv_state_in may alias
 *   conv_state_out.  x must not alias y.
 */
int cawn_syntax_conv(const cawn_desc *d, int32_t C, const float *x, const float *w,
                     const float *bias, const float *conv_state_in, float *y,
                     float *conv_state_out, void *stream);

/*
 * Fused forward (Sec. 3.2 - 3.5): conv front-end, gate, phasor, phase accumulation, clamp.
 *   mag, ang     [B][L][J] (pre-conv when conv_k > 0), strides d->in_stride_*
 *   gamma, theta [J]
 *   conv_w       [2][J][conv_k] (stream 0 = mag, 1 = ang), conv_b [2][J] or NULL; both ignored
 *                when conv_k = 0
 *   state_in     state blob or NULL (= sequence start: zero state, zero history)
 *   z_re, z_im   [B][L][J], strides d->out_stride_*; z_im == z_re + J with out_stride_t = 2J
 *                gives the paper's Concat(P_re, P_im) rows
 *   state_out    state blob or NULL; MAY alias state_in (streaming in place)
 *   ckpt         cawn_ckpt_bytes() or NULL when no backward will follow
 *   gate_mask    [B][L][ceil(J/32)] uint32, bit (j%32) of word j/32 = g, or NULL
 *   workspace    >= cawn_workspace_bytes(d)
 * Inputs must not alias outputs.
 */
int cawn_phase_accumulate_fwd(const cawn_desc *d, const float *mag, const float *ang,
                              const float *gamma, const float *theta, const float *conv_w,
                              const float *conv_b, const void *state_in, float *z_re, float *z_im,
                              void *state_out, void *ckpt, uint32_t *gate_mask, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * Backward of the fused forward (Sec. 3.4 last paragraph, Sec. 3.5): reverse-time adjoint
 *   G[t] = dZ[t] + conj(lambda) G[t+1]   (the output clamp passes the gradient),
 * returned per-element gradient clamp(G, +-grad_clamp) chained to the amplitude (no gate factor:
 * straight-through) and to the phase (gate factor), then through SiLU', the conv clamp's
 * sub-gradient and the transposed conv.  Parameter gradients: per-(b,t) terms clamped to
 * +-grad_clamp, then summed in a fixed order (bitwise repeatable).
 *   mag, ang, gamma, theta, conv_w, conv_b, state_in: exactly what the forward call received
 *   ckpt         written by that forward call (same d->L, H, F); required when dgamma or dtheta
 *                is requested, may be NULL otherwise
 *   dz_re, dz_im [B][L][J], strides d->out_stride_*
 *   dstate_out   gradient w.r.t. state_out (state-blob layout) or NULL (= zeros: truncated BPTT)
 *   dmag, dang   [B][L][J], strides d->in_stride_*
 *   dgamma, dtheta [J] or NULL; dconv_w [2][J][conv_k], dconv_b [2][J] or NULL
 *   dstate_in    state-blob layout or NULL
 */
int cawn_phase_accumulate_bwd(const cawn_desc *d, const float *mag, const float *ang,
                              const float *gamma, const float *theta, const float *conv_w,
                              const float *conv_b, const void *state_in, const void *ckpt,
                              const float *dz_re, const float *dz_im, const void *dstate_out,
                              float *dmag, float *dang, float *dgamma, float *dtheta,
                              float *dconv_w, float *dconv_b, void *dstate_in, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * The same two operations with the per-head input valve of Sec. 3.3 ("Hard-Threshold Gating",
 * gated-push equations of Sec. 3.4) in place of the per-lane threshold; d->gate_mode must be 1.
 *   valve        [B][L][H] fp32 logits, dense.  The decision sigmoid(v - 3) >= valve_eps is
 *                taken on the fp32 logit, evaluated in double precision.
 *   gate_mask    bit j = the valve of lane j's head is open
 *   dvalve       [B][L][H] gradient w.r.t. the logits (straight-through: closed valves get one
 *                too), or NULL
 * Everything else as in cawn_phase_accumulate_fwd / _bwd (d->gate_tau is ignored).  The workspace
 * size depends on gate_mode: ask cawn_workspace_bytes with the same descriptor.
 */
int cawn_phase_accumulate_valve_fwd(const cawn_desc *d, const float *mag, const float *ang,
                                    const float *valve, const float *gamma, const float *theta,
                                    const float *conv_w, const float *conv_b, const void *state_in,
                                    float *z_re, float *z_im, void *state_out, void *ckpt,
                                    uint32_t *gate_mask, void *workspace, size_t workspace_bytes,
                                    void *stream);
int cawn_phase_accumulate_valve_bwd(const cawn_desc *d, const float *mag, const float *ang,
                                    const float *valve, const float *gamma, const float *theta,
                                    const float *conv_w, const float *conv_b, const void *state_in,
                                    const void *ckpt, const float *dz_re, const float *dz_im,
                                    const void *dstate_out, float *dmag, float *dang, float *dvalve,
                                    float *dgamma, float *dtheta, float *dconv_w, float *dconv_b,
                                    void *dstate_in, void *workspace, size_t workspace_bytes,
                                    void *stream);

/*
 * Forward with the data-dependent retention gate of Sec. 3.3 (item 4 of the projection list,
 * "Frequency-Dependent Retention"): in the accumulation equations of Sec. 3.4 the constant
 * gamma[j] is replaced by gamma[t][h][k] = sigmoid(ret[t][h] + ret_bias[k]), which scales what
 * arrives from token t-1.  d->ret_mode must be 1; d->gate_mode selects the gate as above.
 *   valve        [B][L][H] logits when d->gate_mode == 1, ignored (may be NULL) otherwise
 *   ret          [B][L][H] fp32 retention logits, dense (the per-head projection, its own bias
 *                included)
 *   ret_bias     [F] fp32, the static per-harmonic bias b_k (paper: linear from +3 to 0); part
 *                of the lane constants (see d->lane_consts_cached)
 * There is no gamma argument.  Everything else, errors included, as in
 * cawn_phase_accumulate_fwd; head widths as for gate_mode 1; the workspace size depends on
 * ret_mode.  A workspace's cached lane constants are only valid for the ret_mode they were built
 * with.
 */
int cawn_phase_accumulate_ret_fwd(const cawn_desc *d, const float *mag, const float *ang,
                                  const float *valve, const float *ret, const float *ret_bias,
                                  const float *theta, const float *conv_w, const float *conv_b,
                                  const void *state_in, float *z_re, float *z_im, void *state_out,
                                  void *ckpt, uint32_t *gate_mask, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Backward of cawn_phase_accumulate_ret_fwd.  The adjoint of token t reaches token t-1 through
 * gamma[t]: G[t] = dZ[t] + gamma[t+1] conj(e^{i theta}) G[t+1]; the retention's own gradient is
 * d gamma[t] = Re(conj(G[t]) e^{i theta} S[t-1]) per lane, clamped to +-grad_clamp like every
 * returned per-element gradient, chained through the sigmoid and summed over the harmonics of a
 * head.  ret_bias is static (Sec. 3.3): it receives no gradient.
 *   dvalve       [B][L][H] or NULL (d->gate_mode == 1 only, ignored otherwise)
 *   dret         [B][L][H] gradient w.r.t. the retention logits, or NULL
 *   ckpt         required: the forward state before each token enters d gamma
 * There is no gamma / dgamma.  Everything else as in cawn_phase_accumulate_bwd.
 */
int cawn_phase_accumulate_ret_bwd(const cawn_desc *d, const float *mag, const float *ang,
                                  const float *valve, const float *ret, const float *ret_bias,
                                  const float *theta, const float *conv_w, const float *conv_b,
                                  const void *state_in, const void *ckpt, const float *dz_re,
                                  const float *dz_im, const void *dstate_out, float *dmag,
                                  float *dang, float *dvalve, float *dret, float *dtheta,
                                  float *dconv_w, float *dconv_b, void *dstate_in, void *workspace,
                                  size_t workspace_bytes, void *stream);
/*
 * Forward with bfloat16 activations in memory (the paper runs the network in bf16 and this
 * accumulator in fp32: Sec. 3.5, Sec. 6.1): mag, ang, z_re, z_im hold bf16 values (the upper 16 bits
 * of an fp32), strides count bf16 elements; inputs are widened exactly, all arithmetic, the carried
 * state, the checkpoints and the lane constants stay fp32, outputs are rounded to nearest even.
 * d->gate_mode and d->ret_mode select the variant: valve is read when gate_mode == 1; ret and
 * ret_bias when ret_mode == 1 (gamma is then ignored), gamma otherwise; unused ones may be NULL.
 * Needs an even H*F, even strides and 4-byte aligned mag/ang (CAWN_EUNSUPPORTED otherwise).
 * Everything else as in cawn_phase_accumulate_fwd.
 */
int cawn_phase_accumulate_bf16_fwd(const cawn_desc *d, const uint16_t *mag, const uint16_t *ang,
                                   const float *valve, const float *ret, const float *ret_bias,
                                   const float *gamma, const float *theta, const float *conv_w,
                                   const float *conv_b, const void *state_in, uint16_t *z_re,
                                   uint16_t *z_im, void *state_out, void *ckpt, uint32_t *gate_mask,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Forward with the depth-wise harmonic convolution fused behind the output clamp (the first step of
 * the paper's "Convolutional SwiGLU Ear", Sec. 3.6; its backward is cawn_phase_accumulate_hconv_bwd).  The
 * clamped state of a token is read as 2 H channels (plane p = real / imaginary, head h) of F
 * positions (the harmonics k of the head) and every channel is convolved along k with its own three
 * taps and bias, zeros beyond both ends of the head:
 *   zc_p[b][t][h*F + k] = hconv_b[p][h] + sum_{i<3} hconv_w[p][h][i] * z_p[b][t][h*F + k + i - 1].
 * The paper gives neither the kernel size nor the padding of this convolution; three taps (as in its
 * temporal convolution), symmetric zero padding and one bias per channel are this library's reading.
 * d->hconv_k must be 3.  F must divide 32, or be 64, 128 or 256, and be at least 32 with gate_mode 1
 * or ret_mode 1 (CAWN_EUNSUPPORTED otherwise).
 *   hconv_w  device [2][H][3] fp32;  hconv_b  device [2][H] fp32 or NULL (zeros)
 *   zc_re, zc_im  outputs, laid out like z_re, z_im of cawn_phase_accumulate_fwd
 *   activations_bf16  0: mag, ang, zc_re, zc_im are fp32;  1: bfloat16 with the rules of
 *                     cawn_phase_accumulate_bf16_fwd (the convolution runs in fp32 on the unrounded
 *                     clamped state; only its result is rounded)
 * state_out, ckpt and gate_mask are those of the unconvolved recurrence.  valve / ret / ret_bias /
 * gamma are selected by d->gate_mode and d->ret_mode as in cawn_phase_accumulate_bf16_fwd.  The lane
 * constants that d->lane_consts_cached keeps include hconv_w and hconv_b; the workspace size depends
 * on d->hconv_k.  Everything else as in cawn_phase_accumulate_fwd.
 */
int cawn_phase_accumulate_hconv_fwd(const cawn_desc *d, const void *mag, const void *ang,
                                    const float *valve, const float *ret, const float *ret_bias,
                                    const float *gamma, const float *theta, const float *conv_w,
                                    const float *conv_b, const float *hconv_w, const float *hconv_b,
                                    const void *state_in, void *zc_re, void *zc_im, void *state_out,
                                    void *ckpt, uint32_t *gate_mask, void *workspace,
                                    size_t workspace_bytes, int32_t activations_bf16, void *stream);

/*
 * Backward of cawn_phase_accumulate_hconv_fwd (Sec. 3.6 trained end to end with the layer, Sec. 4): the
 * upstream gradients dc_re, dc_im are those of the CONVOLVED output.  The kernel applies the transposed
 * harmonic convolution while it reads them,
 *   dz_p[k] = w_p[h][0] dc_p[k+1] + w_p[h][1] dc_p[k] + w_p[h][2] dc_p[k-1]   (inside the head only),
 * runs the backward of cawn_phase_accumulate_bwd on dz, and returns beside its gradients
 *   dhconv_w [2][H][3]:  d w_p[h][i] = sum over b, t, k of dc_p[k] * z_p[k + i - 1]
 *   dhconv_b [2][H]:     d b_p[h]    = sum over b, t, k of dc_p[k]
 * where z is the clamped state of the forward (rebuilt from ckpt, never read from memory; the output
 * clamp passes the gradient).  Neither is clamped by grad_clamp; both follow accumulate_param_grads and
 * may be NULL.  d->hconv_k must be 3, head widths as in the forward; ckpt is required.
 * d->gate_mode and d->ret_mode select the variant as in the forward: valve is read and dvalve written when
 * gate_mode == 1; ret, ret_bias are read and dret written when ret_mode == 1 (gamma is then ignored and dgamma
 * must be NULL), gamma otherwise; unused ones may be NULL.  Those variants are the backward of
 * cawn_phase_accumulate_valve_bwd / _ret_bwd behind the same transposed convolution.
 *   activations_bf16  0: mag, ang, dc_re, dc_im, dmag, dang are fp32;  1: bfloat16 with the rules of
 *                     cawn_phase_accumulate_bf16_bwd (every other gradient stays fp32)
 * dc_re, dc_im use the out strides.  The lane constants that d->lane_consts_cached keeps include hconv_w
 * and hconv_b.  Everything else (arguments, layouts, ownership, errors) as in cawn_phase_accumulate_bwd.
 */
int cawn_phase_accumulate_hconv_bwd(const cawn_desc *d, const void *mag, const void *ang,
                                    const float *valve, const float *ret, const float *ret_bias,
                                    const float *gamma, const float *theta, const float *conv_w,
                                    const float *conv_b, const float *hconv_w, const float *hconv_b,
                                    const void *state_in, const void *ckpt, const void *dc_re,
                                    const void *dc_im, const void *dstate_out, void *dmag, void *dang,
                                    float *dvalve, float *dret, float *dgamma, float *dtheta,
                                    float *dconv_w, float *dconv_b, float *dhconv_w, float *dhconv_b,
                                    void *dstate_in, void *workspace, size_t workspace_bytes,
                                    int32_t activations_bf16, void *stream);

/*
 * Backward of cawn_phase_accumulate_bf16_fwd: mag, ang, dz_re, dz_im are read and dmag, dang are
 * written as bfloat16 (rounded to nearest even); every other gradient, the state gradients and
 * the checkpoints are fp32.  Streams and gradients that the descriptor's modes do not use are
 * ignored and may be NULL (dgamma with ret_mode 1, dvalve without gate_mode 1, dret without
 * ret_mode 1).  The conv history inside state_in is fp32 as in every other call.  Everything else
 * as in cawn_phase_accumulate_bwd / _valve_bwd / _ret_bwd.
 */
int cawn_phase_accumulate_bf16_bwd(const cawn_desc *d, const uint16_t *mag, const uint16_t *ang,
                                   const float *valve, const float *ret, const float *ret_bias,
                                   const float *gamma, const float *theta, const float *conv_w,
                                   const float *conv_b, const void *state_in, const void *ckpt,
                                   const uint16_t *dz_re, const uint16_t *dz_im,
                                   const void *dstate_out, uint16_t *dmag, uint16_t *dang,
                                   float *dvalve, float *dret, float *dgamma, float *dtheta,
                                   float *dconv_w, float *dconv_b, void *dstate_in, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * cawn_phase_accumulate_fwd for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace
 * is a static device array inside the library, CAWN_STATIC_WS_BYTES = 8 MiB per GPU, held until the
 * process ends; the call allocates and frees nothing.  Arguments, results and errors are those of
 * cawn_phase_accumulate_fwd (d->gate_mode, d->ret_mode and d->hconv_k must be 0) without `workspace`
 * and `workspace_bytes`.  A descriptor whose forward-only scratch
 *   1 KiB + lane table (~66 rows of H*F floats) + 32 bytes * B * ceil(L/256) * roundup(H*F, 256)
 * exceeds 8 MiB is refused with CAWN_EWORKSPACE before anything is enqueued (B=8, H*F=768, L=8192
 * fits; pass longer sequences in chunks).  Every call on one GPU shares that GPU's array: calls
 * that overlap in time on one GPU race (order them on one stream), and d->lane_consts_cached refers
 * to the previous call of THIS entry point on that GPU.  The first call on a device also writes the
 * array's header; make that call outside graph capture.
 */
int cawn_phase_accumulate_fwd_static(const cawn_desc *d, const float *mag, const float *ang,
                                     const float *gamma, const float *theta, const float *conv_w,
                                     const float *conv_b, const void *state_in, float *z_re,
                                     float *z_im, void *state_out, void *ckpt, uint32_t *gate_mask,
                                     void *stream);

/*
 * Measurement aid, not part of the layer: a plain streaming copy with the forward's traffic shape
 * (two fp32 streams of n elements read, two written: 8 bytes in and 8 bytes out per element, every
 * byte touched once).  What it reaches on the device at hand is the practical ceiling against which
 * the HBM roofline fractions of the scan kernels are read.  n must be a multiple of 4 and the four
 * device pointers 16-byte aligned (CAWN_EUNSUPPORTED otherwise); inputs must not alias outputs.
 */
int cawn_stream_copy(const float *in0, const float *in1, float *out0, float *out1, size_t n,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CAWN_H_ */
