// Forward entry: the decode-step kernel (calls of a few tokens) and which family of scan kernels a longer call
// runs.  The scan kernel itself is cawn_fwd_kernel.hpp; its families are instantiated in cawn_fwd_<family>.hip.
#include "cawn_fwd_kernel.hpp"

namespace cawn {

// Short calls (autoregressive decoding, Sec. 5.2 of the paper: one token per call with the state
// carried in place): no tiles, no chain.  One thread per (batch row, lane) walks the call's few tokens
// in order, with exactly the arithmetic of the tiled kernel's front-end and recurrence.
#ifndef CAWN_STEP_MAX_L
#define CAWN_STEP_MAX_L 16
#endif
template <int KC>
__global__ __launch_bounds__(256) void step_kernel(const FwdArgs a)
{
    constexpr int HALO = KC > 0 ? KC - 1 : 0;
    constexpr int HALO1 = HALO > 0 ? HALO : 1, KC1 = KC > 0 ? KC : 1;
    // harmonic convolution (Sec. 3.6): the block's 256 lanes hold whole heads; neighbours meet in LDS
    __shared__ float sZ[2][256 + 2];
    const int j = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    const bool active = j < a.J;
    const int jc = active ? j : 0;      // lanes beyond J compute on lane 0's data and store nothing
    const float *tb = a.table + jc;
    const float lr = tb[(size_t)R_LR * a.Jp], li = tb[(size_t)R_LI * a.Jp];
    const float rb = tb[(size_t)R_RBIAS * a.Jp];
    float hw[2][3] = {{0.f, 0.f, 0.f}, {0.f, 0.f, 0.f}}, hb[2] = {0.f, 0.f};
    if (a.hconv) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            hb[p] = tb[(size_t)(R_W0 + 2 * KC + 6 + p) * a.Jp];
#pragma unroll
            for (int k = 0; k < 3; ++k) hw[p][k] = tb[(size_t)(R_W0 + 2 * KC + 3 * p + k) * a.Jp];
        }
    }
    const int hk = jc % a.F;
    float wm[KC1], wa[KC1], bm = 0.f, ba = 0.f;
#pragma unroll
    for (int k = 0; k < KC1; ++k) wm[k] = wa[k] = 0.f;
    if (KC > 0) {
        bm = tb[(size_t)R_BIAS_M * a.Jp];
        ba = tb[(size_t)R_BIAS_A * a.Jp];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            wm[k] = tb[(size_t)(R_W0 + k) * a.Jp];
            wa[k] = tb[(size_t)(R_W0 + KC + k) * a.Jp];
        }
    }
    // everything this thread reads from the state is read before anything is written: in place is fine
    float Sr = 0.f, Si = 0.f, hm[HALO1], ha[HALO1];     // hm/ha: the HALO pre-conv rows before the next token
#pragma unroll
    for (int r = 0; r < HALO1; ++r) hm[r] = ha[r] = 0.f;
    if (a.state_in) {
        Sr = a.state_in[((size_t)b * 2 + 0) * a.J + jc];
        Si = a.state_in[((size_t)b * 2 + 1) * a.J + jc];
        const float *tail_in = a.state_in + (size_t)a.B * 2 * a.J;
#pragma unroll
        for (int r = 0; r < HALO; ++r) {
            hm[r] = tail_in[((size_t)(b * HALO + r) * 2 + 0) * a.J + jc];
            ha[r] = tail_in[((size_t)(b * HALO + r) * 2 + 1) * a.J + jc];
        }
    }
    const int W = (a.J + 31) >> 5;
    for (int t = 0; t < a.L; ++t) {
        if (a.ckpt && active && t % CKPT_T == 0) {     // the state before every CKPT_T-th token
            a.ckpt[(((size_t)b * a.nTc + t / CKPT_T) * 2 + 0) * a.J + j] = Sr;
            a.ckpt[(((size_t)b * a.nTc + t / CKPT_T) * 2 + 1) * a.J + j] = Si;
        }
        const size_t off = (size_t)b * a.isb + (size_t)t * a.ist + jc;
        const float um = a.bf16 ? from_bf16(reinterpret_cast<const uint16_t *>(a.mag)[off]) : a.mag[off];
        const float ua = a.bf16 ? from_bf16(reinterpret_cast<const uint16_t *>(a.ang)[off]) : a.ang[off];
        float zm, xm, phi;
        if (KC > 0) {
            zm = bm;
            float za = ba;
#pragma unroll
            for (int k = 0; k < HALO; ++k) {
                zm = __builtin_fmaf(wm[k], hm[k], zm);
                za = __builtin_fmaf(wa[k], ha[k], za);
            }
            zm = __builtin_fmaf(wm[KC1 - 1], um, zm);
            za = __builtin_fmaf(wa[KC1 - 1], ua, za);
            const float cm = clampf(zm, a.conv_clamp), ca = clampf(za, a.conv_clamp);
            xm = cm * sigmoid_fast(cm);
            phi = ca * sigmoid_fast(ca);
        } else {
            zm = um;
            xm = um;
            phi = ua;
        }
        const float amp = a.amp_mode ? __builtin_fminf(softplus_fast(xm), 10.0f) : xm;
        bool g;
        float ag;
        if (a.valve) {      // per-head valve (Sec. 3.3): beta = sigmoid(logit - 3), zero when closed
            const float vl = a.valve[((size_t)b * a.L + t) * a.H + jc / a.F];
            g = vl >= a.valve_thr;
            ag = g ? amp * sigmoid_fast(vl - 3.0f) : 0.0f;
        } else {
            g = in_gate(a.gs, zm);
            ag = g ? amp : 0.0f;
        }
        float sn, cs;
        if (a.small_angle) sincos_small(phi, sn, cs);
        else sincos_fast(phi, sn, cs);
        const float pr = ag * cs, pi = ag * sn;
        float nr, ni;
        if (a.ret) {        // data-dependent retention (Sec. 3.3 item 4); lr, li are then e^{i theta}
            const float gmv = sigmoid_fast(a.ret[((size_t)b * a.L + t) * a.H + jc / a.F] + rb);
            const float rr = __builtin_fmaf(lr, Sr, -li * Si);
            const float ri = __builtin_fmaf(li, Sr, lr * Si);
            nr = __builtin_fmaf(gmv, rr, pr);
            ni = __builtin_fmaf(gmv, ri, pi);
        } else {
            nr = __builtin_fmaf(lr, Sr, __builtin_fmaf(-li, Si, pr));
            ni = __builtin_fmaf(li, Sr, __builtin_fmaf(lr, Si, pi));
        }
        Sr = nr;
        Si = ni;
        float or_ = clampf(nr, a.out_clamp), oi_ = clampf(ni, a.out_clamp);
        if (a.hconv) {      // (uniform over the launch: every thread of the block takes the barriers)
            sZ[0][threadIdx.x + 1] = or_;
            sZ[1][threadIdx.x + 1] = oi_;
            __syncthreads();
            const float lzr = hk > 0 ? sZ[0][threadIdx.x] : 0.f, lzi = hk > 0 ? sZ[1][threadIdx.x] : 0.f;
            const float rzr = hk < a.F - 1 ? sZ[0][threadIdx.x + 2] : 0.f, rzi = hk < a.F - 1 ? sZ[1][threadIdx.x + 2] : 0.f;
            or_ = __builtin_fmaf(hw[0][2], rzr, __builtin_fmaf(hw[0][1], or_, __builtin_fmaf(hw[0][0], lzr, hb[0])));
            oi_ = __builtin_fmaf(hw[1][2], rzi, __builtin_fmaf(hw[1][1], oi_, __builtin_fmaf(hw[1][0], lzi, hb[1])));
            __syncthreads();
        }
        if (active) {
            const size_t o = (size_t)b * a.osb + (size_t)t * a.ost + j;
            if (a.bf16) {
                reinterpret_cast<uint16_t *>(a.z_re)[o] = to_bf16(or_);
                reinterpret_cast<uint16_t *>(a.z_im)[o] = to_bf16(oi_);
            } else {
                a.z_re[o] = or_;
                a.z_im[o] = oi_;
            }
        }
        if (a.mask) {   // bit j%32 of word j/32: one ballot covers two words
            const unsigned long long bal = __ballot(g && active);
            if ((threadIdx.x & 31) == 0 && active)
                a.mask[((size_t)b * a.L + t) * W + (j >> 5)] = (uint32_t)(bal >> (threadIdx.x & 32));
        }
#pragma unroll
        for (int r = 0; r + 1 < HALO; ++r) { hm[r] = hm[r + 1]; ha[r] = ha[r + 1]; }
        if (HALO > 0) { hm[HALO1 - 1] = um; ha[HALO1 - 1] = ua; }
    }
    if (a.state_out && active) {
        a.state_out[((size_t)b * 2 + 0) * a.J + j] = Sr;
        a.state_out[((size_t)b * 2 + 1) * a.J + j] = Si;
        float *tail_out = a.state_out + (size_t)a.B * 2 * a.J;
#pragma unroll
        for (int r = 0; r < HALO; ++r) {
            tail_out[((size_t)(b * HALO + r) * 2 + 0) * a.J + j] = hm[r];
            tail_out[((size_t)(b * HALO + r) * 2 + 1) * a.J + j] = ha[r];
        }
    }
}

static hipError_t launch_step(const FwdArgs &a, int conv_k, hipStream_t s)
{
    const dim3 grid((unsigned)((a.J + 255) / 256), (unsigned)a.B), block(256);
    switch (conv_k) {
    case 0: hipLaunchKernelGGL(step_kernel<0>, grid, block, 0, s, a); break;
    case 1: hipLaunchKernelGGL(step_kernel<1>, grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL(step_kernel<2>, grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL(step_kernel<3>, grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL(step_kernel<4>, grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    if (a.L <= CAWN_STEP_MAX_L) return launch_step(a, conv_k, s);
    if (a.ret) return a.valve ? launch_fwd_valve_ret(a, conv_k, vec, s) : launch_fwd_ret(a, conv_k, vec, s);
    return a.valve ? launch_fwd_valve(a, conv_k, vec, s) : launch_fwd_plain(a, conv_k, vec, s);
}

}  // namespace cawn
