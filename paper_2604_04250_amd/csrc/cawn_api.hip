// Host side of libcawn: argument checks, workspace layout, the gate's fp32 breakpoints, the lane
// table kernel, the stand-alone Temporal Syntax Cache kernel and the parameter-gradient reduction.
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>

#include "cawn_internal.hpp"
#include "cawn_gate_host.hpp"

namespace cawn {

static std::atomic<uint32_t> g_spin_limit{1u << 20};   // polls (~1 us each): a second of waiting, far beyond any real wait

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static bool desc_ok(const cawn_desc *d)
{
    if (!d) return false;
    if (d->B <= 0 || d->L < 0 || d->H <= 0 || d->F <= 0) return false;
    if ((int64_t)d->H * d->F > (1 << 24)) return false;
    if (d->conv_k < 0) return false;
    if (d->gate_mode != 0 && d->gate_mode != 1) return false;
    if (d->ret_mode != 0 && d->ret_mode != 1) return false;
    if (d->hconv_k != 0 && d->hconv_k != 3) return false;
    return true;
}

// fwd_only: the layout of a workspace that only forward calls use (the allocation-free entry point):
// published words for the forward's tiles, no backward halo, no partial sums.
static WsLayout make_layout(const cawn_desc *d, bool fwd_only = false)
{
    WsLayout w{};
    w.J = d->H * d->F;
    w.Jp = (int)align_up(w.J, 64);
    w.Jp128 = (int)align_up(w.J, 256);   // covers the widest lane block of any kernel variant
    w.nT = (d->L + BwdGeom::TILE_T - 1) / BwdGeom::TILE_T;      // backward tiles (the finer of the two tilings)
    w.nTc = (d->L + CKPT_T - 1) / CKPT_T;
    const int kc = d->conv_k > MAX_KC ? MAX_KC : d->conv_k;
    const int nT_pub = fwd_only ? (d->L + FwdGeom::TILE_T - 1) / FwdGeom::TILE_T : w.nT;
    const size_t tiles_rows = (size_t)d->B * (nT_pub > 0 ? nT_pub : 1);
    size_t o = sizeof(WsHeader);
    w.off_table = o;
    o = align_up(o + (size_t)lane_rows(kc, d->hconv_k != 0) * w.Jp * sizeof(float), 256);
    w.off_agg = o;      // published words are 8 bytes each: value + tag
    o = align_up(o + tiles_rows * 2 * w.Jp128 * sizeof(tagged_t), 256);
    w.off_pre = o;
    o = align_up(o + tiles_rows * 2 * w.Jp128 * sizeof(tagged_t), 256);
    w.off_halo = o;
    if (!fwd_only) o = align_up(o + tiles_rows * (kc > 1 ? kc - 1 : 0) * 2 * w.Jp128 * sizeof(tagged_t), 256);
    w.off_part = o;
    if (!fwd_only) o = align_up(o + tiles_rows * part_rows(kc, d->hconv_k != 0) * w.Jp128 * sizeof(float), 256);
    w.off_vpart = o;    // gate_mode 1: per-group sums of the valve's gradient terms, [B][groups][L]
    if (d->gate_mode == 1 && !fwd_only)
        o = align_up(o + (size_t)d->B * (size_t)(d->H * (d->F >= 32 ? d->F / 32 : 1)) * (size_t)(d->L > 0 ? d->L : 1) * sizeof(float), 256);
    w.off_aggp = o;     // ret_mode 1: third chained word of a tile's aggregate (product of its retentions)
    if (d->ret_mode == 1) o = align_up(o + tiles_rows * w.Jp128 * sizeof(tagged_t), 256);
    w.off_rpart = o;    // ret_mode 1: per-group sums of the retention logits' gradient terms, [B][groups][L]
    if (d->ret_mode == 1 && !fwd_only)
        o = align_up(o + (size_t)d->B * (size_t)(d->H * (d->F >= 32 ? d->F / 32 : 1)) * (size_t)(d->L > 0 ? d->L : 1) * sizeof(float), 256);
    w.off_hpart = o;    // harmonic convolution: per-lane sums of its taps' and biases' gradient terms, [8][Jp]
    if (d->hconv_k != 0 && !fwd_only) o = align_up(o + (size_t)HC_PART_ROWS * w.Jp * sizeof(float), 256);
    w.off_dbg = o;
#ifdef CAWN_TIMING
    o += (size_t)MAX_TILES * 16 * sizeof(unsigned long long);
#endif
    w.total = o;
    return w;
}

// lanes of a 32-lane block that share a valve: heads of F >= 32 lanes span whole blocks
static bool valve_shape_ok(const cawn_desc *d) { return d->F % 32 == 0 || d->F == 16 || d->F == 8; }
static int valve_groups(const cawn_desc *d) { return d->H * (d->F >= 32 ? d->F / 32 : 1); }   // per token

// ------------------------------------------------------------------------------------ kernels
// gate_mode 1: dvalve[b][t][h] = sig (1 - sig) * (sum over the head's groups of vpart[b][g][t]),
// sig = sigmoid(valve - 3): the straight-through gradient of Sec. 3.3.  One thread per (b, h, t),
// t fastest; the groups of a head are summed in index order.  valve == nullptr: the plain sum (the
// retention logits' gradient, whose terms already carry their sigmoid factor per lane).  The calling
// threads share the elements: thread `first` of `stride`.
__device__ __forceinline__ void logit_reduce(const float *__restrict__ vpart, const float *__restrict__ valve,
                                             float *__restrict__ dvalve, int B, int L, int H, int G, long long first,
                                             long long stride)
{
    const long long n = (long long)B * H * L;
    const int gph = G / H;       // groups per head
    for (long long e = first; e < n; e += stride) {
        const int t = (int)(e % L);
        const long long r = e / L;
        const int h = (int)(r % H), b = (int)(r / H);
        float sum = 0.f;
        for (int g = 0; g < gph; ++g) sum += vpart[((size_t)b * G + (size_t)h * gph + g) * L + t];
        const size_t o = ((size_t)b * L + t) * H + h;
        if (valve) {
            const float sg = 1.0f / (1.0f + expf(-(valve[o] - 3.0f)));
            sum *= sg * (1.0f - sg);
        }
        dvalve[o] = sum;
    }
}

__global__ void fill_zero_kernel(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

// Every per-lane constant the scan kernels need, formed in fp64.  One thread per (lane, slot): slot 0 writes the
// lane's plain constants and taps, every other slot one power of lambda (an fp64 pow, sine and cosine each: one
// thread per lane, working through all 26 of them in turn, took 24 us).
// gamma == nullptr (data-dependent retention): the table is built with gamma = 1, i.e. its powers
// are pure rotations, and row R_RBIAS receives the static retention bias b_k of the lane's harmonic.
constexpr int LANE_TABLE_SLOTS = 3 + FwdGeom::NSEG + BwdGeom::NSEG;
__global__ void lane_table_kernel(const float *__restrict__ gamma, const float *__restrict__ theta,
                                  const float *__restrict__ conv_w, const float *__restrict__ conv_b,
                                  const float *__restrict__ ret_bias, int F,
                                  const float *__restrict__ hconv_w, const float *__restrict__ hconv_b,
                                  float *__restrict__ table, int J, int Jp, int conv_k)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int slot = blockIdx.y;
    if (j >= Jp) return;
    auto put = [&](int row, double v) { table[(size_t)row * Jp + j] = (float)v; };
    const bool live = j < J;
    const double g = live ? (gamma ? (double)gamma[j] : 1.0) : 0.0, th = live ? (double)theta[j] : 0.0;
    auto power = [&](int n, double &re, double &im) {
        const double m = n == 0 ? 1.0 : pow(g, (double)n);
        re = m * cos(n * th);
        im = m * sin(n * th);
    };
    if (slot == 1 || slot == 2) {       // lambda^(tile length) as a double-float: forward, backward
        double tr, ti;
        power(slot == 1 ? FwdGeom::TILE_T : BwdGeom::TILE_T, tr, ti);
        const float hr = (float)tr, hi = (float)ti;
        put(slot == 1 ? R_PT_HR : R_PTB_HR, hr);
        put(slot == 1 ? R_PT_HI : R_PTB_HI, hi);
        put(slot == 1 ? R_PT_LR : R_PTB_LR, tr - (double)hr);
        put(slot == 1 ? R_PT_LI : R_PTB_LI, ti - (double)hi);
        return;
    }
    if (slot >= 3) {                    // lambda^(segment start): forward segments, then backward segments
        const bool fwd = slot - 3 < FwdGeom::NSEG;
        const int sgi = fwd ? slot - 3 : slot - 3 - FwdGeom::NSEG;
        double re, im;
        power(sgi * (fwd ? FwdGeom::NSTEP : BwdGeom::NSTEP), re, im);
        put((fwd ? R_PSEG : R_PSEGB) + 2 * sgi, re);
        put((fwd ? R_PSEG : R_PSEGB) + 2 * sgi + 1, im);
        return;
    }
    const double c = cos(th), s = sin(th);
    put(R_LR, g * c);
    put(R_LI, g * s);
    put(R_COS, c);
    put(R_SIN, s);
    put(R_GAMMA, g);
    put(R_RBIAS, live && ret_bias ? (double)ret_bias[j % F] : 0.0);
    put(R_BIAS_M, live && conv_b && conv_k > 0 ? (double)conv_b[j] : 0.0);
    put(R_BIAS_A, live && conv_b && conv_k > 0 ? (double)conv_b[(size_t)J + j] : 0.0);
    for (int sidx = 0; sidx < 2; ++sidx)
        for (int i = 0; i < conv_k; ++i)
            table[(size_t)(R_W0 + sidx * conv_k + i) * Jp + j] =
                live ? conv_w[((size_t)sidx * J + j) * conv_k + i] : 0.0f;
    if (hconv_w) {     // harmonic convolution: the taps [2][H][3] and bias [2][H] of the lane's head, per plane
        const int H = J / F, h = live ? j / F : 0;
        for (int p = 0; p < 2; ++p) {
            for (int i = 0; i < 3; ++i)
                table[(size_t)(R_W0 + 2 * conv_k + 3 * p + i) * Jp + j] = live ? hconv_w[((size_t)p * H + h) * 3 + i] : 0.0f;
            table[(size_t)(R_W0 + 2 * conv_k + 6 + p) * Jp + j] = live && hconv_b ? hconv_b[(size_t)p * H + h] : 0.0f;
        }
    }
}

// Stand-alone Temporal Syntax Cache: one thread per (channel, run of NS tokens).
template <int KC>
__global__ __launch_bounds__(256) void syntax_conv_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                          const float *__restrict__ bias,
                                                          const float *hist_in, float *__restrict__ y,
                                                          float *hist_out, int B, int L, int C,
                                                          long long xsb, long long xst, long long ysb,
                                                          long long yst, float cc, int write_hist_only)
{
    constexpr int NS = 8, HALO = KC - 1;
    const int cblocks = (C + (int)blockDim.x - 1) / (int)blockDim.x;
    const int c = (blockIdx.x % cblocks) * blockDim.x + threadIdx.x;
    const int t0 = (blockIdx.x / cblocks) * NS;
    const int b = blockIdx.y;
    if (c >= C) return;
    if (write_hist_only) {
        // history rows are copied by a second, tiny launch so that hist_in may alias hist_out
        if (t0 != 0) return;
        float rows[HALO > 0 ? HALO : 1];
        for (int q = 0; q < HALO; ++q) {
            const int t = L - HALO + q;
            rows[q] = t >= 0 ? x[(size_t)b * xsb + (size_t)t * xst + c]
                             : (hist_in ? hist_in[((size_t)b * HALO + (t + HALO)) * C + c] : 0.0f);
        }
        for (int q = 0; q < HALO; ++q) hist_out[((size_t)b * HALO + q) * C + c] = rows[q];
        return;
    }
    float wk[KC];
#pragma unroll
    for (int i = 0; i < KC; ++i) wk[i] = w[(size_t)c * KC + i];
    const float bs = bias ? bias[c] : 0.0f;
    float u[NS + HALO];
#pragma unroll
    for (int r = 0; r < NS + HALO; ++r) {
        const int t = t0 - HALO + r;
        float v = 0.0f;
        if (t >= 0 && t < L) v = x[(size_t)b * xsb + (size_t)t * xst + c];
        else if (t < 0 && hist_in && t + HALO >= 0) v = hist_in[((size_t)b * HALO + (t + HALO)) * C + c];
        u[r] = v;
    }
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int t = t0 + i;
        if (t >= L) break;
        float z = bs;
#pragma unroll
        for (int k = 0; k < KC; ++k) z = __builtin_fmaf(wk[k], u[i + k], z);
        const float zc = clampf(z, cc);
        y[(size_t)b * ysb + (size_t)t * yst + c] = zc * sigmoid_fast(zc);
    }
}

// Sum the backward tiles' parameter partials in a fixed order.  One partial is [tile][row][JB] with
// tile = chain * nLB + lb (chain = position-in-time * B + b).  Block = 32 lanes x 32 groups: group g
// sums chains g, g+32, ... of its lane's block in increasing order, then the 32 sub-sums meet in LDS
// and are added in index order -- the association is fixed, so results are bitwise repeatable.
__device__ __forceinline__ void reduce_partials(const float *__restrict__ part, float *__restrict__ out0,
                                                float *__restrict__ out1, float *__restrict__ out2,
                                                float *__restrict__ out3, float *__restrict__ out4, int rows, int conv_k,
                                                int hc_row0, int J, int JB, int nLB, int chains, int accumulate, int bx,
                                                int row)
{
    // one block per (32 lanes, row): bx, row
    constexpr int G = 32;
    __shared__ float sm[G][33];
    const int lane = threadIdx.x % 32, g = threadIdx.x / 32;
    const int j = bx * 32 + lane;
    float acc = 0.0f;
    if (j < J) {
        const int lb = j / JB, jj = j % JB;
        // (eight independent reads in flight per thread; the sum keeps its order)
        const float *src = part + ((size_t)lb * rows + row) * JB + jj;
        const size_t step = (size_t)nLB * rows * JB;      // floats between the same slot of consecutive chains
        int c = g;
        for (; c + 7 * G < chains; c += 8 * G) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(c + u * G) * step];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; c < chains; c += G) acc += src[(size_t)c * step];
    }
    sm[g][lane] = acc;
    __syncthreads();
    if (g == 0 && j < J) {
        float s = 0.0f;
#pragma unroll
        for (int qq = 0; qq < G; ++qq) s += sm[qq][lane];
        // rows: 0 dgamma, 1 dtheta, 2 dbias_m, 3 dbias_a, 4 + s*conv_k + i: dw[s][j][i]; from hc_row0 on (when
        // >= 0): the harmonic convolution's per-lane terms, kept per lane in out4 [8][J] for their own reduction
        float *dst = nullptr;
        if (hc_row0 >= 0 && row >= hc_row0) {
            out4[(size_t)(row - hc_row0) * J + j] = s;
            return;
        }
        if (row == 0) dst = out0 ? out0 + j : nullptr;
        else if (row == 1) dst = out1 ? out1 + j : nullptr;
        else if (row < 4) dst = out3 ? out3 + (size_t)(row - 2) * J + j : nullptr;
        else {
            const int sidx = (row - 4) / conv_k, i = (row - 4) % conv_k;
            dst = out2 ? out2 + ((size_t)sidx * J + j) * conv_k + i : nullptr;
        }
        if (dst) *dst = accumulate ? *dst + s : s;
    }
}

// What follows the backward kernel, in one launch (each small launch costs 4-5 us on this chip whatever it
// does): blocks [0, nbx * rows) sum the parameter partials, the blocks behind them share the logit gradients of
// the valve and of the retention (nsets of them, nb blocks each).
struct EpilogueArgs {
    const float *part;
    float *out0, *out1, *out2, *out3, *out4;
    int rows, conv_k, hc_row0, J, JB, nLB, chains, accumulate, nbx;
    const float *lpart[2], *logit[2];
    float *lout[2];
    int nsets, nb, B, L, H, G;
};
__global__ __launch_bounds__(1024) void bwd_epilogue_kernel(const EpilogueArgs p)
{
    const int nA = p.nbx * p.rows;
    if ((int)blockIdx.x < nA) {
        reduce_partials(p.part, p.out0, p.out1, p.out2, p.out3, p.out4, p.rows, p.conv_k, p.hc_row0, p.J, p.JB, p.nLB,
                        p.chains, p.accumulate, (int)blockIdx.x % p.nbx, (int)blockIdx.x / p.nbx);
        return;
    }
    const int bid = (int)blockIdx.x - nA, set = bid / p.nb, blk = bid % p.nb;
    logit_reduce(p.lpart[set], p.logit[set], p.lout[set], p.B, p.L, p.H, p.G, (long long)blk * blockDim.x + threadIdx.x,
                 (long long)p.nb * blockDim.x);
}

// Harmonic convolution (Sec. 3.6): its taps and biases belong to a (plane, head) channel, so the per-lane sums
// hpart [8][J] (rows: plane-0 taps 0..2, plane-1 taps 0..2, plane-0 bias, plane-1 bias) are summed over the F
// lanes of each head by one wave per output: lane l adds the head's lanes l, l + 64, ... in ascending order, then
// the 64 sums meet in a butterfly of lane exchanges (both partners of an exchange add the same two values, so
// every lane ends with the same bits): the association is fixed, the result repeatable.
__global__ __launch_bounds__(64) void hconv_grad_reduce_kernel(const float *__restrict__ hpart, float *__restrict__ dw,
                                                               float *__restrict__ db, int H, int F, int J, int accumulate)
{
    const int e = blockIdx.x;        // (row, head)
    const int q = e / H, h = e % H;
    const float *src = hpart + (size_t)q * J + (size_t)h * F;
    float s = 0.0f;
    for (int k = threadIdx.x; k < F; k += 64) s += src[k];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    if (threadIdx.x == 0) {
        float *dst = q < 6 ? (dw ? dw + ((size_t)(q / 3) * H + h) * 3 + q % 3 : nullptr)
                           : (db ? db + (size_t)(q - 6) * H + h : nullptr);
        if (dst) *dst = accumulate ? *dst + s : s;
    }
}

// Plain streaming copy with the forward's traffic shape: two fp32 streams in, two out, 8 bytes read and
// 8 bytes written per element, 16-byte non-temporal accesses, every byte touched once.  What this
// kernel reaches is the practical ceiling of the HBM roofline on the chip at hand; it computes nothing.
// (Of the shapes tried at 50 MB .. 1.2 GB -- grid-stride and slab-per-workgroup, 1/2/4 loads in flight,
// 2 .. 32 workgroups per CU, one element per thread -- this one was at or within 3 % of the best.)
typedef float v4f __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_copy_kernel(const v4f *__restrict__ a0, const v4f *__restrict__ a1,
                                                          v4f *__restrict__ o0, v4f *__restrict__ o1, size_t n4)
{
    constexpr int U = 4;     // independent 16-byte loads in flight per stream and thread
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + (U - 1) * stride < n4; i += U * stride) {
        v4f x[U], y[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            x[u] = __builtin_nontemporal_load(a0 + i + u * stride);
            y[u] = __builtin_nontemporal_load(a1 + i + u * stride);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            __builtin_nontemporal_store(x[u], o0 + i + u * stride);
            __builtin_nontemporal_store(y[u], o1 + i + u * stride);
        }
    }
    for (; i < n4; i += stride) {
        o0[i] = a0[i];
        o1[i] = a1[i];
    }
}

static hipError_t build_table(const cawn_desc *d, const WsLayout &w, char *ws, const float *gamma,
                              const float *theta, const float *conv_w, const float *conv_b,
                              const float *ret_bias, hipStream_t s, const float *hconv_w = nullptr,
                              const float *hconv_b = nullptr)
{
    float *table = reinterpret_cast<float *>(ws + w.off_table);
    const int threads = 128;
    hipLaunchKernelGGL(lane_table_kernel, dim3((w.Jp + threads - 1) / threads, LANE_TABLE_SLOTS), dim3(threads), 0, s,
                       gamma, theta, conv_w, conv_b, ret_bias, d->F, hconv_w, hconv_b, table, w.J, w.Jp, d->conv_k);
    return hipGetLastError();
}

static bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace cawn

using namespace cawn;

extern "C" {

size_t cawn_state_bytes(const cawn_desc *d)
{
    if (!desc_ok(d)) return 0;
    const size_t J = (size_t)d->H * d->F;
    const size_t halo = d->conv_k > 1 ? d->conv_k - 1 : 0;
    return (size_t)d->B * 2 * J * sizeof(float) * (1 + halo);
}

size_t cawn_workspace_bytes(const cawn_desc *d)
{
    if (!desc_ok(d)) return 0;
    return make_layout(d).total;
}

size_t cawn_ckpt_bytes(const cawn_desc *d)
{
    if (!desc_ok(d)) return 0;
    const size_t nT = (d->L + CKPT_T - 1) / CKPT_T;
    return (size_t)d->B * nT * 2 * d->H * d->F * sizeof(float);
}

int32_t cawn_tile_len(void) { return CKPT_T; }

const char *cawn_status_string(int st)
{
    switch (st) {
    case CAWN_OK: return "ok";
    case CAWN_EINVAL: return "invalid argument";
    case CAWN_EUNSUPPORTED: return "unsupported configuration";
    case CAWN_EWORKSPACE: return "workspace too small or misaligned";
    case CAWN_ELAUNCH: return "HIP launch or copy failed";
    case CAWN_ETIMEOUT: return "a tile gave up waiting for its predecessor's carry";
    default: return "unknown status";
    }
}

__global__ void init_header_kernel(WsHeader *h, unsigned long long bytes)
{
    h->bytes_lo = (uint32_t)bytes;
    h->bytes_hi = (uint32_t)(bytes >> 32);
}

int cawn_workspace_init(void *workspace, size_t bytes, void *stream)
{
    if (!workspace) return CAWN_EINVAL;
    if (bytes < sizeof(WsHeader) || !aligned(workspace, 256)) return CAWN_EWORKSPACE;
    // the whole buffer: a word counts as published only when its tag matches, and tag 0 never does
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1024), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<uint32_t *>(workspace), bytes / sizeof(uint32_t));
    hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream,
                       reinterpret_cast<WsHeader *>(workspace), (unsigned long long)bytes);
    return hipGetLastError() == hipSuccess ? CAWN_OK : CAWN_ELAUNCH;
}

int cawn_workspace_status(void *workspace, void *stream)
{
    if (!workspace) return CAWN_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return CAWN_ELAUNCH;
    uint32_t err = 0;
    WsHeader *h = reinterpret_cast<WsHeader *>(workspace);
    if (hipMemcpy(&err, &h->error, sizeof(err), hipMemcpyDeviceToHost) != hipSuccess) return CAWN_ELAUNCH;
    if (err) {
        uint32_t zero = 0;
        if (hipMemcpy(&h->error, &zero, sizeof(zero), hipMemcpyHostToDevice) != hipSuccess) return CAWN_ELAUNCH;
        return CAWN_ETIMEOUT;
    }
    return CAWN_OK;
}

void cawn_set_spin_limit(uint32_t polls) { g_spin_limit.store(polls); }

int cawn_theta_init(int32_t H, int32_t F, float *theta_host)
{
    if (H <= 0 || F <= 0 || !theta_host) return CAWN_EINVAL;
    const int64_t J = (int64_t)H * F;
    for (int64_t j = 0; j < J; ++j)
        theta_host[j] = (float)std::pow(10000.0, -2.0 * (double)j / (double)J);
    return CAWN_OK;
}

int cawn_syntax_conv(const cawn_desc *d, int32_t C, const float *x, const float *w, const float *bias,
                     const float *conv_state_in, float *y, float *conv_state_out, void *stream)
{
    if (!d || d->B <= 0 || d->L < 0 || C <= 0 || !w) return CAWN_EINVAL;
    if (d->conv_k < 1) return CAWN_EINVAL;
    if (d->conv_k > MAX_KC) return CAWN_EUNSUPPORTED;
    if (d->L > 0 && (!x || !y)) return CAWN_EINVAL;
    const long long xst = d->in_stride_t ? d->in_stride_t : C, xsb = d->in_stride_b ? d->in_stride_b : (long long)d->L * C;
    const long long yst = d->out_stride_t ? d->out_stride_t : C, ysb = d->out_stride_b ? d->out_stride_b : (long long)d->L * C;
    if (xst < C || yst < C) return CAWN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int NS = 8;
    const dim3 block(256);
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 0 && d->L == 0) continue;
        if (pass == 1 && (!conv_state_out || d->conv_k == 1)) continue;
        const long long nblk = (long long)((C + 255) / 256) * (pass == 0 ? (d->L + NS - 1) / NS : 1);
        if (nblk > 0x7fffffffLL || d->B > 65535) return CAWN_EUNSUPPORTED;
        const dim3 grid((unsigned)nblk, d->B, 1);
#define CAWN_CONV_CASE(K)                                                                          \
    case K:                                                                                        \
        hipLaunchKernelGGL((syntax_conv_kernel<K>), grid, block, 0, s, x, w, bias, conv_state_in, y, \
                           conv_state_out, d->B, d->L, C, xsb, xst, ysb, yst, d->conv_clamp, pass); \
        break;
        switch (d->conv_k) {
            CAWN_CONV_CASE(1) CAWN_CONV_CASE(2) CAWN_CONV_CASE(3) CAWN_CONV_CASE(4)
        }
#undef CAWN_CONV_CASE
        if (hipGetLastError() != hipSuccess) return CAWN_ELAUNCH;
    }
    return CAWN_OK;
}

static int fwd_impl(const cawn_desc *d, const float *mag, const float *ang, const float *valve,
                    const float *ret, const float *ret_bias, const float *gamma, const float *theta, const float *conv_w, const float *conv_b,
                    const void *state_in, float *z_re, float *z_im, void *state_out, void *ckpt,
                    uint32_t *gate_mask, void *workspace, size_t workspace_bytes, void *stream, bool bf16 = false,
                    const float *hconv_w = nullptr, const float *hconv_b = nullptr, bool fwd_only_ws = false)
{
    if (d->conv_k > MAX_KC || (d->amp_mode != 0 && d->amp_mode != 1)) return CAWN_EUNSUPPORTED;
    // the harmonic convolution belongs to its own entry point (which passes the taps)
    if ((d->hconv_k != 0) != (hconv_w != nullptr)) return CAWN_EINVAL;
    // heads are whole inside a 32-lane block, or made of whole blocks (and whole inside the 256 lanes of
    // a short call's workgroup)
    if (d->hconv_k != 0 && !(d->F <= 32 ? 32 % d->F == 0 : (d->F % 32 == 0 && 256 % d->F == 0))) return CAWN_EUNSUPPORTED;
    if (d->hconv_k != 0 && (d->gate_mode == 1 || d->ret_mode == 1) && d->F < 32) return CAWN_EUNSUPPORTED;   // LDS
    if ((d->gate_mode == 1 || d->ret_mode == 1) && !valve_shape_ok(d)) return CAWN_EUNSUPPORTED;
    if (d->gate_mode == 1 && d->ret_mode == 1 && d->F < 16) return CAWN_EUNSUPPORTED;   // LDS for both logit tiles
    hipStream_t s = (hipStream_t)stream;
    const WsLayout w = make_layout(d, fwd_only_ws);
    const long long J = w.J;
    if (d->L == 0) {   // nothing to scan: the state passes through
        if (state_out && state_out != state_in) {
            const size_t nb = cawn_state_bytes(d);
            hipError_t e;
            if (state_in) {
                e = hipMemcpyAsync(state_out, state_in, nb, hipMemcpyDeviceToDevice, s);
            } else {   // a fill kernel rather than a memset node: safe under graph capture
                hipLaunchKernelGGL(fill_zero_kernel, dim3(64), dim3(256), 0, s,
                                   reinterpret_cast<uint32_t *>(state_out), nb / sizeof(uint32_t));
                e = hipGetLastError();
            }
            if (e != hipSuccess) return CAWN_ELAUNCH;
        }
        return CAWN_OK;
    }
    if (!mag || !ang || !theta || !z_re || !z_im || !workspace) return CAWN_EINVAL;
    if (d->ret_mode == 1 ? (!ret || !ret_bias) : !gamma) return CAWN_EINVAL;
    if (d->gate_mode == 1 && !valve) return CAWN_EINVAL;
    if (d->conv_k > 0 && !conv_w) return CAWN_EINVAL;
    // tile indices and tickets are bounded: B x (tiles per sequence) x (32-lane blocks) <= 2^18 per call
    if ((unsigned long long)d->B * ((d->L + FwdGeom::TILE_T - 1) / FwdGeom::TILE_T) * ((J + FwdLPR - 1) / FwdLPR) > MAX_TILES)
        return CAWN_EUNSUPPORTED;
    if (workspace_bytes < w.total || !aligned(workspace, 256)) return CAWN_EWORKSPACE;
    const long long ist = d->in_stride_t ? d->in_stride_t : J, isb = d->in_stride_b ? d->in_stride_b : (long long)d->L * J;
    const long long ost = d->out_stride_t ? d->out_stride_t : J, osb = d->out_stride_b ? d->out_stride_b : (long long)d->L * J;
    if (ist < J || ost < J || isb < 0 || osb < 0) return CAWN_EINVAL;
    if (ist > (1ll << 21) || ost > (1ll << 21)) return CAWN_EUNSUPPORTED;   // in-tile offsets are 32-bit
    // bf16 rows are staged as four-byte words: an even number of lanes, even strides, aligned rows
    if (bf16 && (J % 2 || ist % 2 || isb % 2 || !aligned(mag, 4) || !aligned(ang, 4))) return CAWN_EUNSUPPORTED;

    FwdArgs a{};
    a.bf16 = bf16 ? 1 : 0;
    a.hconv = d->hconv_k != 0 ? 1 : 0;
    a.hcG = d->hconv_k != 0 && d->F > 32 ? d->F / 32 : 1;
    if (d->gate_mode == 1) {
        const float INF = std::numeric_limits<float>::infinity();
        a.gs = GateSet{-INF, INF, INF, -INF};        // no per-lane threshold in this mode
        a.valve = valve;
        a.valve_thr = valve_threshold(d->valve_eps);
    } else if (!make_gate_set(d->conv_k > 0, d->amp_mode, (double)d->conv_clamp, d->gate_tau, &a.gs)) {
        return CAWN_EUNSUPPORTED;
    }
    a.H = d->H; a.F = d->F;
    a.gpb = d->F >= 32 ? 1 : 32 / d->F;
    if (d->ret_mode == 1) {
        a.ret = ret;
        a.aggp = reinterpret_cast<tagged_t *>(reinterpret_cast<char *>(workspace) + w.off_aggp);
    }
    const bool vec = (J % FwdV == 0) && (ist % FwdV == 0) && (isb % FwdV == 0) && (ost % FwdV == 0) &&
                     (osb % FwdV == 0) && aligned(mag, 16) && aligned(ang, 16) && aligned(z_re, 16) &&
                     aligned(z_im, 16) && (!state_in || aligned(state_in, 16)) &&
                     (!state_out || aligned(state_out, 16)) && (!ckpt || aligned(ckpt, 16));
    const int JB = (vec ? FwdV : 1) * FwdLPR;
    const int nLB = (int)((J + JB - 1) / JB);
    const int nTf = (d->L + FwdGeom::TILE_T - 1) / FwdGeom::TILE_T;
    const size_t tiles = (size_t)d->B * nTf * nLB;
    if (tiles > MAX_TILES) return CAWN_EUNSUPPORTED;

    char *ws = reinterpret_cast<char *>(workspace);
    if (!d->lane_consts_cached) {
        if (build_table(d, w, ws, d->ret_mode == 1 ? nullptr : gamma, theta, conv_w, conv_b,
                        d->ret_mode == 1 ? ret_bias : nullptr, s, hconv_w, hconv_b) != hipSuccess) return CAWN_ELAUNCH;
    }
    a.mag = mag; a.ang = ang;
    a.table = reinterpret_cast<const float *>(ws + w.off_table);
    a.state_in = reinterpret_cast<const float *>(state_in);
    a.z_re = z_re; a.z_im = z_im;
    a.state_out = reinterpret_cast<float *>(state_out);
    a.ckpt = reinterpret_cast<float *>(ckpt);
    a.mask = gate_mask;
    a.hdr = reinterpret_cast<WsHeader *>(ws);
    a.agg = reinterpret_cast<tagged_t *>(ws + w.off_agg);
    a.pre = reinterpret_cast<tagged_t *>(ws + w.off_pre);
    a.clear_from = w.off_agg;
    a.B = d->B; a.L = d->L; a.J = (int)J; a.Jp = w.Jp; a.nT = nTf; a.nTc = w.nTc; a.nLB = nLB;
    a.amp_mode = d->amp_mode;
    a.small_angle = (d->conv_k > 0 && d->conv_clamp <= 256.0f) ? 1 : 0;   // |angle| <= SiLU(clamp) <= 41 revolutions
    a.stage16 = (J % 4 == 0 && ist % 4 == 0 && isb % 4 == 0 && aligned(mag, 16) && aligned(ang, 16) &&
                 (!state_in || aligned(state_in, 16))) ? 1 : 0;
    if (bf16) a.stage16 = (J % 8 == 0 && ist % 8 == 0 && isb % 8 == 0 && aligned(mag, 16) && aligned(ang, 16)) ? 1 : 0;
    a.isb = isb; a.ist = ist; a.osb = osb; a.ost = ost;
    a.conv_clamp = d->conv_clamp; a.out_clamp = d->out_clamp;
    a.spin_limit = g_spin_limit.load();
    a.total_tiles = (uint32_t)tiles;
    a.dbg = reinterpret_cast<unsigned long long *>(ws + w.off_dbg);
    if (launch_fwd(a, d->conv_k, vec, s) != hipSuccess) return CAWN_ELAUNCH;
    return CAWN_OK;
}

int cawn_phase_accumulate_fwd(const cawn_desc *d, const float *mag, const float *ang, const float *gamma,
                              const float *theta, const float *conv_w, const float *conv_b,
                              const void *state_in, float *z_re, float *z_im, void *state_out, void *ckpt,
                              uint32_t *gate_mask, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->gate_mode != 0 || d->ret_mode != 0) return CAWN_EINVAL;      // those modes have entry points of their own
    return fwd_impl(d, mag, ang, nullptr, nullptr, nullptr, gamma, theta, conv_w, conv_b, state_in, z_re, z_im, state_out, ckpt,
                    gate_mask, workspace, workspace_bytes, stream);
}

int cawn_phase_accumulate_valve_fwd(const cawn_desc *d, const float *mag, const float *ang, const float *valve,
                                    const float *gamma, const float *theta, const float *conv_w,
                                    const float *conv_b, const void *state_in, float *z_re, float *z_im,
                                    void *state_out, void *ckpt, uint32_t *gate_mask, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->gate_mode != 1 || d->ret_mode != 0) return CAWN_EINVAL;
    return fwd_impl(d, mag, ang, valve, nullptr, nullptr, gamma, theta, conv_w, conv_b, state_in, z_re, z_im,
                    state_out, ckpt, gate_mask, workspace, workspace_bytes, stream);
}

int cawn_phase_accumulate_ret_fwd(const cawn_desc *d, const float *mag, const float *ang, const float *valve,
                                  const float *ret, const float *ret_bias, const float *theta,
                                  const float *conv_w, const float *conv_b, const void *state_in, float *z_re,
                                  float *z_im, void *state_out, void *ckpt, uint32_t *gate_mask, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->ret_mode != 1) return CAWN_EINVAL;
    return fwd_impl(d, mag, ang, d->gate_mode == 1 ? valve : nullptr, ret, ret_bias, nullptr, theta, conv_w, conv_b,
                    state_in, z_re, z_im, state_out, ckpt, gate_mask, workspace, workspace_bytes, stream);
}

static int bwd_impl(const cawn_desc *d, const float *mag, const float *ang, const float *valve,
                    const float *ret, const float *ret_bias,
                    const float *gamma, const float *theta, const float *conv_w, const float *conv_b,
                    const void *state_in, const void *ckpt, const float *dz_re, const float *dz_im,
                    const void *dstate_out, float *dmag, float *dang, float *dvalve, float *dret, float *dgamma,
                    float *dtheta, float *dconv_w, float *dconv_b, void *dstate_in, void *workspace,
                    size_t workspace_bytes, void *stream, bool bf16 = false, const float *hconv_w = nullptr,
                    const float *hconv_b = nullptr, float *dhconv_w = nullptr, float *dhconv_b = nullptr)
{
    if (d->conv_k > MAX_KC || (d->amp_mode != 0 && d->amp_mode != 1)) return CAWN_EUNSUPPORTED;
    // gradients of the convolved output: the harmonic convolution's own entry point only
    const bool hc = d->hconv_k != 0;
    if (hc != (hconv_w != nullptr)) return CAWN_EINVAL;
    if (hc && !(d->F <= 32 ? 32 % d->F == 0 : (d->F % 32 == 0 && 256 % d->F == 0))) return CAWN_EUNSUPPORTED;   // as in the forward
    if (hc && (d->gate_mode == 1 || d->ret_mode == 1) && d->F < 32) return CAWN_EUNSUPPORTED;                   // as in the forward
    if ((d->gate_mode == 1 || d->ret_mode == 1) && !valve_shape_ok(d)) return CAWN_EUNSUPPORTED;
    if (d->gate_mode == 1 && d->ret_mode == 1 && d->F < 16) return CAWN_EUNSUPPORTED;   // as in the forward
    hipStream_t s = (hipStream_t)stream;
    const WsLayout w = make_layout(d);
    const long long J = w.J;
    const int kc = d->conv_k;
    const bool want_w = kc > 0 && (dconv_w || dconv_b);
    // (the retention kernels rebuild the forward state in any case and always emit their partials)
    // (the harmonic convolution's tap gradients need the clamped state: state rebuilt, partials always emitted)
    const bool want_param = dgamma || dtheta || want_w || d->ret_mode == 1 || hc;
    if (d->L == 0) {   // no tokens: the state gradient passes through, parameter gradients are zero
        auto zero = [&](void *p, size_t nfloat) {
            if (!p || !nfloat) return hipSuccess;
            hipLaunchKernelGGL(fill_zero_kernel, dim3(64), dim3(256), 0, s, reinterpret_cast<uint32_t *>(p), nfloat);
            return hipGetLastError();
        };
        const size_t nb = cawn_state_bytes(d);
        hipError_t e = hipSuccess;
        if (dstate_in && dstate_in != dstate_out)
            e = dstate_out ? hipMemcpyAsync(dstate_in, dstate_out, nb, hipMemcpyDeviceToDevice, s)
                           : zero(dstate_in, nb / 4);
        if (e == hipSuccess && !d->accumulate_param_grads) {
            e = zero(dgamma, J);
            if (e == hipSuccess) e = zero(dtheta, J);
            if (e == hipSuccess && kc > 0) e = zero(dconv_w, 2 * J * kc);
            if (e == hipSuccess && kc > 0) e = zero(dconv_b, 2 * J);
            if (e == hipSuccess && hc) e = zero(dhconv_w, (size_t)2 * d->H * 3);
            if (e == hipSuccess && hc) e = zero(dhconv_b, (size_t)2 * d->H);
        }
        return e == hipSuccess ? CAWN_OK : CAWN_ELAUNCH;
    }
    if (!mag || !ang || !theta || !dz_re || !dz_im || !dmag || !dang || !workspace) return CAWN_EINVAL;
    if (d->ret_mode == 1 ? (!ret || !ret_bias || dgamma) : !gamma) return CAWN_EINVAL;
    if (d->gate_mode == 1 && !valve) return CAWN_EINVAL;
    if (kc > 0 && !conv_w) return CAWN_EINVAL;
    if ((dgamma || dtheta || d->ret_mode == 1 || hc) && !ckpt) return CAWN_EINVAL;
    // tile indices and tickets are bounded: B x (tiles per sequence) x (32-lane blocks) <= 2^18 per call
    if ((unsigned long long)d->B * w.nT * ((J + BwdLPR - 1) / BwdLPR) > MAX_TILES) return CAWN_EUNSUPPORTED;
    if (workspace_bytes < w.total || !aligned(workspace, 256)) return CAWN_EWORKSPACE;
    const long long ist = d->in_stride_t ? d->in_stride_t : J, isb = d->in_stride_b ? d->in_stride_b : (long long)d->L * J;
    const long long ost = d->out_stride_t ? d->out_stride_t : J, osb = d->out_stride_b ? d->out_stride_b : (long long)d->L * J;
    if (ist < J || ost < J || isb < 0 || osb < 0) return CAWN_EINVAL;
    if (ist > (1ll << 21) || ost > (1ll << 21)) return CAWN_EUNSUPPORTED;   // in-tile offsets are 32-bit
    // bf16 rows are staged as four-byte words: an even number of lanes, even strides, aligned rows
    if (bf16 && (J % 2 || ist % 2 || isb % 2 || ost % 2 || osb % 2 || !aligned(mag, 4) || !aligned(ang, 4) ||
                 !aligned(dz_re, 4) || !aligned(dz_im, 4))) return CAWN_EUNSUPPORTED;

    BwdArgs a{};
    a.bf16 = bf16 ? 1 : 0;
    if (d->gate_mode == 1) {
        const float INF = std::numeric_limits<float>::infinity();
        a.gs = GateSet{-INF, INF, INF, -INF};        // no per-lane threshold in this mode
        a.valve = valve;
        a.valve_thr = valve_threshold(d->valve_eps);
        a.vpart = dvalve ? reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + w.off_vpart) : nullptr;
    } else if (!make_gate_set(d->conv_k > 0, d->amp_mode, (double)d->conv_clamp, d->gate_tau, &a.gs)) {
        return CAWN_EUNSUPPORTED;
    }
    a.H = d->H; a.F = d->F;
    a.gpb = d->F >= 32 ? 1 : 32 / d->F;
    a.G = valve_groups(d);
    if (d->ret_mode == 1) {
        a.ret = ret;
        a.rpart = dret ? reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + w.off_rpart) : nullptr;
        a.aggp = reinterpret_cast<tagged_t *>(reinterpret_cast<char *>(workspace) + w.off_aggp);
    }
    const bool vec = (J % BwdV == 0) && (ist % BwdV == 0) && (isb % BwdV == 0) && (ost % BwdV == 0) &&
                     (osb % BwdV == 0) && aligned(mag, 8) && aligned(ang, 8) && aligned(dz_re, 8) &&
                     aligned(dz_im, 8) && aligned(dmag, 8) && aligned(dang, 8) &&
                     (!state_in || aligned(state_in, 8)) && (!ckpt || aligned(ckpt, 8)) &&
                     (!dstate_out || aligned(dstate_out, 8)) && (!dstate_in || aligned(dstate_in, 8));
    const int JB = (vec ? BwdV : 1) * BwdLPR;
    const int nLB = (int)((J + JB - 1) / JB);
    const size_t tiles = (size_t)d->B * w.nT * nLB;
    if (tiles > MAX_TILES) return CAWN_EUNSUPPORTED;

    char *ws = reinterpret_cast<char *>(workspace);
    if (!d->lane_consts_cached) {
        if (build_table(d, w, ws, d->ret_mode == 1 ? nullptr : gamma, theta, conv_w, conv_b,
                        d->ret_mode == 1 ? ret_bias : nullptr, s, hconv_w, hconv_b) != hipSuccess) return CAWN_ELAUNCH;
    }
    a.hconv = hc ? 1 : 0;
    a.out_clamp = d->out_clamp;
    a.mag = mag; a.ang = ang; a.dz_re = dz_re; a.dz_im = dz_im;
    a.table = reinterpret_cast<const float *>(ws + w.off_table);
    a.state_in = reinterpret_cast<const float *>(state_in);
    a.ckpt = reinterpret_cast<const float *>(ckpt);
    a.dstate_out = reinterpret_cast<const float *>(dstate_out);
    a.dmag = dmag; a.dang = dang;
    a.dstate_in = reinterpret_cast<float *>(dstate_in);
    a.hdr = reinterpret_cast<WsHeader *>(ws);
    a.agg = reinterpret_cast<tagged_t *>(ws + w.off_agg);
    a.pre = reinterpret_cast<tagged_t *>(ws + w.off_pre);
    a.clear_from = w.off_agg;
    a.halo = reinterpret_cast<tagged_t *>(ws + w.off_halo);
    a.part = reinterpret_cast<float *>(ws + w.off_part);
    a.B = d->B; a.L = d->L; a.J = (int)J; a.Jp = w.Jp; a.nT = w.nT; a.nTc = w.nTc; a.nLB = nLB;
    a.amp_mode = d->amp_mode; a.want_param = want_param ? 1 : 0;
    a.small_angle = (kc > 0 && d->conv_clamp <= 256.0f) ? 1 : 0;
    a.stage16 = (J % 4 == 0 && ist % 4 == 0 && isb % 4 == 0 && aligned(mag, 16) && aligned(ang, 16) &&
                 (!state_in || aligned(state_in, 16))) ? 1 : 0;
    if (bf16) a.stage16 = (J % 8 == 0 && ist % 8 == 0 && isb % 8 == 0 && aligned(mag, 16) && aligned(ang, 16)) ? 1 : 0;
    const long long zq = bf16 ? 8 : 4;       // elements per 16 bytes
    a.stage16z = (J % zq == 0 && ost % zq == 0 && osb % zq == 0 && aligned(dz_re, 16) && aligned(dz_im, 16)) ? 1 : 0;
    a.isb = isb; a.ist = ist; a.osb = osb; a.ost = ost;
    a.conv_clamp = d->conv_clamp; a.grad_clamp = d->grad_clamp;
    a.spin_limit = g_spin_limit.load();
    a.total_tiles = (uint32_t)tiles;
    a.dbg = reinterpret_cast<unsigned long long *>(ws + w.off_dbg);
    if (launch_bwd(a, kc, vec, s) != hipSuccess) return CAWN_ELAUNCH;
    {
        EpilogueArgs p{};
        float *hpart = reinterpret_cast<float *>(ws + w.off_hpart);
        if (dgamma || dtheta || want_w || hc) {
            p.rows = part_rows(kc, hc);
            p.nbx = (int)((J + 31) / 32);
        }
        p.part = a.part;
        p.out0 = dgamma; p.out1 = dtheta; p.out2 = dconv_w; p.out3 = dconv_b; p.out4 = hpart;
        p.conv_k = kc > 0 ? kc : 1;
        p.hc_row0 = hc ? 4 + 2 * kc : -1;
        p.J = (int)J; p.JB = JB; p.nLB = nLB; p.chains = d->B * w.nT; p.accumulate = d->accumulate_param_grads;
        if (a.vpart) { p.lpart[p.nsets] = a.vpart; p.logit[p.nsets] = valve; p.lout[p.nsets] = dvalve; ++p.nsets; }
        if (a.rpart) { p.lpart[p.nsets] = a.rpart; p.logit[p.nsets] = nullptr; p.lout[p.nsets] = dret; ++p.nsets; }
        const long long n = (long long)d->B * d->H * d->L;
        const long long nb = (n + 1023) / 1024;
        p.nb = p.nsets ? (int)(nb < 1024 ? nb : 1024) : 0;
        p.B = d->B; p.L = d->L; p.H = d->H; p.G = a.G;
        const unsigned blocks = (unsigned)(p.nbx * p.rows + p.nb * p.nsets);
        if (blocks) {
            hipLaunchKernelGGL(bwd_epilogue_kernel, dim3(blocks), dim3(1024), 0, s, p);
            if (hipGetLastError() != hipSuccess) return CAWN_ELAUNCH;
        }
        if (hc && (dhconv_w || dhconv_b)) {
            const int nh = HC_PART_ROWS * d->H;
            hipLaunchKernelGGL(hconv_grad_reduce_kernel, dim3((unsigned)nh), dim3(64), 0, s, hpart, dhconv_w,
                               dhconv_b, d->H, d->F, (int)J, d->accumulate_param_grads);
            if (hipGetLastError() != hipSuccess) return CAWN_ELAUNCH;
        }
    }
    return CAWN_OK;
}

int cawn_phase_accumulate_bwd(const cawn_desc *d, const float *mag, const float *ang, const float *gamma,
                              const float *theta, const float *conv_w, const float *conv_b,
                              const void *state_in, const void *ckpt, const float *dz_re, const float *dz_im,
                              const void *dstate_out, float *dmag, float *dang, float *dgamma, float *dtheta,
                              float *dconv_w, float *dconv_b, void *dstate_in, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->gate_mode != 0 || d->ret_mode != 0) return CAWN_EINVAL;      // those modes have entry points of their own
    return bwd_impl(d, mag, ang, nullptr, nullptr, nullptr, gamma, theta, conv_w, conv_b, state_in, ckpt, dz_re, dz_im, dstate_out,
                    dmag, dang, nullptr, nullptr, dgamma, dtheta, dconv_w, dconv_b, dstate_in, workspace, workspace_bytes,
                    stream);
}

int cawn_phase_accumulate_valve_bwd(const cawn_desc *d, const float *mag, const float *ang, const float *valve,
                                    const float *gamma, const float *theta, const float *conv_w,
                                    const float *conv_b, const void *state_in, const void *ckpt,
                                    const float *dz_re, const float *dz_im, const void *dstate_out, float *dmag,
                                    float *dang, float *dvalve, float *dgamma, float *dtheta, float *dconv_w,
                                    float *dconv_b, void *dstate_in, void *workspace, size_t workspace_bytes,
                                    void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->gate_mode != 1 || d->ret_mode != 0) return CAWN_EINVAL;
    return bwd_impl(d, mag, ang, valve, nullptr, nullptr, gamma, theta, conv_w, conv_b, state_in, ckpt, dz_re, dz_im,
                    dstate_out, dmag, dang, dvalve, nullptr, dgamma, dtheta, dconv_w, dconv_b, dstate_in, workspace,
                    workspace_bytes, stream);
}

int cawn_phase_accumulate_bf16_fwd(const cawn_desc *d, const uint16_t *mag, const uint16_t *ang, const float *valve,
                                   const float *ret, const float *ret_bias, const float *gamma, const float *theta,
                                   const float *conv_w, const float *conv_b, const void *state_in, uint16_t *z_re,
                                   uint16_t *z_im, void *state_out, void *ckpt, uint32_t *gate_mask, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    return fwd_impl(d, reinterpret_cast<const float *>(mag), reinterpret_cast<const float *>(ang),
                    d->gate_mode == 1 ? valve : nullptr, d->ret_mode == 1 ? ret : nullptr,
                    d->ret_mode == 1 ? ret_bias : nullptr, d->ret_mode == 1 ? nullptr : gamma, theta, conv_w, conv_b,
                    state_in, reinterpret_cast<float *>(z_re), reinterpret_cast<float *>(z_im), state_out, ckpt,
                    gate_mask, workspace, workspace_bytes, stream, true);
}

int cawn_phase_accumulate_hconv_fwd(const cawn_desc *d, const void *mag, const void *ang, const float *valve,
                                    const float *ret, const float *ret_bias, const float *gamma, const float *theta,
                                    const float *conv_w, const float *conv_b, const float *hconv_w,
                                    const float *hconv_b, const void *state_in, void *zc_re, void *zc_im,
                                    void *state_out, void *ckpt, uint32_t *gate_mask, void *workspace,
                                    size_t workspace_bytes, int32_t activations_bf16, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->hconv_k != 3 || !hconv_w) return CAWN_EINVAL;
    return fwd_impl(d, reinterpret_cast<const float *>(mag), reinterpret_cast<const float *>(ang),
                    d->gate_mode == 1 ? valve : nullptr, d->ret_mode == 1 ? ret : nullptr,
                    d->ret_mode == 1 ? ret_bias : nullptr, d->ret_mode == 1 ? nullptr : gamma, theta, conv_w, conv_b,
                    state_in, reinterpret_cast<float *>(zc_re), reinterpret_cast<float *>(zc_im), state_out, ckpt,
                    gate_mask, workspace, workspace_bytes, stream, activations_bf16 != 0, hconv_w, hconv_b);
}

int cawn_phase_accumulate_hconv_bwd(const cawn_desc *d, const void *mag, const void *ang, const float *valve,
                                    const float *ret, const float *ret_bias, const float *gamma, const float *theta,
                                    const float *conv_w, const float *conv_b, const float *hconv_w, const float *hconv_b,
                                    const void *state_in, const void *ckpt, const void *dc_re, const void *dc_im,
                                    const void *dstate_out, void *dmag, void *dang, float *dvalve, float *dret,
                                    float *dgamma, float *dtheta, float *dconv_w, float *dconv_b, float *dhconv_w,
                                    float *dhconv_b, void *dstate_in, void *workspace, size_t workspace_bytes,
                                    int32_t activations_bf16, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->hconv_k != 3 || !hconv_w) return CAWN_EINVAL;
    const bool valved = d->gate_mode == 1, rmode = d->ret_mode == 1;
    return bwd_impl(d, reinterpret_cast<const float *>(mag), reinterpret_cast<const float *>(ang),
                    valved ? valve : nullptr, rmode ? ret : nullptr, rmode ? ret_bias : nullptr, rmode ? nullptr : gamma,
                    theta, conv_w, conv_b, state_in, ckpt, reinterpret_cast<const float *>(dc_re),
                    reinterpret_cast<const float *>(dc_im), dstate_out, reinterpret_cast<float *>(dmag),
                    reinterpret_cast<float *>(dang), valved ? dvalve : nullptr, rmode ? dret : nullptr, dgamma, dtheta,
                    dconv_w, dconv_b, dstate_in, workspace, workspace_bytes, stream, activations_bf16 != 0, hconv_w,
                    hconv_b, dhconv_w, dhconv_b);
}

int cawn_phase_accumulate_bf16_bwd(const cawn_desc *d, const uint16_t *mag, const uint16_t *ang, const float *valve,
                                   const float *ret, const float *ret_bias, const float *gamma, const float *theta,
                                   const float *conv_w, const float *conv_b, const void *state_in, const void *ckpt,
                                   const uint16_t *dz_re, const uint16_t *dz_im, const void *dstate_out, uint16_t *dmag,
                                   uint16_t *dang, float *dvalve, float *dret, float *dgamma, float *dtheta,
                                   float *dconv_w, float *dconv_b, void *dstate_in, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    const bool valved = d->gate_mode == 1, rmode = d->ret_mode == 1;
    return bwd_impl(d, reinterpret_cast<const float *>(mag), reinterpret_cast<const float *>(ang),
                    valved ? valve : nullptr, rmode ? ret : nullptr, rmode ? ret_bias : nullptr,
                    rmode ? nullptr : gamma, theta, conv_w, conv_b, state_in, ckpt,
                    reinterpret_cast<const float *>(dz_re), reinterpret_cast<const float *>(dz_im), dstate_out,
                    reinterpret_cast<float *>(dmag), reinterpret_cast<float *>(dang), valved ? dvalve : nullptr,
                    rmode ? dret : nullptr, rmode ? nullptr : dgamma, dtheta, dconv_w, dconv_b, dstate_in, workspace,
                    workspace_bytes, stream, true);
}

int cawn_phase_accumulate_ret_bwd(const cawn_desc *d, const float *mag, const float *ang, const float *valve,
                                  const float *ret, const float *ret_bias, const float *theta,
                                  const float *conv_w, const float *conv_b, const void *state_in, const void *ckpt,
                                  const float *dz_re, const float *dz_im, const void *dstate_out, float *dmag,
                                  float *dang, float *dvalve, float *dret, float *dtheta, float *dconv_w,
                                  float *dconv_b, void *dstate_in, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->ret_mode != 1) return CAWN_EINVAL;
    const bool valved = d->gate_mode == 1;
    return bwd_impl(d, mag, ang, valved ? valve : nullptr, ret, ret_bias, nullptr, theta, conv_w, conv_b, state_in,
                    ckpt, dz_re, dz_im, dstate_out, dmag, dang, valved ? dvalve : nullptr, dret, nullptr, dtheta,
                    dconv_w, dconv_b, dstate_in, workspace, workspace_bytes, stream);
}

int cawn_stream_copy(const float *in0, const float *in1, float *out0, float *out1, size_t n, void *stream)
{
    if (!in0 || !in1 || !out0 || !out1) return CAWN_EINVAL;
    if (n % 4 || !aligned(in0, 16) || !aligned(in1, 16) || !aligned(out0, 16) || !aligned(out1, 16)) return CAWN_EUNSUPPORTED;
    if (n == 0) return CAWN_OK;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CAWN_ELAUNCH;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    }
    const size_t n4 = n / 4;
    size_t blocks = (n4 + 255) / 256;
    const size_t resident = (size_t)cus * 2;       // two workgroups of 4 waves per CU
    if (blocks > resident) blocks = resident;
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<const v4f *>(in0), reinterpret_cast<const v4f *>(in1),
                       reinterpret_cast<v4f *>(out0), reinterpret_cast<v4f *>(out1), n4);
    return hipGetLastError() == hipSuccess ? CAWN_OK : CAWN_ELAUNCH;
}

// ---------------------------------------------------------------------- allocation-free forward
// The workspace of this entry point is a static device array instead of caller memory.  `scratch`
// names the array for device code only: on the host it is a stand-in, never an address.  The device
// address is asked for once per device (hipGetSymbolAddress, with that device current) and kept;
// every launch and fill below takes that pointer.
#ifndef CAWN_STATIC_WS_BYTES
#define CAWN_STATIC_WS_BYTES (8u << 20)
#endif
static __device__ __align__(256) unsigned char scratch[CAWN_STATIC_WS_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];      // per device: the array's address there, once known
}

int cawn_phase_accumulate_fwd_static(const cawn_desc *d, const float *mag, const float *ang, const float *gamma,
                                     const float *theta, const float *conv_w, const float *conv_b,
                                     const void *state_in, float *z_re, float *z_im, void *state_out, void *ckpt,
                                     uint32_t *gate_mask, void *stream)
{
    if (!desc_ok(d)) return CAWN_EINVAL;
    if (d->gate_mode != 0 || d->ret_mode != 0 || d->hconv_k != 0) return CAWN_EINVAL;
    // sizes beyond the static array are refused before anything touches the device
    if (make_layout(d, true).total > (size_t)CAWN_STATIC_WS_BYTES) return CAWN_EWORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return CAWN_ELAUNCH;
    void *ws = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ws) {
        // first call on this device.  The array is zero when the module is loaded (no word carries a
        // tag); only the header's size field, read when the epoch wraps, has to be written.  Two
        // threads racing here find the same address and enqueue the same idempotent store.
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CAWN_ELAUNCH;
        hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream,
                           reinterpret_cast<WsHeader *>(p), (unsigned long long)CAWN_STATIC_WS_BYTES);
        if (hipGetLastError() != hipSuccess) return CAWN_ELAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
        ws = p;
    }
    return fwd_impl(d, mag, ang, nullptr, nullptr, nullptr, gamma, theta, conv_w, conv_b, state_in, z_re, z_im,
                    state_out, ckpt, gate_mask, ws, (size_t)CAWN_STATIC_WS_BYTES, stream, false, nullptr, nullptr, true);
}

}  // extern "C"
