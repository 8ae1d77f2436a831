// Fused forward: Temporal Syntax Cache conv -> clamp -> SiLU -> gate -> phasor -> causal phase
// accumulation -> clamp, single pass over HBM (Sec. 3.2 - 3.5 of the paper).
//
// Parallel structure.  The recurrence S[t] = p[t] + lambda S[t-1] has a per-lane constant
// multiplier, so a run of n tokens acts on an incoming state as  S_out = E + lambda^n S_in,
// with E the run's result from a zero state.  Three levels use that:
//   thread    : V adjacent lanes x NSTEP consecutive tokens, serial, phasors kept in registers;
//   workgroup : NSEG such segments = one tile of TILE_T tokens; segment results meet in LDS;
//   grid      : tiles of one (batch row, lane block) form a chain in time.  A tile publishes its
//               aggregate E, then walks back over earlier tiles' aggregates until it meets one
//               that already knows its inclusive prefix (decoupled look-back), and publishes
//               its own.  Tiles take their position from an atomic ticket, so a tile only ever
//               waits for tiles that are already running.
// After the carry is known each thread replays its NSTEP tokens from the true incoming state,
// clamps and stores.  Per token-lane HBM traffic: 8 bytes in, 8 bytes out.
#include "cawn_internal.hpp"

namespace cawn {

// Tuning aid, compiled only with -DCAWN_TIMING: per-tile time stamps (100 MHz counter) of the
// chain-owning thread, written behind the parameter partials in the workspace.
#ifdef CAWN_TIMING
#define CAWN_STAMP(k) do { if (tid == (NSEG - 1) * LPR) a.dbg[(size_t)ticket * 16 + (k)] = wall_clock64(); } while (0)
#else
#define CAWN_STAMP(k) do { } while (0)
#endif

template <int V> struct Vec;
template <> struct Vec<1> {
    static __device__ __forceinline__ void ld(float (&d)[1], const float *p) { d[0] = *p; }
    static __device__ __forceinline__ void st(float *p, const float (&s)[1]) { *p = s[0]; }
};
template <> struct Vec<2> {
    static __device__ __forceinline__ void ld(float (&d)[2], const float *p)
    {
        float2 t = *reinterpret_cast<const float2 *>(p);
        d[0] = t.x; d[1] = t.y;
    }
    static __device__ __forceinline__ void st(float *p, const float (&s)[2])
    {
        *reinterpret_cast<float2 *>(p) = make_float2(s[0], s[1]);
    }
};
template <> struct Vec<4> {
    static __device__ __forceinline__ void ld(float (&d)[4], const float *p)
    {
        float4 t = *reinterpret_cast<const float4 *>(p);
        d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
    }
    static __device__ __forceinline__ void st(float *p, const float (&s)[4])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(s[0], s[1], s[2], s[3]);
    }
};

template <int V, int KC>
__global__ __launch_bounds__(Geom::NSEG *FwdLPR, CAWN_FWD_WAVES) void fwd_kernel(const FwdArgs a)
{
    constexpr int NSTEP = Geom::NSTEP, NSEG = Geom::NSEG, LPR = FwdLPR;
    constexpr int JB = V * LPR;
    constexpr int HALO = KC > 0 ? KC - 1 : 0;
    constexpr int NR = NSTEP + HALO;

    __shared__ float sE[NSEG][2][JB];
    __shared__ float sCarry[2][JB];
    __shared__ uint32_t sTicket, sLast;

    const int tid = threadIdx.x;
    const int lv = tid % LPR, seg = tid / LPR;
    if (tid == 0) {
        sTicket = __hip_atomic_fetch_add(&a.hdr->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sLast = 0;
    }
    __syncthreads();
    const uint32_t ticket = sTicket;
    CAWN_STAMP(0);
    const int lb = ticket % a.nLB;
    const int rest = ticket / a.nLB;
    const int b = rest % a.B, tt = rest / a.B;
    const uint32_t chain_stride = (uint32_t)a.B * a.nLB;
    const int j0 = lb * JB + lv * V;
    const bool active = j0 < a.J;
    const int t0 = tt * TILE_T + seg * NSTEP;
    const int HALO_ROWS = HALO;
    const float *tail_in = a.state_in ? a.state_in + (size_t)a.B * 2 * a.J : nullptr;

    // ---- lane constants
    float lr[V], li[V], pfr[V], pfi[V], psr[V], psi[V];
    float wm[KC > 0 ? KC : 1][V], wa[KC > 0 ? KC : 1][V], bm[V], ba[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { lr[v] = li[v] = pfr[v] = pfi[v] = 0.f; psr[v] = 1.f; psi[v] = 0.f; bm[v] = ba[v] = 0.f; }
    if (active) {
        const float *tb = a.table + j0;
        Vec<V>::ld(lr, tb + (size_t)R_LR * a.Jp);
        Vec<V>::ld(li, tb + (size_t)R_LI * a.Jp);
        Vec<V>::ld(pfr, tb + (size_t)(R_PSEG + 2) * a.Jp);       // lambda^NSTEP
        Vec<V>::ld(pfi, tb + (size_t)(R_PSEG + 3) * a.Jp);
        Vec<V>::ld(psr, tb + (size_t)(R_PSEG + 2 * seg) * a.Jp); // lambda^(NSTEP*seg)
        Vec<V>::ld(psi, tb + (size_t)(R_PSEG + 2 * seg + 1) * a.Jp);
        if (KC > 0) {
            Vec<V>::ld(bm, tb + (size_t)R_BIAS_M * a.Jp);
            Vec<V>::ld(ba, tb + (size_t)R_BIAS_A * a.Jp);
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                Vec<V>::ld(wm[k], tb + (size_t)(R_W0 + k) * a.Jp);
                Vec<V>::ld(wa[k], tb + (size_t)(R_W0 + KC + k) * a.Jp);
            }
        }
    }

    // ---- input rows: time t0-HALO+r, r = 0..NR-1
    float um[NR][V], ua[NR][V];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int t = t0 - HALO_ROWS + r;
#pragma unroll
        for (int v = 0; v < V; ++v) um[r][v] = ua[r][v] = 0.f;
        if (active) {
            if (t >= 0 && t < a.L) {
                const size_t off = (size_t)b * a.isb + (size_t)t * a.ist + j0;
                Vec<V>::ld(um[r], a.mag + off);
                Vec<V>::ld(ua[r], a.ang + off);
            } else if (HALO > 0 && t < 0 && tail_in) {
                const int q = t + HALO_ROWS;
                if (q >= 0) {
                    const size_t off = ((size_t)(b * HALO_ROWS + q) * 2) * a.J + j0;
                    Vec<V>::ld(um[r], tail_in + off);
                    Vec<V>::ld(ua[r], tail_in + off + a.J);
                }
            }
        }
    }

#ifdef CAWN_TIMING
    wait_stores_done();
#endif
    CAWN_STAMP(1);
    // ---- front-end, phasors, local scan from zero
    float pr[NSTEP][V], pi[NSTEP][V];
    float Er[V], Ei[V];
    uint32_t gbits[NSTEP];
#pragma unroll
    for (int v = 0; v < V; ++v) Er[v] = Ei[v] = 0.f;
#pragma unroll
    for (int i = 0; i < NSTEP; ++i) {
        gbits[i] = 0;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float zm, xm, phi;
            if (KC > 0) {
                zm = bm[v];
                float za = ba[v];
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    zm = __builtin_fmaf(wm[k][v], um[i + k][v], zm);
                    za = __builtin_fmaf(wa[k][v], ua[i + k][v], za);
                }
                const float cm = clampf(zm, a.conv_clamp), ca = clampf(za, a.conv_clamp);
                xm = cm * sigmoid_fast(cm);
                phi = ca * sigmoid_fast(ca);
            } else {
                zm = um[i][v];
                xm = zm;
                phi = ua[i][v];
            }
            const float amp = a.amp_mode ? __builtin_fminf(softplus_fast(xm), 10.0f) : xm;
            const bool g = in_gate(a.gs, zm);
            float s, c;
            sincos_fast(phi, s, c);
            const float ag = g ? amp : 0.0f;
            pr[i][v] = ag * c;
            pi[i][v] = ag * s;
            gbits[i] |= (g && active ? 1u : 0u) << v;
            const float nr = __builtin_fmaf(lr[v], Er[v], __builtin_fmaf(-li[v], Ei[v], pr[i][v]));
            const float ni = __builtin_fmaf(li[v], Er[v], __builtin_fmaf(lr[v], Ei[v], pi[i][v]));
            Er[v] = nr;
            Ei[v] = ni;
        }
    }

    // ---- optional gate mask: bit j%32 of word j/32
    if (a.mask) {
        constexpr int TPW = 32 / V;                 // threads per 32-lane word
        const int W = (a.J + 31) >> 5;
#pragma unroll
        for (int i = 0; i < NSTEP; ++i) {
            uint32_t m = gbits[i] << (V * (lv % TPW));
#pragma unroll
            for (int o = 1; o < TPW; o <<= 1) m |= (uint32_t)__shfl_xor((int)m, o, 64);
            const int t = t0 + i;
            if ((lv % TPW) == 0 && active && t < a.L)
                a.mask[((size_t)b * a.L + t) * W + (j0 >> 5)] = m;
        }
    }

    // ---- segments meet in LDS
    CAWN_STAMP(2);
#pragma unroll
    for (int v = 0; v < V; ++v) {
        sE[seg][0][lv * V + v] = Er[v];
        sE[seg][1][lv * V + v] = Ei[v];
    }
    __syncthreads();
    CAWN_STAMP(3);
    float Xr[V], Xi[V];   // state entering my segment, from a zero tile input
#pragma unroll
    for (int v = 0; v < V; ++v) Xr[v] = Xi[v] = 0.f;
    for (int q = 0; q < seg; ++q) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float er = sE[q][0][lv * V + v], ei = sE[q][1][lv * V + v];
            const float nr = __builtin_fmaf(pfr[v], Xr[v], __builtin_fmaf(-pfi[v], Xi[v], er));
            const float ni = __builtin_fmaf(pfi[v], Xr[v], __builtin_fmaf(pfr[v], Xi[v], ei));
            Xr[v] = nr;
            Xi[v] = ni;
        }
    }
    // ---- chain.  The threads of the last segment own the tile aggregate: they publish it, do the
    //      look-back and publish the prefix, all within their own wave (stores are waited for with
    //      that wave's vmcnt, so no workgroup barrier sits on the publication path).
    const bool is_tail_seg = seg == NSEG - 1;
    float Tr[V], Ti[V], hr[V], hi[V], qr[V], qi[V];
    const size_t slot = (size_t)ticket * 2 * JB + lv * V;
    if (is_tail_seg) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            Tr[v] = __builtin_fmaf(pfr[v], Xr[v], __builtin_fmaf(-pfi[v], Xi[v], Er[v]));
            Ti[v] = __builtin_fmaf(pfi[v], Xr[v], __builtin_fmaf(pfr[v], Xi[v], Ei[v]));
            hr[v] = hi[v] = qr[v] = qi[v] = 0.f;
        }
        if (active) {   // lambda^TILE_T as a double-float
            const float *tb = a.table + j0;
            Vec<V>::ld(hr, tb + (size_t)R_PT_HR * a.Jp);
            Vec<V>::ld(hi, tb + (size_t)R_PT_HI * a.Jp);
            Vec<V>::ld(qr, tb + (size_t)R_PT_LR * a.Jp);
            Vec<V>::ld(qi, tb + (size_t)R_PT_LI * a.Jp);
        }
        float cr[V], ci[V];
#pragma unroll
        for (int v = 0; v < V; ++v) cr[v] = ci[v] = 0.f;
        if (tt == 0) {
            if (a.state_in && active) {
                Vec<V>::ld(cr, a.state_in + ((size_t)b * 2 + 0) * a.J + j0);
                Vec<V>::ld(ci, a.state_in + ((size_t)b * 2 + 1) * a.J + j0);
            }
        } else {
            if (tt + 1 < a.nT) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    coherent_store(a.agg + slot + v, Tr[v]);
                    coherent_store(a.agg + slot + JB + v, Ti[v]);
                }
                wait_stores_done();
                if (lv == 0) flag_store(a.flags + ticket, ST_AGG);
            }
            CAWN_STAMP(4);
            if (!look_back<V, false, LPR>(a.flags, a.agg, a.pre, ticket - chain_stride, chain_stride, tt, JB, lv * V,
                                          lv, hr, hi, qr, qi, a.spin_limit, cr, ci)) {
                // gave up: flag the workspace, keep going so that every wave exits
                if (lv == 0) __hip_atomic_store(&a.hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        CAWN_STAMP(5);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            sCarry[0][lv * V + v] = cr[v];
            sCarry[1][lv * V + v] = ci[v];
        }
        if (a.ckpt && active) {
            float *ck = a.ckpt + (((size_t)b * a.nT + tt) * 2) * a.J + j0;
            Vec<V>::st(ck, cr);
            Vec<V>::st(ck + a.J, ci);
        }
    }
    __syncthreads();

    CAWN_STAMP(6);
    // ---- true state entering my segment; the tile's inclusive prefix for the chain
    float Sr[V], Si[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float cr = sCarry[0][lv * V + v], ci = sCarry[1][lv * V + v];
        Sr[v] = __builtin_fmaf(psr[v], cr, __builtin_fmaf(-psi[v], ci, Xr[v]));
        Si[v] = __builtin_fmaf(psi[v], cr, __builtin_fmaf(psr[v], ci, Xi[v]));
    }
    if (is_tail_seg) {
        if (tt + 1 < a.nT) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float cr = sCarry[0][lv * V + v], ci = sCarry[1][lv * V + v];
                float P_r, P_i;
                chain_step<false>(Tr[v], Ti[v], hr[v], hi[v], qr[v], qi[v], cr, ci, P_r, P_i);
                coherent_store(a.pre + slot + v, P_r);
                coherent_store(a.pre + slot + JB + v, P_i);
            }
            wait_stores_done();
            if (lv == 0) flag_store(a.flags + ticket, ST_PREFIX);
        }
        if (lv == 0) {
            wait_stores_done();
            const uint32_t old = __hip_atomic_fetch_add(&a.hdr->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old + 1 == a.total_tiles) sLast = 1;
        }
    }
    CAWN_STAMP(7);

    // ---- replay from the true state, clamp, store
#pragma unroll
    for (int i = 0; i < NSTEP; ++i) {
        const int t = t0 + i;
        float zr[V], zi[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float nr = __builtin_fmaf(lr[v], Sr[v], __builtin_fmaf(-li[v], Si[v], pr[i][v]));
            const float ni = __builtin_fmaf(li[v], Sr[v], __builtin_fmaf(lr[v], Si[v], pi[i][v]));
            Sr[v] = nr;
            Si[v] = ni;
            zr[v] = clampf(nr, a.out_clamp);
            zi[v] = clampf(ni, a.out_clamp);
        }
        if (active && t < a.L) {
            const size_t off = (size_t)b * a.osb + (size_t)t * a.ost + j0;
            Vec<V>::st(a.z_re + off, zr);
            Vec<V>::st(a.z_im + off, zi);
            if (t == a.L - 1 && a.state_out) {
                Vec<V>::st(a.state_out + ((size_t)b * 2 + 0) * a.J + j0, Sr);
                Vec<V>::st(a.state_out + ((size_t)b * 2 + 1) * a.J + j0, Si);
            }
        }
    }

    CAWN_STAMP(8);
    // ---- conv history for the next call: last HALO pre-conv rows (written by the last tile,
    //      after its carry arrived, i.e. after the first tile has consumed state_in: safe in place)
    if (HALO > 0 && a.state_out && tt == a.nT - 1 && seg == 0 && active) {
        float *tail_out = a.state_out + (size_t)a.B * 2 * a.J;
        for (int q = 0; q < HALO_ROWS; ++q) {
            const int t = a.L - HALO_ROWS + q;
            float vm[V], va[V];
#pragma unroll
            for (int v = 0; v < V; ++v) vm[v] = va[v] = 0.f;
            if (t >= 0) {
                const size_t off = (size_t)b * a.isb + (size_t)t * a.ist + j0;
                Vec<V>::ld(vm, a.mag + off);
                Vec<V>::ld(va, a.ang + off);
            } else if (tail_in) {
                const size_t off = ((size_t)(b * HALO_ROWS + (t + HALO_ROWS)) * 2) * a.J + j0;
                Vec<V>::ld(vm, tail_in + off);
                Vec<V>::ld(va, tail_in + off + a.J);
            }
            const size_t o = ((size_t)(b * HALO_ROWS + q) * 2) * a.J + j0;
            Vec<V>::st(tail_out + o, vm);
            Vec<V>::st(tail_out + o + a.J, va);
        }
    }

    // ---- the tile that finishes last leaves the control words zeroed for the next call
    __syncthreads();
    if (sLast) {
        for (uint32_t i = tid; i < a.total_tiles; i += blockDim.x) flag_store(a.flags + i, ST_NONE);
        if (tid == 0) {
            flag_store(&a.hdr->ticket, 0u);
            flag_store(&a.hdr->done, 0u);
        }
    }
}

template <int V>
static hipError_t launch_fwd_v(const FwdArgs &a, int conv_k, hipStream_t s)
{
    dim3 grid(a.total_tiles), block(Geom::NSEG * FwdLPR);
    switch (conv_k) {
    case 0: hipLaunchKernelGGL((fwd_kernel<V, 0>), grid, block, 0, s, a); break;
    case 1: hipLaunchKernelGGL((fwd_kernel<V, 1>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((fwd_kernel<V, 2>), grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL((fwd_kernel<V, 3>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((fwd_kernel<V, 4>), grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    return vec ? launch_fwd_v<FwdV>(a, conv_k, s) : launch_fwd_v<1>(a, conv_k, s);
}

}  // namespace cawn
