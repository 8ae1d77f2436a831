// Fused forward: Temporal Syntax Cache conv -> clamp -> SiLU -> gate -> phasor -> causal phase
// accumulation -> clamp, single pass over HBM (Sec. 3.2 - 3.5 of the paper).
//
// Parallel structure.  The recurrence S[t] = p[t] + lambda S[t-1] has a per-lane constant
// multiplier, so a run of n tokens acts on an incoming state as  S_out = E + lambda^n S_in,
// with E the run's result from a zero state.  Three levels use that:
//   thread    : V adjacent lanes x NSTEP consecutive tokens, serial, phasors kept in registers;
//   workgroup : NSEG such segments = one tile of TILE_T tokens; segment results meet in LDS;
//   grid      : tiles of one (batch row, lane block) form a chain in time.  A tile publishes its
//               aggregate E, then looks back over earlier tiles' aggregates until it meets one that
//               already knows its inclusive prefix (decoupled look-back), and publishes its own.
// After the carry is known each thread replays its NSTEP tokens from the true incoming state,
// clamps and stores.  Per token-lane HBM traffic: 8 bytes in, 8 bytes out.
//
// Scheduling.  The kernel is persistent: about as many workgroups as fit on the chip are launched
// and each loops over tiles, handed out by one atomic ticket in the order (time tile, batch row,
// lane block).  Tickets go out in time order, so a tile only ever waits for tiles that a running
// workgroup already holds; all chains advance together, so tiles that happen to be slow (some
// address classes of the 128-byte lane-block rows are, by a quarter) are spread over every
// workgroup instead of leaving a few chains to finish alone; and the lane blocks of one row are
// in flight together, which keeps DRAM pages busy.  The ticket, the input rows and the lane
// constants of the NEXT tile are fetched while the current tile is in its communication phase,
// whose memory round trips would otherwise leave the SIMDs idle.
#pragma once
#include <type_traits>

#include "cawn_internal.hpp"

namespace cawn {

#ifndef CAWN_FWD_NB
#define CAWN_FWD_NB 2       // predecessors read per look-back round trip
#endif

// Tuning aid, compiled only with -DCAWN_TIMING: per-tile time stamps (100 MHz counter) of the
// chain-owning thread, written behind the parameter partials in the workspace.
#ifdef CAWN_TIMING
#define CAWN_STAMP(k) do { if (tid == (NSEG - 1) * LPR) a.dbg[(size_t)id * 16 + (k)] = wall_clock64(); } while (0)
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

// Position of a ticket in the problem: tickets count (time tile, batch row, lane block), lane block fastest.
struct TileId {
    int lb, b, tt;
    uint32_t id;     // unique tile index (workspace slot); the chain predecessor is id - B
};
__device__ __forceinline__ TileId decode_tile(uint32_t ticket, int nLB, int B, int nT)
{
    const uint32_t per_tt = (uint32_t)B * nLB;
    const uint32_t tt = ticket / per_tt, r = ticket - tt * per_tt;
    TileId t;
    t.tt = (int)tt;
    t.b = (int)(r / nLB);
    t.lb = (int)(r - (uint32_t)t.b * nLB);
    t.id = ((uint32_t)t.lb * nT + t.tt) * B + t.b;
    return t;
}

// Stage the lane constants a forward tile keeps in registers (table rows R_LR .. R_LR + NCR - 1 of
// lane block lb) in LDS, 16 bytes per lane per load: 8 lanes cover a 32-lane row, a wave 8 rows.
// Called by one wave.  Table rows are 256-byte aligned and padded, so every address is valid.
template <int NCR, int JB>
__device__ __forceinline__ void stage_consts(float *sC, const float *table, int Jp, int lb, int lane)
{
    static_assert(JB == 32, "8 lanes x 16 bytes per row");
    const int r_in = lane >> 3, c_in = (lane & 7) * 4;
    const float *src = table + ((size_t)(R_LR + r_in) * Jp + (size_t)lb * JB + c_in);
#pragma unroll
    for (int i = 0; i < (NCR + 7) / 8; ++i) {
        if (i * 8 + r_in < NCR) {
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_global_load_lds(src + (size_t)(i * 8) * Jp, sC + (size_t)(i * 8) * JB, 16, 0, 0);
#else
            (void)src;
            (void)sC;
#endif
        }
    }
}

// VALVE: gate_mode 1, the per-head input valve of Sec. 3.3 in place of the per-lane threshold.
// RET: ret_mode 1, the retention of Sec. 3.3 item 4: gamma[t] = sigmoid(logit[t][head] + b_k) scales
// what arrives from token t-1 (accumulation equations of Sec. 3.4, printed with gamma_{t,j}).  A run of
// tokens then acts on an incoming state as S_out = E + (product of the run's gammas) e^{i n theta} S_in:
// the lane table holds pure rotations and every level carries the real product beside its aggregate.
// BF: activations (mag, ang in; z_re, z_im out) are bfloat16 in memory; arithmetic, state and
// checkpoints stay fp32 (Sec. 3.5 / Sec. 6.1 of the paper: the network runs in bf16, the accumulator in
// fp32).  A staged row of JB bf16 lanes is handled as JB/2 four-byte words; outputs are rounded to
// nearest even by the hardware conversion.
// (with bf16 rows the staged tile is half as large and a third workgroup fits a CU's LDS; the variants
// without the per-token retentions also fit its registers)
// HC: the depth-wise harmonic convolution of Sec. 3.6 applied to the clamped output before it is
// stored: channel = (plane, head), three taps along the harmonics of the head, zeros beyond its ends.
// Neighbouring harmonics are neighbouring lanes of a row.  A head wider than a lane block (F = 32 G,
// G > 1) is handled by one workgroup drawing the G tickets of the head's blocks together and taking
// them in order (every other group from the top block down): the lane of a block that borders the
// next block to come leaves its value and its unfinished output in LDS, and the bordering lane of
// that next block completes the output and stores it next to its own.
template <int V, int KC, bool VALVE, bool RET, bool BF, bool HC>
__global__ __launch_bounds__(FwdGeom::NSEG *FwdLPR, (BF && !RET && !HC) ? CAWN_FWD_WAVES + 1 : CAWN_FWD_WAVES) void fwd_kernel(const FwdArgs a)
{
    static_assert(!BF || V == 1, "bf16 activations: one lane per thread");
    static_assert(!HC || V == 1, "harmonic convolution: one lane per thread");
    constexpr int TILE_T = FwdGeom::TILE_T, NSTEP = FwdGeom::NSTEP, NSEG = FwdGeom::NSEG, LPR = FwdLPR;
    constexpr int JB = V * LPR;
    constexpr int HALO = KC > 0 ? KC - 1 : 0;
    constexpr int KC1 = KC > 0 ? KC : 1;
    constexpr int NT = NSEG * LPR;                 // threads
    constexpr int NW = NT / 64;                    // waves
    constexpr int JBS = BF ? JB / 2 : JB;          // four-byte words per staged row
    constexpr int NRTP = staged_rows<TILE_T, JBS, HALO>();   // staged rows per stream: time tile_t0-HALO+rr
    static_assert(JB <= 256 && 256 % JB == 0, "a staged row must fit a wave");
    static_assert(NW >= 2, "one wave owns the chain, the others stage the next tile");

    __shared__ __attribute__((aligned(16))) float sU[2 * NRTP][JBS];  // [stream*NRTP + rr][lane]
    // element (row, lane) of the staged rows as fp32
    auto su = [&](int r, int l) -> float {
        if constexpr (BF) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(&sU[r][0])[l] << 16);
        else return sU[r][l];
    };
    __shared__ float sE[NSEG][2][JB];
    __shared__ float sCarry[2][JB];
    constexpr int NCR = R_W0 - R_LR + 2 * KC + (HC ? HC_ROWS : 0);     // staged lane-constant rows
    // (only rows below NCR are ever staged; HC needs the room of the padding)
    __shared__ __attribute__((aligned(16))) float sC[HC ? NCR : (NCR + 7) / 8 * 8][JB];
    // valve / retention groups per lane block: F >= 8, or F >= 16 with both (LDS: two workgroups per CU)
    // (HC: one group, F >= 32 -- the two rows of unfinished outputs take the room)
    constexpr int GPB_MAX = HC ? 1 : ((VALVE && RET) ? 2 : 4);
    __shared__ float sV[VALVE ? FwdGeom::TILE_T * GPB_MAX : 1];
    __shared__ float sR[RET ? FwdGeom::TILE_T * GPB_MAX : 1];     // retention logits, laid out like sV
    __shared__ float sP[RET ? NSEG : 1][JB];                      // product of each segment's retentions
    // HC: value and unfinished output of the block's last lane, per token and plane, for the next block
    __shared__ float sHZ[2][HC ? FwdGeom::TILE_T : 1], sHP[2][HC ? FwdGeom::TILE_T : 1];
    __shared__ uint32_t sTicket[2], sLast, sEpoch;

    const int tid = threadIdx.x;
    const int lv = tid % LPR, seg = tid / LPR;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // (wave index: scalar)
    const uint32_t qtiles = (uint32_t)a.nLB * a.B * a.nT;     // all tiles of the call
    const bool is_tail_seg = seg == NSEG - 1;
    const bool owner_wave = wave == NW - 1;        // the wave holding the last segment owns the chain
    const float *tail_in = a.state_in ? a.state_in + (size_t)a.B * 2 * a.J : nullptr;

    if (tid == 0) {
        const uint32_t e = flag_load(&a.hdr->epoch);     // both round trips at once
        const uint32_t t = __hip_atomic_fetch_add(&a.hdr->ticket[0], HC ? (uint32_t)a.hcG : 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sEpoch = e;
        sTicket[0] = t;
        sLast = 0;
    }
    __syncthreads();
    uint32_t ticket = (uint32_t)__builtin_amdgcn_readfirstlane((int)sTicket[0]);   // wave-uniform: index math stays scalar
    const uint32_t epoch = (uint32_t)__builtin_amdgcn_readfirstlane((int)sEpoch);
    const uint32_t tag = make_tag(epoch);      // of every word this call publishes

    // From here on the kernel's arguments are read from the kernel-argument segment again in every
    // phase of a tile (scalar loads next to their use; `ARGS_AGAIN()` makes the compiler forget what it
    // loaded) instead of living in scalar registers across the loop: kept there, they and what the
    // compiler derives from them overflow the scalar register file, and every overflowing value costs
    // vector registers and lane moves.
    typedef const __attribute__((address_space(4))) FwdArgs *KArgs;
    KArgs ap = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
#define a (*ap)
#define ARGS_AGAIN() asm volatile("" : "+s"(ap))
    // Stage a tile's input rows in LDS.  The chain-owning wave stays out of it: a wave's memory
    // operations complete in order, and its polls of other tiles must not queue behind a tile's
    // worth of HBM reads.
    const int ist32 = (int)a.ist;
    auto stage_tile = [&](const TileId &T) {
        if (owner_wave) return;
        if (wave == 0) stage_consts<NCR, JB>(&sC[0][0], a.table, a.Jp, T.lb, lane);
        if (VALVE && wave == 0) stage_valve<TILE_T, JB>(&sV[0], a.valve, T.b, T.tt * TILE_T, T.lb, a.L, a.H, a.F, a.gpb, lane);
        if (RET && wave == 0) stage_valve<TILE_T, JB>(&sR[0], a.ret, T.b, T.tt * TILE_T, T.lb, a.L, a.H, a.F, a.gpb, lane);
        // (bf16: rows of J/2 words at half the strides; the fp32 conv history is read at its point of use)
        if (a.stage16)
            stage_rows<TILE_T, JBS, HALO, 16>(&sU[0][0], a.mag, a.ang, BF ? nullptr : tail_in, T.b, T.tt * TILE_T, T.lb,
                                      BF ? a.J / 2 : a.J, a.L, BF ? a.isb / 2 : a.isb, BF ? ist32 / 2 : ist32, wave, NW - 1, lane);
        else
            stage_rows<TILE_T, JBS, HALO, 4>(&sU[0][0], a.mag, a.ang, BF ? nullptr : tail_in, T.b, T.tt * TILE_T, T.lb,
                                     BF ? a.J / 2 : a.J, a.L, BF ? a.isb / 2 : a.isb, BF ? ist32 / 2 : ist32, wave, NW - 1, lane);
    };

    // HC, heads of G > 1 lane blocks: a group of G tickets is one head's blocks; groups with an odd index
    // take them from the last block down, so that at any time the workgroups of the grid are spread over
    // all positions in a head (in step on one position they would all read and write one 128-byte
    // address class of the rows at a time, i.e. a part of the memory channels)
    auto tile_of = [&](uint32_t tk) {
        if (HC) {
            const uint32_t G = (uint32_t)a.hcG, g = tk / G, p_ = tk - g * G;
            tk = g * G + ((g & 1u) ? G - 1u - p_ : p_);
        }
        return decode_tile(tk, a.nLB, a.B, a.nT);
    };
    TileId T{};
    if (ticket < qtiles) {
        T = tile_of(ticket);
        stage_tile(T);
    }

    wait_vm<0>();     // the first tile's staged rows

    float lr[V], li[V], pfr[V], pfi[V], psr[V], psi[V];
    float wm[KC1][V], wa[KC1][V], bm[V], ba[V];
    float rb[V];                                   // RET: static retention bias of my lanes
    float hw[2][3], hb[2];                         // HC: taps and bias of my lane's two channels

    for (int it = 0; ticket < qtiles; ++it) {
        ARGS_AGAIN();
        const GateSet gs_ = {a.gs.a1, a.gs.b1, a.gs.a2, a.gs.b2};
        const uint32_t id = T.id;
        const int b = T.b, tt = T.tt;
        const int j0 = T.lb * JB + lv * V;
        const bool active = j0 < a.J;
        const int t0 = tt * TILE_T + seg * NSTEP;

        // ticket of the next tile: asked for now, parked in LDS after the front-end (the round trip
        // of the atomic stays off the path to the barrier below)
        uint32_t ticket_ahead;   // (only thread 0's copy is ever set or read; no initialiser, so no
                             // merge of values that would wait for the atomic right here)
        // (HC: the tickets of a head's lane blocks are drawn together, a multiple of hcG first)
        const uint32_t hcG = HC ? (uint32_t)a.hcG : 1u;
        if (tid == 0) {
            if (HC && (ticket + 1) % hcG != 0)
                ticket_ahead = ticket + 1;
            else
                ticket_ahead = __hip_atomic_fetch_add(&a.hdr->ticket[0], hcG, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // ---- the staged rows have landed (each wave waited for its own loads: before the loop, or
        //      at the end of the previous iteration)
        lds_barrier();
        CAWN_STAMP(0);

        // ---- lane constants of this tile's lane block, staged with its rows
        {
            auto cst = [&](float(&d)[V], int r) {
#pragma unroll
                for (int v = 0; v < V; ++v) d[v] = sC[r - R_LR][lv * V + v];
            };
            cst(lr, R_LR);
            cst(li, R_LI);
            cst(pfr, R_PSEG + 2);                 // lambda^NSTEP
            cst(pfi, R_PSEG + 3);
            cst(psr, R_PSEG + 2 * seg);           // lambda^(NSTEP*seg)
            cst(psi, R_PSEG + 2 * seg + 1);
#pragma unroll
            for (int v = 0; v < V; ++v) {
                bm[v] = ba[v] = 0.f;
#pragma unroll
                for (int k = 0; k < KC1; ++k) wm[k][v] = wa[k][v] = 0.f;
            }
            if (RET) cst(rb, R_RBIAS);
            if (HC) {
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    hb[p] = sC[R_W0 + 2 * KC + 6 + p - R_LR][lv];
#pragma unroll
                    for (int k = 0; k < 3; ++k) hw[p][k] = sC[R_W0 + 2 * KC + 3 * p + k - R_LR][lv];
                }
            }
            if (KC > 0) {
                cst(bm, R_BIAS_M);
                cst(ba, R_BIAS_A);
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    cst(wm[k], R_W0 + k);
                    cst(wa[k], R_W0 + KC + k);
                }
            }
        }

        // ---- front-end, phasors, local scan from zero.  Rows come from LDS as a sliding window.
        float pr[NSTEP][V], pi[NSTEP][V];
        float Er[V], Ei[V];
        float gm[RET ? NSTEP : 1][V], Pth[V];     // RET: retention of each token, product over my tokens
        uint32_t gbits[NSTEP];
        const bool zero_hist = HALO > 0 && !tail_in && tt == 0 && seg == 0;   // rows before a sequence start
        // bf16: the carried conv history is fp32 and is not staged; the one segment that needs it reads it
        // here (and waits for it here, so that no wait for it lands in the common path)
        float hwm[KC1][V], hwa[KC1][V];
#pragma unroll
        for (int k = 0; k < KC1; ++k)
#pragma unroll
            for (int v = 0; v < V; ++v) hwm[k][v] = hwa[k][v] = 0.f;
        const bool hist_bf = BF && HALO > 0 && tail_in && tt == 0 && seg == 0;
        if (hist_bf) {
#pragma unroll
            for (int k = 0; k < HALO; ++k) {
                const size_t o = ((size_t)(b * HALO + k) * 2) * a.J + (active ? j0 : 0);
                hwm[k][0] = tail_in[o];
                hwa[k][0] = tail_in[o + a.J];
            }
            wait_vm<0>();
        }
        // (my lane's valve group in the block is lane / F when heads are narrower than the block)
        const int vbase = (VALVE || RET) ? (a.F >= JB ? 0 : (lv * V) / a.F) * TILE_T + seg * NSTEP : 0;
        // The mode switches are uniform over the launch; each combination gets its own straight-line
        // copy of the loop, so that the tokens' dependent chains (exp -> rcp -> sin/cos) interleave.
        auto front_end = [&](auto amp_c, auto small_c, auto mask_c) {
            constexpr bool AMP = decltype(amp_c)::value, SMALL = decltype(small_c)::value;
            constexpr bool MASK = decltype(mask_c)::value;
            float wnm[KC1][V], wna[KC1][V];           // window: rows i .. i+KC-1 of my segment
            // (row r of my segment lives in slot r % KC1: no register shuffling as the window slides)
#pragma unroll
            for (int k = 0; k < KC1 - 1; ++k) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    wnm[k % KC1][v] = zero_hist ? 0.f : (hist_bf ? hwm[k][v] : su(seg * NSTEP + k, lv * V + v));
                    wna[k % KC1][v] = zero_hist ? 0.f : (hist_bf ? hwa[k][v] : su(NRTP + seg * NSTEP + k, lv * V + v));
                }
            }
#pragma unroll
            for (int v = 0; v < V; ++v) { Er[v] = Ei[v] = 0.f; Pth[v] = 1.f; }
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                gbits[i] = 0;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    wnm[(i + HALO) % KC1][v] = su(seg * NSTEP + i + HALO, lv * V + v);
                    wna[(i + HALO) % KC1][v] = su(NRTP + seg * NSTEP + i + HALO, lv * V + v);
                }
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float zm, xm, phi;
                    if (KC > 0) {
                        zm = bm[v];
                        float za = ba[v];
#pragma unroll
                        for (int k = 0; k < KC; ++k) {
                            zm = __builtin_fmaf(wm[k][v], wnm[(i + k) % KC1][v], zm);
                            za = __builtin_fmaf(wa[k][v], wna[(i + k) % KC1][v], za);
                        }
                        const float cm = clampf(zm, a.conv_clamp), ca = clampf(za, a.conv_clamp);
                        xm = cm * sigmoid_fast(cm);
                        phi = ca * sigmoid_fast(ca);
                    } else {
                        zm = wnm[i % KC1][v];
                        xm = zm;
                        phi = wna[i % KC1][v];
                    }
                    const float amp = AMP ? __builtin_fminf(softplus_fast(xm), 10.0f) : xm;
                    bool g;
                    float ag;
                    if (VALVE) {      // beta = sigmoid(logit - 3), zero when the valve is closed
                        const float vl = sV[vbase + i];
                        g = vl >= a.valve_thr;
                        ag = g ? amp * sigmoid_fast(vl - 3.0f) : 0.0f;
                    } else {
                        g = in_gate(gs_, zm);
                        ag = g ? amp : 0.0f;
                    }
                    float s, c;
                    if (SMALL) sincos_small(phi, s, c);
                    else sincos_fast(phi, s, c);
                    pr[i][v] = ag * c;
                    pi[i][v] = ag * s;
                    if (MASK) gbits[i] |= g ? (1u << v) : 0u;
                    float nr, ni;
                    if (RET) {
                        const float gmv = sigmoid_fast(sR[vbase + i] + rb[v]);
                        gm[i][v] = gmv;
                        Pth[v] *= gmv;
                        const float rr = __builtin_fmaf(lr[v], Er[v], -li[v] * Ei[v]);
                        const float ri = __builtin_fmaf(li[v], Er[v], lr[v] * Ei[v]);
                        nr = __builtin_fmaf(gmv, rr, pr[i][v]);
                        ni = __builtin_fmaf(gmv, ri, pi[i][v]);
                    } else {
                        nr = __builtin_fmaf(lr[v], Er[v], __builtin_fmaf(-li[v], Ei[v], pr[i][v]));
                        ni = __builtin_fmaf(li[v], Er[v], __builtin_fmaf(lr[v], Ei[v], pi[i][v]));
                    }
                    Er[v] = nr;
                    Ei[v] = ni;
                }
            }
        };
        {
            using T_ = std::true_type;
            using F_ = std::false_type;
            switch ((a.amp_mode ? 4 : 0) | (a.small_angle ? 2 : 0) | (a.mask ? 1 : 0)) {
            case 0: front_end(F_{}, F_{}, F_{}); break;
            case 1: front_end(F_{}, F_{}, T_{}); break;
            case 2: front_end(F_{}, T_{}, F_{}); break;
            case 3: front_end(F_{}, T_{}, T_{}); break;
            case 4: front_end(T_{}, F_{}, F_{}); break;
            case 5: front_end(T_{}, F_{}, T_{}); break;
            case 6: front_end(T_{}, T_{}, F_{}); break;
            default: front_end(T_{}, T_{}, T_{}); break;
            }
        }
        CAWN_STAMP(2);

        ARGS_AGAIN();
        // ---- optional gate mask: bit j%32 of word j/32
        if (a.mask) {
            constexpr int TPW = 32 / V;                 // threads per 32-lane word
            const int W = (a.J + 31) >> 5;
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                uint32_t m = (active ? gbits[i] : 0u) << (V * (lv % TPW));
#pragma unroll
                for (int o = 1; o < TPW; o <<= 1) m |= (uint32_t)__shfl_xor((int)m, o, 64);
                const int t = t0 + i;
                if ((lv % TPW) == 0 && active && t < a.L)
                    a.mask[((size_t)b * a.L + t) * W + (j0 >> 5)] = m;
            }
        }

        // ---- segments meet in LDS; after this barrier nobody reads the staged rows any more
#pragma unroll
        for (int v = 0; v < V; ++v) {
            sE[seg][0][lv * V + v] = Er[v];
            sE[seg][1][lv * V + v] = Ei[v];
            if (RET) sP[seg][lv * V + v] = Pth[v];
        }
        if (tid == 0) sTicket[(it + 1) & 1] = ticket_ahead;
        lds_barrier();
        CAWN_STAMP(3);

        // ---- start staging the next tile (it lands during this tile's communication phase)
        const uint32_t next_ticket = (uint32_t)__builtin_amdgcn_readfirstlane((int)sTicket[(it + 1) & 1]);
        TileId Tn{};
        if (next_ticket < qtiles) {
            Tn = tile_of(next_ticket);
            stage_tile(Tn);
        }

        ARGS_AGAIN();
        float Xr[V], Xi[V];   // state entering my segment, from a zero tile input
        float Cs[V];          // RET: product of the retentions of the segments before mine
#pragma unroll
        for (int v = 0; v < V; ++v) { Xr[v] = Xi[v] = 0.f; Cs[v] = 1.f; }
        for (int qq = 0; qq < seg; ++qq) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float er = sE[qq][0][lv * V + v], ei = sE[qq][1][lv * V + v];
                float nr, ni;
                if (RET) {
                    const float pq = sP[qq][lv * V + v];
                    const float rr = __builtin_fmaf(pfr[v], Xr[v], -pfi[v] * Xi[v]);
                    const float ri = __builtin_fmaf(pfi[v], Xr[v], pfr[v] * Xi[v]);
                    nr = __builtin_fmaf(pq, rr, er);
                    ni = __builtin_fmaf(pq, ri, ei);
                    Cs[v] *= pq;
                } else {
                    nr = __builtin_fmaf(pfr[v], Xr[v], __builtin_fmaf(-pfi[v], Xi[v], er));
                    ni = __builtin_fmaf(pfi[v], Xr[v], __builtin_fmaf(pfr[v], Xi[v], ei));
                }
                Xr[v] = nr;
                Xi[v] = ni;
            }
        }

        // ---- chain.  The threads of the last segment own the tile aggregate: they publish it, do
        //      the look-back and publish the prefix, all within their own wave (stores are waited
        //      for with that wave's vmcnt, so no workgroup barrier sits on the publication path).
        const size_t slot = (size_t)id * 2 * JB + lv * V;
        if (is_tail_seg) {
            float Tr[V], Ti[V], hr[V], hi[V], qr[V], qi[V];
            float Pt[V];      // RET: product of the whole tile's retentions
#pragma unroll
            for (int v = 0; v < V; ++v) {
                if (RET) {
                    const float rr = __builtin_fmaf(pfr[v], Xr[v], -pfi[v] * Xi[v]);
                    const float ri = __builtin_fmaf(pfi[v], Xr[v], pfr[v] * Xi[v]);
                    Tr[v] = __builtin_fmaf(Pth[v], rr, Er[v]);
                    Ti[v] = __builtin_fmaf(Pth[v], ri, Ei[v]);
                    Pt[v] = Cs[v] * Pth[v];
                } else {
                    Tr[v] = __builtin_fmaf(pfr[v], Xr[v], __builtin_fmaf(-pfi[v], Xi[v], Er[v]));
                    Ti[v] = __builtin_fmaf(pfi[v], Xr[v], __builtin_fmaf(pfr[v], Xi[v], Ei[v]));
                    Pt[v] = 1.f;
                }
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
                        tagged_store(a.agg + slot + v, Tr[v], tag);
                        tagged_store(a.agg + slot + JB + v, Ti[v], tag);
                        if (RET) tagged_store(a.aggp + (size_t)id * JB + lv * V + v, Pt[v], tag);
                    }
                }
                if (!look_back<V, false, LPR, CAWN_FWD_NB, RET>(a.agg, a.pre, id - (uint32_t)a.B, (uint32_t)a.B, tt, JB, lv * V, lv,
                                                 hr, hi, qr, qi, a.spin_limit, tag, cr, ci, a.aggp)) {
                    // gave up: flag the workspace, keep going so that every wave exits
                    if (lv == 0) __hip_atomic_store(&a.hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            CAWN_STAMP(5);
            // Every load of this block is complete from here on, on every path: a load that some path
            // never uses would stay "in flight" in the compiler's bookkeeping and cost a full wait
            // where its register is reused -- in the replay below, behind the prefix stores.
#pragma unroll
            for (int v = 0; v < V; ++v) asm volatile("" ::"v"(hr[v]), "v"(hi[v]), "v"(qr[v]), "v"(qi[v]));
#pragma unroll
            for (int v = 0; v < V; ++v) {
                sCarry[0][lv * V + v] = cr[v];
                sCarry[1][lv * V + v] = ci[v];
            }
            if (tt + 1 < a.nT) {   // the tile's inclusive prefix for the chain
                float P_r[V], P_i[V];
#pragma unroll
                for (int v = 0; v < V; ++v)
                    chain_step<false>(Tr[v], Ti[v], hr[v], hi[v], qr[v], qi[v], RET ? Pt[v] * cr[v] : cr[v],
                                      RET ? Pt[v] * ci[v] : ci[v], P_r[v], P_i[v]);
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    tagged_store(a.pre + slot + v, P_r[v], tag);
                    tagged_store(a.pre + slot + JB + v, P_i[v], tag);
                }
            }
        }
        lds_barrier_raw();     // the next tile's rows are still on their way
        CAWN_STAMP(6);

        ARGS_AGAIN();
        // ---- true state entering my segment
        float Sr[V], Si[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float cr = sCarry[0][lv * V + v], ci = sCarry[1][lv * V + v];
            if (RET) {
                const float rr = __builtin_fmaf(psr[v], cr, -psi[v] * ci);
                const float ri = __builtin_fmaf(psi[v], cr, psr[v] * ci);
                Sr[v] = __builtin_fmaf(Cs[v], rr, Xr[v]);
                Si[v] = __builtin_fmaf(Cs[v], ri, Xi[v]);
            } else {
                Sr[v] = __builtin_fmaf(psr[v], cr, __builtin_fmaf(-psi[v], ci, Xr[v]));
                Si[v] = __builtin_fmaf(psi[v], cr, __builtin_fmaf(psr[v], ci, Xi[v]));
            }
        }

        // ---- checkpoints for the backward pass: the state before every CKPT_T-th token.  The one at
        //      the start of my segment goes out here, the others from inside the replay.
        float *ckp = a.ckpt ? a.ckpt + (((size_t)b * a.nTc + t0 / CKPT_T) * 2) * a.J + (active ? j0 : 0) : nullptr;
        const uint32_t ck_step = (uint32_t)a.J * 2u * 4u;       // bytes from one checkpoint of a lane to the next
        if (ckp && active && t0 < a.L) {
            Vec<V>::st(ckp, Sr);
            Vec<V>::st(ckp + a.J, Si);
        }

        // ---- replay from the true state, clamp, store.  Addresses are a wave-uniform base plus a
        //      32-bit offset; a tile that lies wholly inside the tensor stores without per-row checks.
        {
            constexpr uint32_t ES = BF ? 2u : 4u;          // bytes per output element
            const size_t obase = ((size_t)b * a.osb + (size_t)(tt * TILE_T) * a.ost + (size_t)T.lb * JB) * ES;
            float *zre = reinterpret_cast<float *>(reinterpret_cast<char *>(a.z_re) + obase);
            float *zim = reinterpret_cast<float *>(reinterpret_cast<char *>(a.z_im) + obase);
            const uint32_t ost32 = (uint32_t)a.ost;
            uint32_t off = ((uint32_t)(seg * NSTEP) * ost32 + (uint32_t)(lv * V)) * ES;   // bytes
            const bool full = (tt + 1) * TILE_T <= a.L && (T.lb + 1) * JB <= a.J;
            const bool plain = full && !(a.state_out && tt == a.nT - 1);   // no per-row checks at all
            // HC: where my lane sits in its head; which neighbour comes from, or goes to, the next block
            const int hq = HC ? (int)((uint32_t)T.lb % hcG) : 0;
            const int hk = HC ? (a.F >= JB ? hq * JB + lv : j0 % a.F) : 0;
            const bool h_first = hk == 0, h_last = hk == a.F - 1;
            // (h_dn: this group goes down the head; the roles of the block's first and last lane swap)
            const bool h_dn = HC && ((ticket / hcG) & 1u);
            const bool h_lo = HC && lv == 0 && hq > 0, h_hi = HC && lv == LPR - 1 && hq + 1 < (int)hcG;
            const bool h_prev = h_dn ? h_hi : h_lo;     // my outer neighbour was left in LDS by the previous tile
            const bool h_defer = h_dn ? h_lo : h_hi;    // my output waits for the next tile
            const bool h_zl = h_first || (h_defer && h_dn), h_zr = h_last || (h_defer && !h_dn);
            const float h_wr = h_dn ? hw[0][0] : hw[0][2], h_wi = h_dn ? hw[1][0] : hw[1][2];   // tap that completes it
            const bool h_tl = h_prev && !h_dn, h_tr = h_prev && h_dn;        // which neighbour comes from LDS
            // where the completed output is stored (0: this lane has none to complete)
            const ptrdiff_t h_back = h_prev ? (h_dn ? (ptrdiff_t)ES : -(ptrdiff_t)ES) : 0;
            auto replay = [&](auto plain_c, auto multi_c, auto ck_c) {
                constexpr bool PLAIN = decltype(plain_c)::value;
                constexpr bool CK = decltype(ck_c)::value;       // checkpoints wanted (uniform over the launch)
                // heads of several lane blocks (1, 2); this tile completes outputs of the previous one (2)
                constexpr bool MULTI = HC && decltype(multi_c)::value > 0, RECV = HC && decltype(multi_c)::value == 2;
                if constexpr (HC) {
                    // The harmonic convolution, four tokens at a time: the recurrence of the four, then all
                    // their lane exchanges and LDS reads (one wait instead of one per token), then outputs.
                    // No branch in here, so the steps stay one block of code.  MULTI (a head spans several
                    // blocks): every lane reads the slot of its row (a broadcast) and selects; every lane
                    // writes -- the deferring lane into the slot, the others into words of sE that only they
                    // write and nobody reads before the next tile rewrites them; the deferring lane's global
                    // stores are masked off and the receiving lane of the next tile stores the completed
                    // element: a second store that only the receiving lane executes (streamed stores are not merged
                    // in a cache: a second store from every lane, repeating its first, doubled the tile's writes).
                    constexpr int CH = 4;
                    static_assert(NSTEP % CH == 0, "whole chunks");
#pragma unroll
                    for (int c0 = 0; c0 < NSTEP; c0 += CH) {
                        float z_r[CH], z_i[CH], lzr[CH], lzi[CH], rzr[CH], rzi[CH], dpr[CH], dpi[CH];
#pragma unroll
                        for (int k = 0; k < CH; ++k) {
                            const int i = c0 + k;
                            float nr, ni;
                            if (RET) {
                                const float rr = __builtin_fmaf(lr[0], Sr[0], -li[0] * Si[0]);
                                const float ri = __builtin_fmaf(li[0], Sr[0], lr[0] * Si[0]);
                                nr = __builtin_fmaf(gm[i][0], rr, pr[i][0]);
                                ni = __builtin_fmaf(gm[i][0], ri, pi[i][0]);
                            } else {
                                nr = __builtin_fmaf(lr[0], Sr[0], __builtin_fmaf(-li[0], Si[0], pr[i][0]));
                                ni = __builtin_fmaf(li[0], Sr[0], __builtin_fmaf(lr[0], Si[0], pi[i][0]));
                            }
                            Sr[0] = nr;
                            Si[0] = ni;
                            if (CK && (i + 1) % CKPT_T == 0 && i + 1 < NSTEP && (PLAIN || (active && t0 + i + 1 < a.L))) {
                                float *cq = reinterpret_cast<float *>(reinterpret_cast<char *>(ckp) + (uint32_t)((i + 1) / CKPT_T) * ck_step);
                                cq[0] = nr;       // (checkpoints are read back by the backward of the same step: cached stores)
                                cq[a.J] = ni;
                            }
                            z_r[k] = clampf(nr, a.out_clamp);
                            z_i[k] = clampf(ni, a.out_clamp);
                            if (!PLAIN && t0 + i == a.L - 1 && a.state_out && active) {
                                a.state_out[((size_t)b * 2 + 0) * a.J + j0] = nr;
                                a.state_out[((size_t)b * 2 + 1) * a.J + j0] = ni;
                            }
                        }
#pragma unroll
                        for (int k = 0; k < CH; ++k) {
                            const int ix = seg * NSTEP + c0 + k;
                            lzr[k] = __shfl_up(z_r[k], 1, 64);
                            lzi[k] = __shfl_up(z_i[k], 1, 64);
                            rzr[k] = __shfl_down(z_r[k], 1, 64);
                            rzi[k] = __shfl_down(z_i[k], 1, 64);
                            dpr[k] = dpi[k] = 0.f;     // the neighbouring block's unfinished output, completed
                            if constexpr (RECV) {
                                const float nzr = sHZ[0][ix], nzi = sHZ[1][ix];
                                lzr[k] = h_tl ? nzr : lzr[k];
                                lzi[k] = h_tl ? nzi : lzi[k];
                                rzr[k] = h_tr ? nzr : rzr[k];
                                rzi[k] = h_tr ? nzi : rzi[k];
                                dpr[k] = __builtin_fmaf(h_wr, z_r[k], sHP[0][ix]);     // (same head: same taps)
                                dpi[k] = __builtin_fmaf(h_wi, z_i[k], sHP[1][ix]);
                            }
                        }
#pragma unroll
                        for (int k = 0; k < CH; ++k) {
                            const int ix = seg * NSTEP + c0 + k;
                            const float l_r = h_zl ? 0.f : lzr[k], l_i = h_zl ? 0.f : lzi[k];
                            const float r_r = h_zr ? 0.f : rzr[k], r_i = h_zr ? 0.f : rzi[k];
                            const float cr_ = __builtin_fmaf(hw[0][2], r_r, __builtin_fmaf(hw[0][1], z_r[k], __builtin_fmaf(hw[0][0], l_r, hb[0])));
                            const float ci_ = __builtin_fmaf(hw[1][2], r_i, __builtin_fmaf(hw[1][1], z_i[k], __builtin_fmaf(hw[1][0], l_i, hb[1])));
                            if constexpr (MULTI) {      // (the reads of these slots, above, come first in this wave)
                                float *wz = h_defer ? &sHZ[0][ix] : &sE[seg][0][lv];
                                float *wp = h_defer ? &sHP[0][ix] : &sE[seg][1][lv];
                                constexpr int PL = FwdGeom::TILE_T;      // from plane 0 to plane 1 of a slot
                                wz[0] = z_r[k];
                                wz[h_defer ? PL : 0] = z_i[k];
                                wp[0] = cr_;
                                wp[h_defer ? PL : 0] = ci_;
                            }
                            // (the deferring lane stores nothing: the receiving lane of the head's next block
                            // stores the completed element, so exactly one store reaches that address)
                            if ((PLAIN || (active && t0 + c0 + k < a.L)) && !(MULTI && h_defer)) {
                                char *pr_ = reinterpret_cast<char *>(zre) + off, *pi_ = reinterpret_cast<char *>(zim) + off;
                                // A head that spans several blocks leaves one element of each row segment to another
                                // tile's store: such rows take the default policy, which merges the two stores in the
                                // cache (streamed, they reach memory as two partial writes of one line: 309 against
                                // 232 us on the training-step shape).  Rows stored by one tile alone are streamed.
                                auto put = [&](char *q, float v) {
                                    if constexpr (BF) {     // (half lines: default policy, see the plain replay below)
                                        *reinterpret_cast<uint16_t *>(q) = to_bf16(v);
                                    } else {
                                        if constexpr (MULTI) *reinterpret_cast<float *>(q) = v;
                                        else st_stream(reinterpret_cast<float *>(q), v);
                                    }
                                };
                                put(pr_, cr_);
                                put(pi_, ci_);
                                if constexpr (RECV) {
                                    if (h_prev) {       // (one lane per segment: a store under its own EXEC mask)
                                        put(pr_ + h_back, dpr[k]);
                                        put(pi_ + h_back, dpi[k]);
                                    }
                                }
                            }
                            off += ost32 * ES;
                        }
                    }
                } else {
#pragma unroll
                for (int i = 0; i < NSTEP; ++i) {
                    const int t = t0 + i;
                    float zr[V], zi[V];
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        float nr, ni;
                        if (RET) {
                            const float rr = __builtin_fmaf(lr[v], Sr[v], -li[v] * Si[v]);
                            const float ri = __builtin_fmaf(li[v], Sr[v], lr[v] * Si[v]);
                            nr = __builtin_fmaf(gm[i][v], rr, pr[i][v]);
                            ni = __builtin_fmaf(gm[i][v], ri, pi[i][v]);
                        } else {
                            nr = __builtin_fmaf(lr[v], Sr[v], __builtin_fmaf(-li[v], Si[v], pr[i][v]));
                            ni = __builtin_fmaf(li[v], Sr[v], __builtin_fmaf(lr[v], Si[v], pi[i][v]));
                        }
                        Sr[v] = nr;
                        Si[v] = ni;
                        zr[v] = clampf(nr, a.out_clamp);
                        zi[v] = clampf(ni, a.out_clamp);
                    }
                    if (CK && (i + 1) % CKPT_T == 0 && i + 1 < NSTEP && (PLAIN || (active && t + 1 < a.L))) {
                        float *cq = reinterpret_cast<float *>(reinterpret_cast<char *>(ckp) + (uint32_t)((i + 1) / CKPT_T) * ck_step);
                        Vec<V>::st(cq, Sr);       // the state before token t + 1
                        Vec<V>::st(cq + a.J, Si);
                    }
                    if (PLAIN || (active && t < a.L)) {
                        if constexpr (BF) {
                            // (a row segment of 32 bf16 lanes is half a 128-byte line: the default policy lets the cache
                            // join it with its neighbour's half; streamed, the forward took 155 against 136 us)
                            *reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(zre) + off) = to_bf16(zr[0]);
                            *reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(zim) + off) = to_bf16(zi[0]);
                        } else {
                            static_assert(V == 1, "streamed output stores: one lane per thread");
                            st_stream(reinterpret_cast<float *>(reinterpret_cast<char *>(zre) + off), zr[0]);
                            st_stream(reinterpret_cast<float *>(reinterpret_cast<char *>(zim) + off), zi[0]);
                        }
                    }
                    if (!PLAIN && t == a.L - 1 && a.state_out && active) {
                        Vec<V>::st(a.state_out + ((size_t)b * 2 + 0) * a.J + j0, Sr);
                        Vec<V>::st(a.state_out + ((size_t)b * 2 + 1) * a.J + j0, Si);
                    }
                    off += ost32 * ES;
                }
                }
            };
            // What is still in flight ahead of this tile's output stores must be complete now: the next
            // tile's staged rows (needed after the next barrier).  The output stores themselves (the
            // 2 * NSTEP youngest operations when no row needed a check) are left in flight.
            // (a tile that completes its predecessor's outputs issues twice the stores, more than the 63 a
            // wave can leave in flight behind its wait: the wait below then covers half of the tile's own
            // stores, about 4 us in a tile of 12; the first tile of a group does not)
            const bool recv_tile = HC && (h_dn ? hq + 1 < (int)hcG : hq > 0);
            using M0 = std::integral_constant<int, 0>;
            using M1 = std::integral_constant<int, 1>;
            using M2 = std::integral_constant<int, 2>;
            using T_ = std::true_type;
            using F_ = std::false_type;
            auto replay_ck = [&](auto plain_c, auto multi_c) {
                if (ckp) replay(plain_c, multi_c, T_{});
                else replay(plain_c, multi_c, F_{});
            };
            if (plain) {
                if (recv_tile) replay_ck(T_{}, M2{});
                else if (HC && hcG > 1) replay_ck(T_{}, M1{});
                else replay_ck(T_{}, M0{});
                wait_vm<(2 * NSTEP < 63 ? 2 * NSTEP : 63)>();
            } else {
                if (recv_tile) replay_ck(F_{}, M2{});
                else if (HC && hcG > 1) replay_ck(F_{}, M1{});
                else replay_ck(F_{}, M0{});
                wait_vm<0>();
            }
        }
        CAWN_STAMP(8);

        // ---- conv history for the next call: last HALO pre-conv rows (written by the last tile,
        //      after its carry arrived, i.e. after the first tile has consumed state_in: safe in place)
        if (HALO > 0 && a.state_out && tt == a.nT - 1 && is_tail_seg && active) {
            float *tail_out = a.state_out + (size_t)a.B * 2 * a.J;
            for (int r = 0; r < HALO; ++r) {
                const int t = a.L - HALO + r;
                float vm[V], va[V];
#pragma unroll
                for (int v = 0; v < V; ++v) vm[v] = va[v] = 0.f;
                if (t >= 0) {
                    const size_t off = (size_t)b * a.isb + (size_t)t * a.ist + j0;
                    if constexpr (BF) {
                        vm[0] = from_bf16(reinterpret_cast<const uint16_t *>(a.mag)[off]);
                        va[0] = from_bf16(reinterpret_cast<const uint16_t *>(a.ang)[off]);
                    } else {
                        Vec<V>::ld(vm, a.mag + off);
                        Vec<V>::ld(va, a.ang + off);
                    }
                } else if (tail_in) {
                    const size_t off = ((size_t)(b * HALO + (t + HALO)) * 2) * a.J + j0;
                    Vec<V>::ld(vm, tail_in + off);
                    Vec<V>::ld(va, tail_in + off + a.J);
                }
                const size_t o = ((size_t)(b * HALO + r) * 2) * a.J + j0;
                Vec<V>::st(tail_out + o, vm);
                Vec<V>::st(tail_out + o + a.J, va);
            }
        }

        ticket = next_ticket;
        T = Tn;
    }

#undef a
#undef ARGS_AGAIN
    // ---- the workgroup that leaves last resets the tickets and advances the epoch for the next call.
    //      Workgroups are counted, not tiles: every one of the grid has then drawn its last ticket.
    if (tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add(&a.hdr->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sLast = (old + 1 == gridDim.x) ? 1u : 0u;
    }
    __syncthreads();
    if (sLast) finish_call(a.hdr, a.clear_from, epoch, tid, blockDim.x);
}

template <int V, int KC, bool VALVE, bool RET, bool BF, bool HC>
static hipError_t launch_fwd_vkh(const FwdArgs &a0, hipStream_t s)
{
    // persistent grid: what fits on the chip (asked once per kernel)
    static int per_cu = 0, cus = 0;
    if (per_cu == 0) {
        int dev = 0, n = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorUnknown;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fwd_kernel<V, KC, VALVE, RET, BF, HC>, FwdGeom::NSEG * FwdLPR, 0) != hipSuccess)
            return hipErrorUnknown;
        cus = prop.multiProcessorCount;
        per_cu = n > 0 ? n : 1;
    }
    FwdArgs a = a0;
    const long long resident = (long long)per_cu * cus;
    const long long tiles = (long long)a.nLB * a.B * a.nT;
    const long long wgs = tiles < resident ? (tiles > 0 ? tiles : 1) : resident;
    dim3 grid((unsigned)wgs), block(FwdGeom::NSEG * FwdLPR);
    hipLaunchKernelGGL((fwd_kernel<V, KC, VALVE, RET, BF, HC>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <int V, int KC, bool VALVE, bool RET, bool BF>
static hipError_t launch_fwd_vk(const FwdArgs &a, hipStream_t s)
{
#ifndef CAWN_DEV_PLAIN
    if constexpr (V == 1) {
        if (a.hconv) return launch_fwd_vkh<1, KC, VALVE, RET, BF, true>(a, s);
    }
#endif
    return launch_fwd_vkh<V, KC, VALVE, RET, BF, false>(a, s);
}

// Tuning aid: -DCAWN_DEV_KC=<k> compiles only the conv_k = k kernels and -DCAWN_DEV_PLAIN only the
// threshold-mode fp32 ones without the harmonic convolution (a build for timing one variant in
// seconds; every other variant then fails to launch with hipErrorInvalidValue).  The library is
// always built without them.
template <int V, bool VALVE, bool RET, bool BF>
static hipError_t launch_fwd_vmb(const FwdArgs &a, int conv_k, hipStream_t s)
{
#ifdef CAWN_DEV_PLAIN
    if constexpr (VALVE || RET || BF) return hipErrorInvalidValue; else
#endif
    switch (conv_k) {
#ifdef CAWN_DEV_KC
    case CAWN_DEV_KC: return launch_fwd_vk<V, CAWN_DEV_KC, VALVE, RET, BF>(a, s);
#else
    case 0: return launch_fwd_vk<V, 0, VALVE, RET, BF>(a, s);
    case 1: return launch_fwd_vk<V, 1, VALVE, RET, BF>(a, s);
    case 2: return launch_fwd_vk<V, 2, VALVE, RET, BF>(a, s);
    case 3: return launch_fwd_vk<V, 3, VALVE, RET, BF>(a, s);
    case 4: return launch_fwd_vk<V, 4, VALVE, RET, BF>(a, s);
#endif
    default: return hipErrorInvalidValue;
    }
}
template <int V, bool VALVE, bool RET>
static hipError_t launch_fwd_vm(const FwdArgs &a, int conv_k, hipStream_t s)
{
    return a.bf16 ? launch_fwd_vmb<V, VALVE, RET, true>(a, conv_k, s) : launch_fwd_vmb<V, VALVE, RET, false>(a, conv_k, s);
}

// One translation unit per family of forward kernels (gate mode x retention mode): they compile side by side.
template <bool VALVE, bool RET>
static hipError_t launch_fwd_family(const FwdArgs &a, int conv_k, bool vec, hipStream_t s)
{
    return vec ? launch_fwd_vm<FwdV, VALVE, RET>(a, conv_k, s) : launch_fwd_vm<1, VALVE, RET>(a, conv_k, s);
}
hipError_t launch_fwd_plain(const FwdArgs &a, int conv_k, bool vec, hipStream_t s);        // threshold gate, constant retention
hipError_t launch_fwd_valve(const FwdArgs &a, int conv_k, bool vec, hipStream_t s);        // per-head valve, constant retention
hipError_t launch_fwd_ret(const FwdArgs &a, int conv_k, bool vec, hipStream_t s);          // threshold gate, data-dependent retention
hipError_t launch_fwd_valve_ret(const FwdArgs &a, int conv_k, bool vec, hipStream_t s);    // valve and data-dependent retention

}  // namespace cawn
