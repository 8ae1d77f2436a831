// Fused backward (Sec. 3.4 last paragraph, Sec. 3.5 of the paper): reverse-time adjoint scan
//   G[t] = dZ[t] + conj(lambda) G[t+1]
// with the front-end recomputed in-kernel, chained to the amplitude (straight-through: no gate
// factor), the phase (gate factor), SiLU', the conv clamp's sub-gradient and the transposed conv.
// Per token-lane HBM traffic: 8 B inputs + 8 B upstream gradient in, 8 B input gradient out.
//
// Same three-level structure as the forward, run against time: tiles of one (batch row, lane
// block) form a chain from the last tile to the first, joined by a decoupled look-back over
// adjoint aggregates.  What differs:
//   * the adjoint aggregate of a tile needs only the upstream gradients, so it is published
//     BEFORE the expensive front-end recompute, which then hides the chain's memory round trips;
//   * the pre-conv input rows are staged once per tile in LDS (direct global->LDS loads): the
//     conv, its halo and the weight gradient all read them from there, not from registers;
//   * parameter gradients need the forward state S[t-1]; every thread rebuilds it for its own tokens
//     from the checkpoint the forward stored for the first of them;
//   * the transposed conv needs the conv pre-activation gradients of the next conv_k-1 tokens.
//     Inside a tile they cross segments through LDS; across tiles the later tile (earlier in the
//     chain) publishes its first conv_k-1 rows through the workspace.
// Parameter gradients leave each tile as per-lane partial sums (fixed order inside the tile) and
// are summed over tiles by a second kernel in a fixed order: results are bitwise repeatable.
#pragma once
#include <type_traits>

#include "cawn_internal.hpp"

namespace cawn {

#ifdef CAWN_TIMING
#define BWD_STAMP(k) do { if (threadIdx.x == 0) a.dbg[(size_t)ticket * 16 + (k)] = wall_clock64(); } while (0)
#else
#define BWD_STAMP(k) do { } while (0)
#endif

// x + (x moved across lanes by a DPP control): row_ror:n is 0x120 + n (rotate within a row of 16).
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
// rows 1 and 3 of the wave add lane 15 of the row below them (row_bcast:15); rows 0 and 2 add zero
__device__ __forceinline__ float dpp_add_bcast15(float x)
{
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x142, 0xA, 0xF, false));
}

// Whole-wave shifts by one lane (DPP wave_shr:1 / wave_shl:1): lane i takes lane i-1's (i+1's) value, the
// first (last) lane keeps its own.
__device__ __forceinline__ float wave_shift_up(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), 0x138, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_shift_down(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), 0x130, 0xF, 0xF, false));
}

template <int V> struct BVec;
template <> struct BVec<1> {
    static __device__ __forceinline__ void ld(float (&d)[1], const float *p) { d[0] = *p; }
    static __device__ __forceinline__ void st(float *p, const float (&s)[1]) { *p = s[0]; }
};
template <> struct BVec<2> {
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

// Access at a wave-uniform base plus a 32-bit per-lane byte offset: the addressing mode that costs no
// vector ALU work (scalar base register + 32-bit offset register).
template <int V>
__device__ __forceinline__ void ldu(float (&d)[V], const float *ubase, uint32_t boff)
{
    BVec<V>::ld(d, reinterpret_cast<const float *>(reinterpret_cast<const char *>(ubase) + boff));
}
template <int V>
__device__ __forceinline__ void stu(float *ubase, uint32_t boff, const float (&x)[V])
{
    BVec<V>::st(reinterpret_cast<float *>(reinterpret_cast<char *>(ubase) + boff), x);
}

// Sum of w over the lanes that share a head inside the 32-lane block (8, 16 or 32 lanes).  Rotations
// within each row of 16 lanes leave the row's sum in all of its lanes (four full-rate adds); a 32-lane
// group then takes the lower row's sum into its upper row.  The total is valid in the lanes for which
// head_sum_lane() holds.
__device__ __forceinline__ float head_sum(float w, int vwidth)
{
    if (vwidth >= 16) {
        w = dpp_add<0x128>(w);
        w = dpp_add<0x124>(w);
        w = dpp_add<0x122>(w);
        w = dpp_add<0x121>(w);
        if (vwidth == 32) w = dpp_add_bcast15(w);
    } else {
#pragma unroll
        for (int o = 4; o >= 1; o >>= 1)
            if (o < vwidth) w += __shfl_xor(w, o, 64);
    }
    return w;
}
__device__ __forceinline__ bool head_sum_lane(int lv, int vwidth)
{
    return vwidth >= 16 ? (lv == vwidth - 16 || (vwidth == 16 && lv == 16)) : (lv % vwidth == 0);
}

// VALVE: gate_mode 1, the per-head input valve of Sec. 3.3 in place of the per-lane threshold.
// RET: ret_mode 1, the retention gamma[t] = sigmoid(logit[t][head] + b_k) of Sec. 3.3 item 4.  The
// adjoint then is G[t] = dZ[t] + gamma[t+1] conj(e^{i theta}) G[t+1]; every level carries the MESSAGE
// M[t] = gamma[t] conj(e^{i theta}) G[t] that token t hands to token t-1 (so a run of tokens never needs
// its neighbour's retention) and, beside each aggregate, the real product of the run's retentions; the
// lane table holds pure rotations.  The logit's gradient needs S[t-1], so these kernels always rebuild
// the forward state (PARAM).
// BF: activations (mag, ang, dz_re, dz_im in; dmag, dang out) are bfloat16 in memory, as in the forward.
// HC: the forward ended in the depth-wise harmonic convolution of Sec. 3.6 (three taps along the harmonics of
// each head, per plane), so dz_re / dz_im are gradients of the CONVOLVED output C.  The transposed convolution
//   dZ[k] = w0 dC[k+1] + w1 dC[k] + w2 dC[k-1]      (positions outside the head contribute nothing)
// is applied as the staged gradients are read; a lane block's neighbours (lanes -1 and 32) are staged beside
// the rows.  The tap gradients d w_i = sum dC[k] Z[k+i-1] = sum_k' Z[k'] dC[k'-i+1] pair a thread's own
// clamped state Z (rebuilt in the front-end) with the same three gradients, read again from LDS there; they
// leave the tile as 8 more rows of per-lane partial sums.
template <int V, int KC, bool PARAM, bool VALVE, bool RET, bool BF, bool HC = false>
__global__ __launch_bounds__(BwdGeom::NSEG *BwdLPR, CAWN_BWD_WAVES) void bwd_kernel(const BwdArgs a)
{
    static_assert(!HC || (PARAM && V == 1), "harmonic convolution: with the state rebuild, one lane per thread");
    static_assert(!BF || V == 1, "bf16 activations: one lane per thread");
    static_assert(!RET || (PARAM && V == 1), "retention kernels rebuild the forward state; one lane per thread");
    // The valve and retention kernels sit at the register budget.  They keep the reduced angle instead
    // of its sin and cos between the front-end and the reverse pass, park the conv taps in LDS during
    // the reverse pass and fetch the reverse-pass constants after the front-end.
    constexpr bool LEAN = VALVE || RET;
    constexpr int TILE_T = BwdGeom::TILE_T, NSTEP = BwdGeom::NSTEP, NSEG = BwdGeom::NSEG, LPR = BwdLPR;
    constexpr int JB = V * LPR;
    constexpr int HALO = KC > 0 ? KC - 1 : 0;
    constexpr int HALO1 = HALO > 0 ? HALO : 1;
    constexpr int KC1 = KC > 0 ? KC : 1;
    constexpr int ROWS = 4 + 2 * KC + (HC ? HC_PART_ROWS : 0);
    constexpr int NT = NSEG * LPR, NW = NT / 64;
    constexpr int JBS = BF ? JB / 2 : JB;          // four-byte words per staged row
    constexpr uint32_t ES = BF ? 2u : 4u;          // bytes per activation element
    constexpr int NRTP = staged_rows<TILE_T, JBS, HALO>();   // staged rows per stream: time tile_t0-HALO+rr
    static_assert(HALO <= NSTEP, "conv halo must fit in one segment");
    static_assert(!VALVE || V == 1, "the valve's lane reduction takes one lane per thread");
    static_assert(LPR == 32, "the partial-sum reduction pairs the two segments of a wave");
    static_assert(JB <= 64 && 64 % JB == 0, "a staged row must fit a wave");

    __shared__ __attribute__((aligned(16))) float sU[2 * NRTP][JBS];  // [stream*NRTP + rr][lane]
    // element (row, lane) of the staged rows as fp32
    auto su = [&](int r, int l) -> float {
        if constexpr (BF) return from_bf16(reinterpret_cast<const uint16_t *>(&sU[r][0])[l]);
        else return sU[r][l];
    };
    // PF: the upstream gradients of a tile are staged in LDS a tile ahead (direct-to-LDS loads issued
    // while the previous tile is in its front-end), so that a tile starts its local adjoint, and
    // publishes its aggregate, without waiting for memory.  The 32 KB this takes fit beside the rest
    // only because arrays with disjoint lifetimes share storage: the conv-gradient halo rows (written
    // after the reverse pass) lie over the segment aggregates (dead by then), and the partial-sum
    // staging lies over the input rows (dead after the last weight-gradient read, one more barrier).
    constexpr bool PF = !VALVE && !RET;
    // SDZ: the upstream gradients pass through LDS at all.  The valve and retention kernels load them into
    // registers, except behind the harmonic convolution: its transposed form and its tap gradients read three
    // neighbouring lanes of every gradient, twice in a tile, so there the tile's gradients are staged too -- at
    // the top of the tile itself, not a tile ahead (see OVL below for where the 32 KB come from).
    constexpr bool SDZ = PF || HC;
    constexpr int NRZ = staged_rows<TILE_T, JBS, 0>();                // staged rows per gradient stream
    __shared__ __attribute__((aligned(16))) float sDz[SDZ ? 2 * NRZ : 1][JBS];    // [stream*NRZ + token][lane]
    // ... and with them the four lane constants the local adjoint needs (lambda, lambda^NSTEP): a wave's
    // memory operations complete in issue order, so a load issued at the top of a tile returns only after
    // the previous tile's output stores have been acknowledged
    // HC: ... and the lane block's harmonic-convolution taps (table rows R_W0 + 2 KC + 0 .. 7)
    __shared__ float sLam[SDZ ? (HC ? 4 + HC_ROWS : 4) : 1][JB];
    // HC: the gradients of the two lanes beside the lane block, [plane][side: lane -1, lane JB][token]
    __shared__ float sEdge[HC ? 4 * NRZ : 1];
    constexpr int N_EB = NSEG * 2 * JB, N_HALO = NW * HALO1 * 2 * JB;
    // OVL: the valve and retention kernels behind the harmonic convolution (fp32 rows) stage a tile's gradients at
    // its top and read them for the last time in the tap pass, in the middle of the tile: what is written only
    // after the barrier that follows that pass -- the conv-gradient halo rows, the valve's and the retention
    // logits' gradient terms, the partial-sum staging -- lies over them.  With that the kernel fits twice on a
    // compute unit.
    constexpr bool OVL = HC && !PF && !BF;
    constexpr int N_RED = NW * ROWS * JB, N_VT = BwdGeom::TILE_T * 4;
    static_assert(!OVL || N_RED + N_HALO + 2 * N_VT <= 2 * NRZ * JBS, "what lies over the staged gradients fits there");
    __shared__ float sPool[PF ? (N_EB > N_HALO ? N_EB : N_HALO) : (OVL ? N_EB : N_EB + N_HALO)];
    float (*sEb)[2][JB] = reinterpret_cast<float (*)[2][JB]>(&sPool[0]);
    float (*sHalo)[HALO1][2][JB] = reinterpret_cast<float (*)[HALO1][2][JB]>(OVL ? &sDz[0][0] + N_RED : &sPool[PF ? 0 : N_EB]);   // [NW]: first rows of each wave's earlier segment
    __shared__ float sCarry[2][JB];
    // (bf16 rows are half as large and the harmonic convolution adds 8 partial rows: that combination has LDS to
    // spare and keeps the staging in an array of its own)
    constexpr bool RED_OVER_ROWS = PF && !(BF && HC);
    __shared__ float sRedOwn[(PARAM && !RED_OVER_ROWS && !OVL) ? NW : 1][ROWS][JB];
    static_assert(!RED_OVER_ROWS || (size_t)NW * ROWS * JB <= (size_t)2 * NRTP * JBS, "the partial-sum staging fits over the input rows");
    float (*sRed)[ROWS][JB] = RED_OVER_ROWS ? reinterpret_cast<float (*)[ROWS][JB]>(&sU[0][0])
                                            : (OVL ? reinterpret_cast<float (*)[ROWS][JB]>(&sDz[0][0]) : sRedOwn);
    constexpr int GPB_MAX = 4;                    // valve groups per lane block (F >= 8)
    static_assert(N_VT == BwdGeom::TILE_T * GPB_MAX, "");
    __shared__ float sV[VALVE ? BwdGeom::TILE_T * GPB_MAX : 1];      // valve logits, [group][token]
    __shared__ float sVpOwn[VALVE && !OVL ? BwdGeom::TILE_T * GPB_MAX : 1];     // valve gradient terms summed over a group's lanes
    float *sVp = OVL ? &sDz[0][0] + N_RED + N_HALO : sVpOwn;
    __shared__ float sTaps[LEAN ? 2 * KC1 : 1][JB];                 // conv taps of the lane block (valve kernels)
    __shared__ float sPb[RET ? NSEG : 1][JB];                        // product of each wave's retentions
    __shared__ float sPt[RET ? 1 : 1][JB];                           // product of the tile's retentions (head group)
    __shared__ float sRpOwn[RET && !OVL ? BwdGeom::TILE_T * GPB_MAX : 1];       // retention-logit gradient terms per (group, token)
    float *sRp = OVL ? &sDz[0][0] + N_RED + N_HALO + N_VT : sRpOwn;
    __shared__ uint32_t sTicket[2], sLast, sEpoch;     // tickets of this tile and the next one

    const int tid_ = threadIdx.x;
    const float *tail_in = a.state_in ? a.state_in + (size_t)a.B * 2 * a.J : nullptr;
    const float *dtail_out = a.dstate_out ? a.dstate_out + (size_t)a.B * 2 * a.J : nullptr;
    const uint32_t chain_stride = (uint32_t)a.B * a.nLB;
    const uint32_t ost32 = (uint32_t)a.ost, ist32 = (uint32_t)a.ist;
    uint32_t ticket_ahead = 0;   // thread 0: the ticket asked for in this tile, until it is parked in LDS
    if (tid_ == 0) {
        const uint32_t e = flag_load(&a.hdr->epoch);     // all three round trips at once
        const uint32_t t = __hip_atomic_fetch_add(&a.hdr->ticket[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sEpoch = e;
        sTicket[0] = t;
        sLast = 0;
    }
    __syncthreads();
    uint32_t ticket = (uint32_t)__builtin_amdgcn_readfirstlane((int)sTicket[0]);   // wave-uniform: index math stays scalar
    const uint32_t epoch = (uint32_t)__builtin_amdgcn_readfirstlane((int)sEpoch);
    const uint32_t tag = make_tag(epoch);      // of every word this call publishes

    // Persistent: each workgroup loops over tiles, handed out in chain order by an atomic ticket.  A
    // workgroup also holds the ticket of its next tile: it asks for it just before the previous tile's
    // output stores go out (a wave's memory operations complete in issue order: asked for behind them,
    // at the top of a tile, the answer would arrive only after they are acknowledged, and the next tile
    // must be known early, for its staged gradients).  Every workgroup works through its tickets in
    // increasing order and a tile waits only for lower tickets, so the lowest unfinished ticket is always
    // some workgroup's current tile: no wait can last.  (Holding tickets two tiles ahead was tried: the
    // reserved tiles start later and their successors in other workgroups wait for them, +3 % to +30 %.)
    // The kernel's arguments are read from the kernel-argument segment again in every phase of a tile
    // (scalar loads next to their use, `ARGS_AGAIN()` makes the compiler forget what it loaded) instead
    // of living in scalar registers across the loop: kept there they overflow the scalar register file,
    // and every overflowing value costs vector instructions (lane writes and reads) on each use.
    const uint32_t total_tiles_ = a.total_tiles;
    typedef const __attribute__((address_space(4))) BwdArgs *KArgs;
    for (int it = 0; ticket < total_tiles_; ++it) {
    KArgs ap = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
#define a (*ap)
#define ARGS_AGAIN() asm volatile("" : "+s"(ap))
    // (opaque copies: anything computed from them is computed inside the loop and does not occupy
    // registers across it)
    int tid = tid_;
    asm volatile("" : "+v"(tid));
    const int lv = tid % LPR, seg = tid / LPR;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // (wave index: scalar)
    const float *table = a.table;      // (the same for the lane table's base and row pitch: the ~30 row
    int Jp = a.Jp;                     // addresses are then formed per tile instead of living in scalar
    asm volatile("" : "+s"(table), "+s"(Jp));   // registers across the loop, which spilled)
    BWD_STAMP(1);
    const int lb = ticket % a.nLB;
    const int rest = ticket / a.nLB;
    const int b = rest % a.B, ttr = rest / a.B;       // ttr: position in the chain (0 = last tile in time)
    const int tt = a.nT - 1 - ttr;
    const int j0 = lb * JB + lv * V;
    const bool active = j0 < a.J;
    // Lane constants are read unconditionally; lanes beyond J read lane 0's (their results are never
    // stored, and no value crosses lanes).
    const uint32_t jb = (uint32_t)(active ? j0 : 0) * 4u;
    auto row = [&](int r) { return table + (size_t)r * Jp; };
    const int t0 = tt * TILE_T + seg * NSTEP;
    const bool head = seg == 0;                       // owns the tile's adjoint aggregate and the chain
    const bool chained = ttr > 0;                     // has a predecessor in the chain
    const bool feeds = tt > 0;                        // has a successor in the chain

    // (the wave that owns the chain runs at raised priority until the tile's prefix is out: what it does in
    // that span -- aggregate, look-back, prefix -- is what other tiles wait for; 0.5 % on the whole kernel)
    if (wave == 0) __builtin_amdgcn_s_setprio(2);
    // ---- upstream gradients of my tokens (registers), then the tile's input rows (LDS)
    float dzr[NSTEP][V], dzi[NSTEP][V];     // upstream dS, later overwritten by d(pre-activation)
    // a tile that lies wholly inside the tensors loads and stores without per-row checks
    const bool full = (tt + 1) * TILE_T <= a.L && (lb + 1) * JB <= a.J;
    // (upstream gradients of tile (b_, tt_, lb_) into sDz: rows of J lanes, or J/2 words with bf16)
    auto stage_dz = [&](int b_, int tt_, int lb_, int wv, int nwv) {
        if (wave == NW - 1) {       // rows R_LR, R_LI, then R_PSEGB + 2, + 3 of the lane block: two loads of two rows
            [[maybe_unused]] const int jl = lb_ * JB + (lane & (JB - 1));
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_global_load_lds(table + (size_t)(R_LR + (lane >> 5)) * Jp + jl, &sLam[0][0], 4, 0, 0);
            __builtin_amdgcn_global_load_lds(table + (size_t)(R_PSEGB + 2 + (lane >> 5)) * Jp + jl, &sLam[2][0], 4, 0, 0);
            if constexpr (HC) {
#pragma unroll
                for (int q = 0; q < HC_ROWS / 2; ++q)
                    __builtin_amdgcn_global_load_lds(table + (size_t)(R_W0 + 2 * KC + 2 * q + (lane >> 5)) * Jp + jl,
                                                     &sLam[4 + 2 * q][0], 4, 0, 0);
            }
#endif
        }
        if constexpr (HC) {
            // the two neighbour lanes of the block, 64 tokens per instruction; rows past the end and lanes
            // outside the tensor read a valid address (their values are masked where they are used)
            // (a side whose neighbour lies in another head is never used: not fetched.  Heads of 32 lanes or
            // fewer need none, heads of 64 one side per block)
            const bool need_lo = ((lb_ * JB) & (a.F - 1)) != 0, need_hi = ((lb_ * JB + JB) & (a.F - 1)) != 0;
            for (int e = wv; e < 8; e += nwv) {
                const int plane = e >> 2, side = (e >> 1) & 1, half = e & 1;
                if (side ? !need_hi : !need_lo) continue;
                int t = tt_ * TILE_T + half * 64 + lane;
                t = t < a.L ? t : a.L - 1;
                int j = side ? lb_ * JB + JB : lb_ * JB - 1;
                j = j < 0 ? 0 : (j >= a.J ? a.J - 1 : j);
                // (bf16: the four-byte word that holds the element -- strides and the block's first lane are even, so
                // lane -1 is the upper half of its word and lane JB the lower half of its own)
                const size_t e_ = (size_t)b_ * a.osb + (size_t)t * a.ost + j;
                const float *src = BF ? reinterpret_cast<const float *>(reinterpret_cast<const uint16_t *>(plane ? a.dz_im : a.dz_re) + (e_ & ~(size_t)1))
                                      : (plane ? a.dz_im : a.dz_re) + e_;
#if defined(__HIP_DEVICE_COMPILE__)
                __builtin_amdgcn_global_load_lds(src, &sEdge[(plane * 2 + side) * NRZ + half * 64], 4, 0, 0);
#else
                (void)src;
#endif
            }
        }
        if (a.stage16z)
            stage_rows<TILE_T, JBS, 0, 16>(&sDz[0][0], a.dz_re, a.dz_im, nullptr, b_, tt_ * TILE_T, lb_, BF ? a.J / 2 : a.J, a.L,
                                   BF ? a.osb / 2 : a.osb, BF ? (int)a.ost / 2 : (int)a.ost, wv, nwv, lane);
        else
            stage_rows<TILE_T, JBS, 0, 4>(&sDz[0][0], a.dz_re, a.dz_im, nullptr, b_, tt_ * TILE_T, lb_, BF ? a.J / 2 : a.J, a.L,
                                  BF ? a.osb / 2 : a.osb, BF ? (int)a.ost / 2 : (int)a.ost, wv, nwv, lane);
    };
    // HC: the gradients of convolved-output positions k-1, k, k+1 of token i of my segment ([0], [1], [2]), zero
    // where the position lies outside my head or the token outside the tensor.  Head widths are powers of two.
    // My own position comes from LDS, the neighbours' by a lane exchange of it (lanes 0 and 31 of the block take
    // the staged edge instead).  What depends on the lane alone is set up once per pass from an opaque copy of
    // the thread index, not carried across the tile; every read is unconditional and pinned, so that the
    // choices below are selects on loaded values (a read inside one arm of a choice becomes a branch around it).
    struct HcLane { int own, edge, nlive; bool use_lo, use_hi, first, last; };
    auto hc_setup = [&]() {
        int t_ = tid_;
        asm volatile("" : "+v"(t_));
        const int lv_ = t_ % LPR, sg_ = t_ / LPR;
        const int kh = (lb * JB + lv_) & (a.F - 1);
        HcLane k;
        k.own = sg_ * NSTEP * (BF ? 2 * JBS : JBS) + lv_;         // element offset of (my first token, my lane) in a plane of sDz
        k.edge = (lv_ == 0 ? 0 : NRZ) + sg_ * NSTEP;             // word offset of my first token in my side of sEdge
        const int left = a.L - (tt * TILE_T + sg_ * NSTEP);
        k.nlive = full ? NSTEP : ((lb * JB + lv_ < a.J) ? (left < 0 ? 0 : (left > NSTEP ? NSTEP : left)) : 0);
        k.first = kh == 0;
        k.last = kh == a.F - 1;
        // (the staged edge is taken only where it was fetched: a block edge inside a head.  At a head's end the
        // shifted value stands in -- finite data that the callers' zero tap or final select discards)
        k.use_lo = lv_ == 0 && !k.first;
        k.use_hi = lv_ == LPR - 1 && !k.last;
        return k;
    };
    auto hc_read = [&](auto full_c, int i, const HcLane &k, float (&cr)[3], float (&ci)[3]) {
        constexpr bool FULL = decltype(full_c)::value;
        if constexpr (HC) {
            float c0r, c0i, er = sEdge[k.edge + i], ei = sEdge[2 * NRZ + k.edge + i];
            if constexpr (BF) {
                c0r = from_bf16(reinterpret_cast<const uint16_t *>(&sDz[0][0])[k.own + i * 2 * JBS]);
                c0i = from_bf16(reinterpret_cast<const uint16_t *>(&sDz[NRZ][0])[k.own + i * 2 * JBS]);
                // the staged word's half that is my neighbour: upper for lane -1, lower for lane JB
                const uint32_t wr = __float_as_uint(er), wi = __float_as_uint(ei);
                er = __uint_as_float(k.use_lo ? (wr & 0xffff0000u) : (wr << 16));
                ei = __uint_as_float(k.use_lo ? (wi & 0xffff0000u) : (wi << 16));
            } else {
                c0r = (&sDz[0][0])[k.own + i * JBS];
                c0i = (&sDz[NRZ][0])[k.own + i * JBS];
            }
            asm volatile("" : "+v"(c0r), "+v"(c0i), "+v"(er), "+v"(ei));
            if constexpr (!FULL) {      // rows and lanes outside the tensor staged a valid address: their values count as zero
                const bool live = i < k.nlive;
                c0r = live ? c0r : 0.f;
                c0i = live ? c0i : 0.f;
                er = live ? er : 0.f;
                ei = live ? ei : 0.f;
            }
            // (whole-wave shifts by one lane, in the vector ALU: they cross the two segments of a wave at lanes
            // 31 | 32, exactly the lanes that take the staged edge instead.  Positions outside the head are NOT
            // zeroed here: the callers fold that into the taps, or into the finished sums, once per tile.)
            // The shifts are statements of their own, in front of every choice: written inside one arm of a `?:` a
            // shift runs under that arm's narrowed EXEC mask, and a lane whose source lane is switched off keeps its
            // own value.  (Cross-lane operations are convergent: the compiler does not move them under a condition.)
            const float mr = wave_shift_up(c0r), mi = wave_shift_up(c0i), pr = wave_shift_down(c0r), pi = wave_shift_down(c0i);
            cr[0] = k.use_lo ? er : mr;
            ci[0] = k.use_lo ? ei : mi;
            cr[2] = k.use_hi ? er : pr;
            ci[2] = k.use_hi ? ei : pi;
            cr[1] = c0r;
            ci[1] = c0i;
        }
    };
    if (SDZ) {
        if (!PF || it == 0) {      // a workgroup's first tile: nobody staged its gradients ahead
            stage_dz(b, tt, lb, wave, NW);
            wait_vm<0>();
            lds_barrier();
        }
        // (later tiles: staged during the previous tile, complete before its closing barrier)
        auto dz_from_lds = [&](auto full_c) {
            constexpr bool FULL = decltype(full_c)::value;
            if constexpr (HC) {     // transposed harmonic convolution of the staged gradients
                float w_[2][3];
#pragma unroll
                for (int p_ = 0; p_ < 2; ++p_)
#pragma unroll
                    for (int q = 0; q < 3; ++q) w_[p_][q] = sLam[4 + 3 * p_ + q][lv];
                const HcLane hk = hc_setup();
#pragma unroll
                for (int p_ = 0; p_ < 2; ++p_) {     // a neighbour outside my head contributes nothing
                    w_[p_][0] = hk.last ? 0.f : w_[p_][0];      // tap 0 meets the gradient at k+1
                    w_[p_][2] = hk.first ? 0.f : w_[p_][2];     // tap 2 the one at k-1
                }
#pragma unroll
                for (int i = 0; i < NSTEP; ++i) {
                    float cr[3], ci[3];
                    hc_read(full_c, i, hk, cr, ci);
                    dzr[i][0] = __builtin_fmaf(w_[0][0], cr[2], __builtin_fmaf(w_[0][1], cr[1], w_[0][2] * cr[0]));
                    dzi[i][0] = __builtin_fmaf(w_[1][0], ci[2], __builtin_fmaf(w_[1][1], ci[1], w_[1][2] * ci[0]));
                    if (i & 1) __builtin_amdgcn_sched_barrier(0);     // (two tokens' reads in flight, not all eight)
                }
                return;
            }
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                const int r = seg * NSTEP + i;
                float vr, vi;
                if constexpr (BF) {
                    vr = from_bf16(reinterpret_cast<const uint16_t *>(&sDz[r][0])[lv]);
                    vi = from_bf16(reinterpret_cast<const uint16_t *>(&sDz[NRZ + r][0])[lv]);
                } else {
                    vr = sDz[r][lv];
                    vi = sDz[NRZ + r][lv];
                }
                const bool live = FULL || (active && t0 + i < a.L);     // rows and lanes outside the tensor staged a valid address
                dzr[i][0] = live ? vr : 0.f;
                dzi[i][0] = live ? vi : 0.f;
            }
        };
        // (a tile that lies wholly inside the tensors takes the rows as they are: no per-row selects)
        if (full) dz_from_lds(std::true_type{});
        else dz_from_lds(std::false_type{});
    } else {
        const size_t gbase = ((size_t)b * a.osb + (size_t)(tt * TILE_T) * a.ost + (size_t)lb * JB) * ES;
        const float *gre = reinterpret_cast<const float *>(reinterpret_cast<const char *>(a.dz_re) + gbase);
        const float *gim = reinterpret_cast<const float *>(reinterpret_cast<const char *>(a.dz_im) + gbase);
        uint32_t off = ((uint32_t)(seg * NSTEP) * ost32 + (uint32_t)(lv * V)) * ES;      // bytes
        auto ldg = [&](float (&d)[V], const float *ub, uint32_t bo) {
            // (read once: streamed, like the staged rows; bf16 rows are half lines and keep the default policy)
            if constexpr (BF) d[0] = from_bf16(*reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(ub) + bo));
            else d[0] = __builtin_nontemporal_load(reinterpret_cast<const float *>(reinterpret_cast<const char *>(ub) + bo));
        };
        if (full) {
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                ldg(dzr[i], gre, off);
                ldg(dzi[i], gim, off);
                off += ost32 * ES;
            }
        } else {
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
#pragma unroll
                for (int v = 0; v < V; ++v) dzr[i][v] = dzi[i][v] = 0.f;
                if (active && t0 + i < a.L) {
                    ldg(dzr[i], gre, off);
                    ldg(dzi[i], gim, off);
                }
                off += ost32 * ES;
            }
        }
    }
    // ---- retention logits of my tokens (one per token and head: the lanes of a head read one address)
    float gm[RET ? NSTEP : 1][V];           // logit, then the retention itself
    if (RET) {
        const float *rp = a.ret + (size_t)b * a.L * a.H + (active ? j0 : 0) / a.F;
#pragma unroll
        for (int i = 0; i < NSTEP; ++i) {
            const int t = t0 + i < a.L ? t0 + i : a.L - 1;     // rows past the end: a valid address, the value is harmless
            gm[i][0] = rp[(size_t)t * a.H];
        }
    }
    // ---- lane constants
    float lr[V], li[V], pnr[V], pni[V];
    float wmf[KC1][V], waf[KC1][V], bm[V], ba[V];   // taps for the front-end
    if (PF) {       // staged with the gradients (lanes beyond J hold table padding: their results are never stored)
        lr[0] = sLam[0][lv];
        li[0] = sLam[1][lv];
        pnr[0] = sLam[2][lv];
        pni[0] = sLam[3][lv];
    } else {
        ldu<V>(lr, row(R_LR), jb);
        ldu<V>(li, row(R_LI), jb);
        ldu<V>(pnr, row(R_PSEGB + 2), jb);                       // lambda^NSTEP
        ldu<V>(pni, row(R_PSEGB + 3), jb);
    }
    // the forward state before my first token: the checkpoint of my segment (PF: fetched here, so that it
    // has arrived with the staged rows; the other kernels fetch it behind that wait, next to the
    // constants of the reverse pass)
    float kr[V], ki[V];
#pragma unroll
    for (int v = 0; v < V; ++v) kr[v] = ki[v] = 0.f;
    auto load_ckpt = [&]() {
        if (PARAM && active && a.ckpt && t0 < a.L) {
            const float *ck = a.ckpt + (((size_t)b * a.nTc + t0 / CKPT_T) * 2) * a.J + j0;
            BVec<V>::ld(kr, ck);
            BVec<V>::ld(ki, ck + a.J);
        }
    };
    if (PF) load_ckpt();
    float rb[V];
#pragma unroll
    for (int v = 0; v < V; ++v) rb[v] = 0.f;
    if (RET) ldu<V>(rb, row(R_RBIAS), jb);
#pragma unroll
    for (int v = 0; v < V; ++v) {
        bm[v] = ba[v] = 0.f;
#pragma unroll
        for (int k = 0; k < KC1; ++k) wmf[k][v] = waf[k][v] = 0.f;
    }
    if (KC > 0) {
        ldu<V>(bm, row(R_BIAS_M), jb);
        ldu<V>(ba, row(R_BIAS_A), jb);
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            ldu<V>(wmf[k], row(R_W0 + k), jb);
            ldu<V>(waf[k], row(R_W0 + KC + k), jb);
        }
    }
    if (LEAN && KC > 0 && seg == 0) {      // (read back after the barrier before the transposed conv)
#pragma unroll
        for (int k = 0; k < KC; ++k)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                sTaps[k][lv * V + v] = wmf[k][v];
                sTaps[KC + k][lv * V + v] = waf[k][v];
            }
    }

    // ---- the tile's input rows go to LDS (needed from the front-end on; issued after the loads the
    //      local adjoint waits for, so that it does not wait for these as well)
    // (bf16: rows of J/2 words at half the strides; the fp32 conv history is read at its points of use)
    if (a.stage16)
        stage_rows<TILE_T, JBS, HALO, 16>(&sU[0][0], a.mag, a.ang, BF ? nullptr : tail_in, b, tt * TILE_T, lb, BF ? a.J / 2 : a.J,
                                  a.L, BF ? a.isb / 2 : a.isb, BF ? (int)a.ist / 2 : (int)a.ist, wave, NW, lane);
    else
        stage_rows<TILE_T, JBS, HALO, 4>(&sU[0][0], a.mag, a.ang, BF ? nullptr : tail_in, b, tt * TILE_T, lb, BF ? a.J / 2 : a.J,
                                 a.L, BF ? a.isb / 2 : a.isb, BF ? (int)a.ist / 2 : (int)a.ist, wave, NW, lane);

    if (VALVE && wave == 0) stage_valve<TILE_T, JB>(&sV[0], a.valve, b, tt * TILE_T, lb, a.L, a.H, a.F, a.gpb, lane);

    // gradient of the carried state joins the last token
    if (a.dstate_out && active && a.L - 1 >= t0 && a.L - 1 < t0 + NSTEP) {
        float xr[V], xi[V];
        BVec<V>::ld(xr, a.dstate_out + ((size_t)b * 2 + 0) * a.J + j0);
        BVec<V>::ld(xi, a.dstate_out + ((size_t)b * 2 + 1) * a.J + j0);
#pragma unroll
        for (int i = 0; i < NSTEP; ++i)
            if (t0 + i == a.L - 1) {
#pragma unroll
                for (int v = 0; v < V; ++v) { dzr[i][v] += xr[v]; dzi[i][v] += xi[v]; }
            }
    }

    // ---- adjoint from zero over my segment (needs only the upstream gradients)
    float Ebr[V], Ebi[V];
    float Pth[V];           // RET: product of my tokens' retentions
#pragma unroll
    for (int v = 0; v < V; ++v) { Ebr[v] = Ebi[v] = 0.f; Pth[v] = 1.f; }
#pragma unroll
    for (int i = NSTEP - 1; i >= 0; --i) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            if (RET) {      // G = dZ + message from the next token; my message = gamma conj(e^{i theta}) G
                const float gmv = sigmoid_fast(gm[i][v] + rb[v]);
                gm[i][v] = gmv;
                Pth[v] *= gmv;
                const float gr_ = dzr[i][v] + Ebr[v], gi_ = dzi[i][v] + Ebi[v];
                Ebr[v] = gmv * __builtin_fmaf(lr[v], gr_, li[v] * gi_);
                Ebi[v] = gmv * __builtin_fmaf(lr[v], gi_, -li[v] * gr_);
            } else {
                const float nr = __builtin_fmaf(lr[v], Ebr[v], __builtin_fmaf(li[v], Ebi[v], dzr[i][v]));
                const float ni = __builtin_fmaf(lr[v], Ebi[v], __builtin_fmaf(-li[v], Ebr[v], dzi[i][v]));
                Ebr[v] = nr;
                Ebi[v] = ni;
            }
        }
    }
    // ---- the segments join in two levels: the two segments of a wave by a lane exchange, the waves
    //      through LDS (a run of tokens acts on what enters it from later tokens as X -> E + conj(lambda^n) X,
    //      RET: X -> E + (product of its retentions) conj(e^{i n theta}) X)
    const bool lower = !(seg & 1);          // my segment is the earlier one of my wave
    float Eor[V], Eoi[V], Po[V];            // aggregate (RET: and product) of my wave's other segment
#pragma unroll
    for (int v = 0; v < V; ++v) {
        Eor[v] = __shfl_xor(Ebr[v], 32, 64);
        Eoi[v] = __shfl_xor(Ebi[v], 32, 64);
        Po[v] = RET ? __shfl_xor(Pth[v], 32, 64) : 1.f;
    }
    if (lower) {        // the wave's aggregate: my segment after the later one
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float ar_, ai_;
            if (RET) {
                ar_ = __builtin_fmaf(Pth[v], __builtin_fmaf(pnr[v], Eor[v], pni[v] * Eoi[v]), Ebr[v]);
                ai_ = __builtin_fmaf(Pth[v], __builtin_fmaf(pnr[v], Eoi[v], -pni[v] * Eor[v]), Ebi[v]);
                sPb[wave][lv * V + v] = Pth[v] * Po[v];
            } else {
                ar_ = __builtin_fmaf(pnr[v], Eor[v], __builtin_fmaf(pni[v], Eoi[v], Ebr[v]));
                ai_ = __builtin_fmaf(pnr[v], Eoi[v], __builtin_fmaf(-pni[v], Eor[v], Ebi[v]));
            }
            sEb[wave][0][lv * V + v] = ar_;
            sEb[wave][1][lv * V + v] = ai_;
        }
    }
    lds_barrier_raw();     // the staged rows are still on their way
    BWD_STAMP(2);
    // (PF: the next tile must be known by the time its gradients are staged; asked for here, the answer
    // arrives with this wave's staged rows, which it waits for below anyway)
    if (PF && tid == 0)
        ticket_ahead = __hip_atomic_fetch_add(&a.hdr->ticket[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float Xr[V], Xi[V];     // adjoint entering my segment (from later segments), zero tile input
    float Cb[V];            // RET: product of the retentions of the segments after mine
    {
        float Yr[V], Yi[V], Cy[V], p2r[V], p2i[V];      // what enters my wave from the later waves; lambda^(2 NSTEP)
#pragma unroll
        for (int v = 0; v < V; ++v) {
            Yr[v] = Yi[v] = 0.f;
            Cy[v] = 1.f;
            p2r[v] = __builtin_fmaf(pnr[v], pnr[v], -pni[v] * pni[v]);
            p2i[v] = 2.0f * pnr[v] * pni[v];
        }
        for (int w = NW - 1; w > wave; --w) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float er = sEb[w][0][lv * V + v], ei = sEb[w][1][lv * V + v];
                float nr, ni;
                if (RET) {
                    const float pq = sPb[w][lv * V + v];
                    nr = __builtin_fmaf(pq, __builtin_fmaf(p2r[v], Yr[v], p2i[v] * Yi[v]), er);
                    ni = __builtin_fmaf(pq, __builtin_fmaf(p2r[v], Yi[v], -p2i[v] * Yr[v]), ei);
                    Cy[v] *= pq;
                } else {
                    nr = __builtin_fmaf(p2r[v], Yr[v], __builtin_fmaf(p2i[v], Yi[v], er));
                    ni = __builtin_fmaf(p2r[v], Yi[v], __builtin_fmaf(-p2i[v], Yr[v], ei));
                }
                Yr[v] = nr;
                Yi[v] = ni;
            }
        }
#pragma unroll
        for (int v = 0; v < V; ++v) {       // the later segment of my wave stands between the earlier one and that
            float lr_, li_;
            if (RET) {
                lr_ = __builtin_fmaf(Po[v], __builtin_fmaf(pnr[v], Yr[v], pni[v] * Yi[v]), Eor[v]);
                li_ = __builtin_fmaf(Po[v], __builtin_fmaf(pnr[v], Yi[v], -pni[v] * Yr[v]), Eoi[v]);
            } else {
                lr_ = __builtin_fmaf(pnr[v], Yr[v], __builtin_fmaf(pni[v], Yi[v], Eor[v]));
                li_ = __builtin_fmaf(pnr[v], Yi[v], __builtin_fmaf(-pni[v], Yr[v], Eoi[v]));
            }
            Xr[v] = lower ? lr_ : Yr[v];
            Xi[v] = lower ? li_ : Yi[v];
            Cb[v] = lower ? Po[v] * Cy[v] : Cy[v];
        }
    }

    // ---- chain, first half: the aggregate goes out before the front-end recompute
    const size_t slot = (size_t)ticket * 2 * JB + lv * V;
    if (head) {
        float Tr[V], Ti[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            if (RET) {
                Tr[v] = __builtin_fmaf(Pth[v], __builtin_fmaf(pnr[v], Xr[v], pni[v] * Xi[v]), Ebr[v]);
                Ti[v] = __builtin_fmaf(Pth[v], __builtin_fmaf(pnr[v], Xi[v], -pni[v] * Xr[v]), Ebi[v]);
                sPt[0][lv * V + v] = Cb[v] * Pth[v];
            } else {
                Tr[v] = __builtin_fmaf(pnr[v], Xr[v], __builtin_fmaf(pni[v], Xi[v], Ebr[v]));
                Ti[v] = __builtin_fmaf(pnr[v], Xi[v], __builtin_fmaf(-pni[v], Xr[v], Ebi[v]));
            }
            sCarry[0][lv * V + v] = Tr[v];     // parked here until the look-back (frees registers)
            sCarry[1][lv * V + v] = Ti[v];
        }
        if (chained && feeds) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                tagged_store(a.agg + slot + v, Tr[v], tag);
                tagged_store(a.agg + slot + JB + v, Ti[v], tag);
                if (RET) tagged_store(a.aggp + (size_t)ticket * JB + lv * V + v, Cb[v] * Pth[v], tag);
            }
        }
    }
    // the staged rows have landed (the head wave leaves the stores of its aggregate, its youngest
    // operations, in flight: their round trip is nobody's business here)
    if (wave == 0 && chained && feeds) wait_vm<(RET ? 3 : 2) * V>();
    else wait_stores_done();
    if (PF && tid == 0) sTicket[(it + 1) & 1] = ticket_ahead;
    lds_barrier();
    BWD_STAMP(3);

    // the constants of the reverse pass, fetched now so that they arrive during the front-end (the
    // valve kernels, at their register budget in the front-end, fetch them after it)
    // (written out twice rather than as a lambda called from two places: with the lambda the
    // compiler allocates scalar registers differently over the whole loop and spills 2.7x as many)
    float psr[V], psi[V], cth[V], sth[V], gam[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { sth[v] = gam[v] = 0.f; cth[v] = 1.f; }
    if (!PF) load_ckpt();
    if (!LEAN) {
        ldu<V>(psr, row(R_PSEGB + 2 * (NSEG - 1 - seg)), jb);    // adjoint: segments after mine
        ldu<V>(psi, row(R_PSEGB + 2 * (NSEG - 1 - seg) + 1), jb);
        if (PARAM) {
            ldu<V>(cth, row(R_COS), jb);
            ldu<V>(sth, row(R_SIN), jb);
            ldu<V>(gam, row(R_GAMMA), jb);
        }
    }
    // ---- front-end recompute, rows from LDS as a sliding window
    float cs[NSTEP][V], sn[NSTEP][V], ag[NSTEP][V], dsm[NSTEP][V];   // ag: a*g*SiLU'(z_ang)
    float am[VALVE ? NSTEP : 1][V];                                  // the amplitude itself (valve gradient)
    // lanes that share a valve: a head, or the part of it inside the 32-lane block (8, 16 or 32).
    // Where my tokens' entries start in sV / sVp is formed again at each use (from an opaque copy of
    // the thread index) rather than kept in a register across the tile.
    const int vwidth = (VALVE || RET) ? (a.F >= JB ? JB : a.F) : 1;
    auto valve_base = [&]() {
        int t_ = tid_;
        asm volatile("" : "+v"(t_));
        const int lv_ = t_ % LPR, seg_ = t_ / LPR;
        const int grp = vwidth == 32 ? 0 : (vwidth == 16 ? lv_ >> 4 : lv_ >> 3);
        return grp * TILE_T + seg_ * NSTEP;
    };
    float Spr[PARAM ? NSTEP : 1][V], Spi[PARAM ? NSTEP : 1][V];      // forward state before each token
    float Efr[V], Efi[V];

    const bool zero_hist = HALO > 0 && !tail_in && tt == 0 && seg == 0;   // rows before a sequence start
    // bf16: the carried conv history is fp32 and is not staged; the one segment that needs it reads it
    // where it uses it (and waits for it there, so that no wait for it lands in the common path)
    const bool hist_bf = BF && HALO > 0 && tail_in && tt == 0 && seg == 0;
    auto hist_row = [&](int k, int sidx) -> float {
        return tail_in[((size_t)(b * HALO + k) * 2 + sidx) * a.J + (active ? j0 : 0)];
    };
    // The mode switches are uniform over the launch; each combination gets its own straight-line
    // copy of the loop, so that the tokens' dependent chains (exp -> rcp -> sin/cos) interleave.
    ARGS_AGAIN();
    const GateSet gs_ = {a.gs.a1, a.gs.b1, a.gs.a2, a.gs.b2};
    auto front_end = [&](auto amp_c, auto small_c) {
        constexpr bool AMP = decltype(amp_c)::value, SMALL = decltype(small_c)::value;
        const int vbase = VALVE ? valve_base() : 0;
        float wnm[KC1][V], wna[KC1][V];
        // (row r of my segment lives in slot r % KC1: no register shuffling as the window slides)
#pragma unroll
        for (int k = 0; k < KC1 - 1; ++k) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                wnm[k % KC1][v] = zero_hist ? 0.f : su(seg * NSTEP + k, lv * V + v);
                wna[k % KC1][v] = zero_hist ? 0.f : su(NRTP + seg * NSTEP + k, lv * V + v);
            }
        }
        if (BF && hist_bf) {
#pragma unroll
            for (int k = 0; k < KC1 - 1; ++k) {
                wnm[k % KC1][0] = hist_row(k, 0);
                wna[k % KC1][0] = hist_row(k, 1);
            }
            wait_vm<0>();
        }
#pragma unroll
        for (int v = 0; v < V; ++v) { Efr[v] = kr[v]; Efi[v] = ki[v]; }      // the true state before my first token
#pragma unroll
        for (int i = 0; i < NSTEP; ++i) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                wnm[(i + HALO) % KC1][v] = su(seg * NSTEP + i + HALO, lv * V + v);
                wna[(i + HALO) % KC1][v] = su(NRTP + seg * NSTEP + i + HALO, lv * V + v);
            }
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float zm, xm, phi, km, ka;
                if (KC > 0) {
                    zm = bm[v];
                    float za = ba[v];
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        zm = __builtin_fmaf(wmf[k][v], wnm[(i + k) % KC1][v], zm);
                        za = __builtin_fmaf(waf[k][v], wna[(i + k) % KC1][v], za);
                    }
                    const float cm = clampf(zm, a.conv_clamp), ca = clampf(za, a.conv_clamp);
                    const float sgm = sigmoid_fast(cm), sga = sigmoid_fast(ca);
                    xm = cm * sgm;
                    phi = ca * sga;
                    // SiLU'(z) = sig (1 + z (1 - sig)) = sig + SiLU(z) (1 - sig); the clamp passes gradient only
                    // inside its range
                    km = __builtin_fabsf(zm) <= a.conv_clamp ? __builtin_fmaf(xm, 1.0f - sgm, sgm) : 0.0f;
                    ka = __builtin_fabsf(za) <= a.conv_clamp ? __builtin_fmaf(phi, 1.0f - sga, sga) : 0.0f;
                } else {
                    zm = wnm[i % KC1][v];
                    xm = zm;
                    phi = wna[i % KC1][v];
                    km = 1.0f;
                    ka = 1.0f;
                }
                float amp = xm;
                if (AMP) {
                    const float sp = softplus_fast(xm);
                    amp = __builtin_fminf(sp, 10.0f);
                    km *= sp < 10.0f ? sigmoid_fast(xm) : 0.0f;
                }
                // (the valve kernels keep the reduced angle, not its sin and cos: one register per
                // token-lane less, paid for with two hardware sin/cos in the reverse pass)
                const float rev = SMALL ? revolutions_small(phi) : revolutions_fast(phi);
                const float s = __builtin_amdgcn_sinf(rev), c = __builtin_amdgcn_cosf(rev);
                float agv;
                if (VALVE) {      // p = beta a e^{i phi}: beta multiplies both returned gradients
                    const float vl = sV[vbase + i];
                    const float beta = vl >= a.valve_thr ? sigmoid_fast(vl - 3.0f) : 0.0f;
                    agv = beta * amp;
                    km *= beta;
                    am[i][v] = amp;
                } else {
                    agv = in_gate(gs_, zm) ? amp : 0.0f;
                }
                cs[i][v] = LEAN ? rev : c;
                sn[i][v] = s;
                dsm[i][v] = km;
                ag[i][v] = agv * ka;
                if (PARAM) {   // forward scan from the checkpoint; the state before token i is kept
                    Spr[i][v] = Efr[v];
                    Spi[i][v] = Efi[v];
                    const float pr = agv * c, pi = agv * s;
                    float nr, ni;
                    if (RET) {
                        nr = __builtin_fmaf(gm[i][v], __builtin_fmaf(lr[v], Efr[v], -li[v] * Efi[v]), pr);
                        ni = __builtin_fmaf(gm[i][v], __builtin_fmaf(li[v], Efr[v], lr[v] * Efi[v]), pi);
                    } else {
                        nr = __builtin_fmaf(lr[v], Efr[v], __builtin_fmaf(-li[v], Efi[v], pr));
                        ni = __builtin_fmaf(li[v], Efr[v], __builtin_fmaf(lr[v], Efi[v], pi));
                    }
                    Efr[v] = nr;
                    Efi[v] = ni;
                }
            }
        }
    };
    {
        using T_ = std::true_type;
        using F_ = std::false_type;
        switch ((a.amp_mode ? 2 : 0) | (a.small_angle ? 1 : 0)) {
        case 0: front_end(F_{}, F_{}); break;
        case 1: front_end(F_{}, T_{}); break;
        case 2: front_end(T_{}, F_{}); break;
        default: front_end(T_{}, T_{}); break;
        }
    }
    float hacc[HC ? HC_PART_ROWS : 1];      // HC: tap gradient terms [plane][tap], then the biases' [plane]
#pragma unroll
    for (int q = 0; q < (HC ? HC_PART_ROWS : 1); ++q) hacc[q] = 0.f;
    if constexpr (HC) {
        // ---- the harmonic convolution's tap and bias terms, in a pass of its own (inside the front-end its
        //      temporaries came on top of the kernel's register peak): the state after token i is the state
        //      before token i+1; Z[t] = clamp(S[t]) meets the gradients at k+1, k, k-1 (taps 0, 1, 2)
        __builtin_amdgcn_sched_barrier(0);
        const HcLane hk = hc_setup();
        auto tap_pass = [&](auto full_c) {
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                const float sr_ = i + 1 < NSTEP ? Spr[i + 1 < NSTEP ? i + 1 : 0][0] : Efr[0];
                const float si_ = i + 1 < NSTEP ? Spi[i + 1 < NSTEP ? i + 1 : 0][0] : Efi[0];
                const float zr_ = clampf(sr_, a.out_clamp), zi_ = clampf(si_, a.out_clamp);
                float cr[3], ci[3];
                hc_read(full_c, i, hk, cr, ci);
#pragma unroll
                for (int q = 0; q < 3; ++q) {
                    hacc[q] = __builtin_fmaf(zr_, cr[2 - q], hacc[q]);
                    hacc[3 + q] = __builtin_fmaf(zi_, ci[2 - q], hacc[3 + q]);
                }
                hacc[6] += cr[1];
                hacc[7] += ci[1];
                // (the sums are used at the end of the tile only; left alone, the compiler moves the whole chain
                // down there and keeps all 48 gradients alive until then)
#pragma unroll
                for (int q = 0; q < HC_PART_ROWS; ++q) asm volatile("" : "+v"(hacc[q]));
            }
        };
        tap_pass(std::false_type{});      // (one copy of the pass: a second one for whole tiles costs more registers than its four selects per token)
        // a neighbour outside my head contributes nothing: tap 0 met the gradient at k+1, tap 2 the one at k-1
        hacc[0] = hk.last ? 0.f : hacc[0];
        hacc[3] = hk.last ? 0.f : hacc[3];
        hacc[2] = hk.first ? 0.f : hacc[2];
        hacc[5] = hk.first ? 0.f : hacc[5];
        __builtin_amdgcn_sched_barrier(0);
    }
    if (LEAN) {
        ldu<V>(psr, row(R_PSEGB + 2 * (NSEG - 1 - seg)), jb);
        ldu<V>(psi, row(R_PSEGB + 2 * (NSEG - 1 - seg) + 1), jb);
        if (PARAM && !RET) {      // (retention kernels: the table's lambda is e^{i theta} itself, and gamma is per token)
            ldu<V>(cth, row(R_COS), jb);
            ldu<V>(sth, row(R_SIN), jb);
            ldu<V>(gam, row(R_GAMMA), jb);
        }
    }

    // The reverse-pass constants must have arrived before the chain's stores below are issued: a
    // wave's memory operations complete in order, so a wait placed after those stores (where the
    // compiler would put it, at the first use) would also wait for the stores' round trip.
#pragma unroll
    for (int v = 0; v < V; ++v)
        asm volatile("" ::"v"(psr[v]), "v"(psi[v]), "v"(cth[v]), "v"(sth[v]), "v"(gam[v]));

    BWD_STAMP(5);
    ARGS_AGAIN();
    // ---- the next tile's upstream gradients start their way into sDz, issued by the waves that would
    //      otherwise only wait for the head wave's look-back.  From here to the end of the tile direct-to-LDS
    //      loads are in flight: every barrier is the raw one (the compiler makes a fence wait for such loads).
    //      (HC: the front-end reads this tile's staged gradients, so the next tile's start behind the barrier
    //      that closes it, below)
    auto stage_next = [&]() {
        const uint32_t nxt = (uint32_t)__builtin_amdgcn_readfirstlane((int)sTicket[(it + 1) & 1]);
        if (nxt < total_tiles_) {
            const int nlb = nxt % a.nLB, nrest = nxt / a.nLB;
            stage_dz(nrest % a.B, a.nT - 1 - nrest / a.B, nlb, wave - 1, NW - 1);
        }
    };
    if (PF && !HC && wave != 0) stage_next();
    // ---- chain, second half: look-back (its round trips were hidden behind the recompute above)
    if (head) {
        float cr[V], ci[V], Tr[V], Ti[V], hr[V], hi[V], qr[V], qi[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            cr[v] = ci[v] = hr[v] = hi[v] = qr[v] = qi[v] = 0.f;
            Tr[v] = sCarry[0][lv * V + v];
            Ti[v] = sCarry[1][lv * V + v];
        }
        ldu<V>(hr, row(R_PTB_HR), jb);      // lambda^TILE_T as a double-float
        ldu<V>(hi, row(R_PTB_HI), jb);
        ldu<V>(qr, row(R_PTB_LR), jb);
        ldu<V>(qi, row(R_PTB_LI), jb);
        if (chained) {
            if (!look_back<V, true, LPR, 1, RET>(a.agg, a.pre, ticket - chain_stride, chain_stride, ttr, JB, lv * V, lv,
                                                 hr, hi, qr, qi, a.spin_limit, tag, cr, ci, a.aggp)) {
                if (lv == 0) __hip_atomic_store(&a.hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // every load of this block has arrived before its stores go out (see above)
#pragma unroll
        for (int v = 0; v < V; ++v) asm volatile("" ::"v"(hr[v]), "v"(hi[v]), "v"(qr[v]), "v"(qi[v]));
#pragma unroll
        for (int v = 0; v < V; ++v) {
            sCarry[0][lv * V + v] = cr[v];
            sCarry[1][lv * V + v] = ci[v];
        }
        if (feeds) {    // P = T + conj(lambda^T) carry: the tile's inclusive prefix
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float P_r, P_i;
                const float pt = RET ? sPt[0][lv * V + v] : 1.f;
                chain_step<true>(Tr[v], Ti[v], hr[v], hi[v], qr[v], qi[v], RET ? pt * cr[v] : cr[v],
                                 RET ? pt * ci[v] : ci[v], P_r, P_i);
                tagged_store(a.pre + slot + v, P_r, tag);
                tagged_store(a.pre + slot + JB + v, P_i, tag);
            }
        }
    }
    if (wave == 0) __builtin_amdgcn_s_setprio(0);
    if (PF) lds_barrier_raw(); else lds_barrier();
    BWD_STAMP(6);
    if (PF && HC && wave != 0) stage_next();

    // ---- true adjoint entering my segment
    float Gr[V], Gi[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float cr = sCarry[0][lv * V + v], ci = sCarry[1][lv * V + v];
        if (RET) {          // the message entering my segment
            Gr[v] = __builtin_fmaf(Cb[v], __builtin_fmaf(psr[v], cr, psi[v] * ci), Xr[v]);
            Gi[v] = __builtin_fmaf(Cb[v], __builtin_fmaf(psr[v], ci, -psi[v] * cr), Xi[v]);
        } else {
            Gr[v] = __builtin_fmaf(psr[v], cr, __builtin_fmaf(psi[v], ci, Xr[v]));      // conj(ps) * carry
            Gi[v] = __builtin_fmaf(psr[v], ci, __builtin_fmaf(-psi[v], cr, Xi[v]));
        }
    }

    ARGS_AGAIN();
    // ---- reverse pass: adjoint, returned gradients, parameter terms
    float acc_g[V], acc_t[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc_g[v] = acc_t[v] = 0.f;
    const int vbase = (VALVE || RET) ? valve_base() : 0;
#pragma unroll
    for (int i = NSTEP - 1; i >= 0; --i) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float nr, ni;
            if (RET) {      // G = dZ + message; the message to the previous token takes my retention
                nr = dzr[i][v] + Gr[v];
                ni = dzi[i][v] + Gi[v];
                Gr[v] = gm[i][v] * __builtin_fmaf(lr[v], nr, li[v] * ni);
                Gi[v] = gm[i][v] * __builtin_fmaf(lr[v], ni, -li[v] * nr);
            } else {
                nr = __builtin_fmaf(lr[v], Gr[v], __builtin_fmaf(li[v], Gi[v], dzr[i][v]));
                ni = __builtin_fmaf(lr[v], Gi[v], __builtin_fmaf(-li[v], Gr[v], dzi[i][v]));
                Gr[v] = nr;
                Gi[v] = ni;
            }
            if (PARAM) {
                const float ct_ = RET ? lr[v] : cth[v], st_ = RET ? li[v] : sth[v];
                const float rr = __builtin_fmaf(ct_, Spr[i][v], -st_ * Spi[i][v]);
                const float ri = __builtin_fmaf(st_, Spr[i][v], ct_ * Spi[i][v]);
                const float tg = __builtin_fmaf(nr, rr, ni * ri);
                const float tth = (RET ? gm[i][v] : gam[v]) * __builtin_fmaf(ni, rr, -nr * ri);
                acc_g[v] += clampf(tg, a.grad_clamp);
                acc_t[v] += clampf(tth, a.grad_clamp);
                if (RET) {  // d gamma, clamped, through the sigmoid, summed over the lanes of the head
                    float wr = active ? clampf(tg, a.grad_clamp) * gm[i][v] * (1.0f - gm[i][v]) : 0.0f;
                    wr = head_sum(wr, vwidth);
                    if (head_sum_lane(lv, vwidth)) sRp[vbase + i] = wr;
                }
            }
            const float gr_ = clampf(nr, a.grad_clamp), gi_ = clampf(ni, a.grad_clamp);
            const float c_ = LEAN ? __builtin_amdgcn_cosf(cs[i][v]) : cs[i][v];
            const float s_ = LEAN ? __builtin_amdgcn_sinf(cs[i][v]) : sn[i][v];
            const float da = __builtin_fmaf(gr_, c_, gi_ * s_);
            const float dph = __builtin_fmaf(gi_, c_, -gr_ * s_);
            if (VALVE) {      // d/d beta, summed over the lanes that share the valve
                float wv = active ? am[i][v] * da : 0.0f;
                if (vwidth >= 16) {
                    // rotations within each row of 16 lanes leave the row's sum in all of its lanes
                    // (four full-rate adds); a 32-lane group then takes the lower row's sum into its
                    // upper row, whose lanes end up with the group's total
                    wv = dpp_add<0x128>(wv);
                    wv = dpp_add<0x124>(wv);
                    wv = dpp_add<0x122>(wv);
                    wv = dpp_add<0x121>(wv);
                    if (vwidth == 32) wv = dpp_add_bcast15(wv);
                    if (lv == vwidth - 16 || (vwidth == 16 && lv == 16)) sVp[vbase + i] = wv;
                } else {
#pragma unroll
                    for (int o = 4; o >= 1; o >>= 1)
                        if (o < vwidth) wv += __shfl_xor(wv, o, 64);
                    if (lv % vwidth == 0) sVp[vbase + i] = wv;
                }
            }
            dzr[i][v] = da * dsm[i][v];          // d/d(conv pre-activation), magnitude stream
            dzi[i][v] = dph * ag[i][v];          //                           angle stream
        }
        // (the valve kernels are at their register budget: keep the tokens' work from interleaving)
        if (VALVE || RET) __builtin_amdgcn_sched_barrier(0);
    }
    BWD_STAMP(7);
    // gradient of the incoming scan state: conj(lambda) G[0]
    if (a.dstate_in && tt == 0 && head && active) {
        float xr[V], xi[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            xr[v] = RET ? Gr[v] : __builtin_fmaf(lr[v], Gr[v], li[v] * Gi[v]);
            xi[v] = RET ? Gi[v] : __builtin_fmaf(lr[v], Gi[v], -li[v] * Gr[v]);
        }
        BVec<V>::st(a.dstate_in + ((size_t)b * 2 + 0) * a.J + j0, xr);
        BVec<V>::st(a.dstate_in + ((size_t)b * 2 + 1) * a.J + j0, xi);
    }

    ARGS_AGAIN();
    // the ticket of the next tile: asked for as late as its answer can still arrive unwaited-for, i.e.
    // ahead of this tile's output stores (a ticket held in reserve is a tile that has not started:
    // its successors in other workgroups wait for it)
    if (!PF && tid == 0)
        ticket_ahead = __hip_atomic_fetch_add(&a.hdr->ticket[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const size_t dbase = ((size_t)b * a.isb + (size_t)(tt * TILE_T) * a.ist + (size_t)lb * JB) * ES;
    float *omag = reinterpret_cast<float *>(reinterpret_cast<char *>(a.dmag) + dbase);
    float *oang = reinterpret_cast<float *>(reinterpret_cast<char *>(a.dang) + dbase);
    uint32_t ooff = ((uint32_t)(seg * NSTEP) * ist32 + (uint32_t)(lv * V)) * ES;      // bytes
    auto sto = [&](float *ub, uint32_t bo, const float (&x)[V]) {
        if constexpr (BF) *reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(ub) + bo) = to_bf16(x[0]);     // (half lines: default policy)
        else st_stream(reinterpret_cast<float *>(reinterpret_cast<char *>(ub) + bo), x[0]);
    };
    if (KC == 0) {
        if (full) {
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                sto(omag, ooff, dzr[i]);
                sto(oang, ooff, dzi[i]);
                ooff += ist32 * ES;
            }
            wait_vm<2 * NSTEP>();       // everything older than these stores has completed (the ticket, the next tile's staged gradients)
        } else {
#pragma unroll
            for (int i = 0; i < NSTEP; ++i) {
                if (active && t0 + i < a.L) {
                    sto(omag, ooff, dzr[i]);
                    sto(oang, ooff, dzi[i]);
                }
                ooff += ist32 * ES;
            }
            wait_vm<0>();
        }
    } else {
        // ---- transposed conv: du[t] = sum_k w[k] dz[t + (KC-1) - k]
        // (the valve kernels are at their register budget: their taps wait in LDS during the reverse
        // pass instead of in 2*KC registers)
        float wm[KC1][V], wa[KC1][V];
#pragma unroll
        for (int k = 0; k < KC; ++k)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                wm[k][v] = LEAN ? sTaps[k][lv * V + v] : wmf[k][v];
                wa[k][v] = LEAN ? sTaps[KC + k][lv * V + v] : waf[k][v];
            }
        // The transposed conv needs the conv pre-activation gradients of the HALO tokens after each
        // segment.  Inside the tile the earlier segment of a wave takes them from the later one by a lane
        // exchange, the later one from the next wave through LDS.  The tile's own first rows go to the
        // tile before it in time through the workspace (published by the head group, which holds them);
        // the tile's last segment takes the rows of the tile after it in time from there itself: only its
        // wave waits for them, and only in front of the segment's last HALO tokens.
        if (HALO > 0) {
            if (lower && wave > 0) {
#pragma unroll
                for (int r = 0; r < HALO; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        sHalo[wave][r][0][lv * V + v] = dzr[r][v];
                        sHalo[wave][r][1][lv * V + v] = dzi[r][v];
                    }
            }
            if (head && feeds) {
                tagged_t *hp = a.halo + (size_t)ticket * HALO * 2 * JB + lv * V;
#pragma unroll
                for (int r = 0; r < HALO; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        tagged_store(hp + (r * 2 + 0) * JB + v, dzr[r][v], tag);
                        tagged_store(hp + (r * 2 + 1) * JB + v, dzi[r][v], tag);
                    }
            }
        }
        const bool plain = full && !dtail_out;     // no per-row checks, no loads in the transposed conv
        const bool last_wave = wave == NW - 1;
        const bool want_rows = HALO > 0 && seg == NSEG - 1 && chained;
        const tagged_t *hin = a.halo + (size_t)(ticket - (chained ? chain_stride : 0u)) * HALO * 2 * JB + lv * V;
        tagged_t xw[HALO1][2][V];
#pragma unroll
        for (int r = 0; r < HALO1; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v) xw[r][0][v] = xw[r][1][v] = 0;
        auto ask_rows = [&]() {
#pragma unroll
            for (int r = 0; r < HALO; ++r)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    xw[r][0][v] = tagged_load(hin + (r * 2 + 0) * JB + v);
                    xw[r][1][v] = tagged_load(hin + (r * 2 + 1) * JB + v);
                }
        };
        if (want_rows) ask_rows();
        if (PF) lds_barrier_raw(); else lds_barrier();
    BWD_STAMP(8);
        float hm[HALO1][V], ha[HALO1][V];       // dz of the HALO tokens after my segment
#pragma unroll
        for (int r = 0; r < HALO1; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                // (the exchange runs in every lane: the later segment's lanes receive rows they do not use)
                const float xm_ = HALO > 0 ? __shfl_xor(dzr[r < HALO ? r : 0][v], 32, 64) : 0.f;
                const float xa_ = HALO > 0 ? __shfl_xor(dzi[r < HALO ? r : 0][v], 32, 64) : 0.f;
                const bool nextw = HALO > 0 && !lower && wave < NW - 1;
                hm[r][v] = lower ? xm_ : (nextw ? sHalo[nextw ? wave + 1 : 0][r][0][lv * V + v] : 0.f);
                ha[r][v] = lower ? xa_ : (nextw ? sHalo[nextw ? wave + 1 : 0][r][1][lv * V + v] : 0.f);
            }
        auto conv_t = [&](auto plain_c, auto lo_c, auto hi_c) {
            constexpr bool PLAIN = decltype(plain_c)::value;     // no per-row checks
            constexpr int I0 = decltype(lo_c)::value, I1 = decltype(hi_c)::value;
#pragma unroll
            for (int i = I0; i < I1; ++i) {
                const int t = t0 + i;
                float dm[V], da[V];
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float sm_ = 0.f, sa_ = 0.f;
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        const int idx = i + (KC - 1) - k;
                        const float zm_ = idx < NSTEP ? dzr[idx < NSTEP ? idx : 0][v] : hm[idx >= NSTEP ? idx - NSTEP : 0][v];
                        const float za_ = idx < NSTEP ? dzi[idx < NSTEP ? idx : 0][v] : ha[idx >= NSTEP ? idx - NSTEP : 0][v];
                        sm_ = __builtin_fmaf(wm[k][v], zm_, sm_);
                        sa_ = __builtin_fmaf(wa[k][v], za_, sa_);
                    }
                    dm[v] = sm_;
                    da[v] = sa_;
                }
                if (PLAIN) {
                    sto(omag, ooff, dm);
                    sto(oang, ooff, da);
                } else if (active && t < a.L) {
                    if (HALO > 0 && dtail_out && t >= a.L - HALO) {   // state_out's history rows are copies of these inputs
                        const int r = t - (a.L - HALO);
                        float xm_[V], xa_[V];
                        const size_t o = ((size_t)(b * HALO + r) * 2) * a.J + j0;
                        BVec<V>::ld(xm_, dtail_out + o);
                        BVec<V>::ld(xa_, dtail_out + o + a.J);
#pragma unroll
                        for (int v = 0; v < V; ++v) { dm[v] += xm_[v]; da[v] += xa_[v]; }
                    }
                    sto(omag, ooff, dm);
                    sto(oang, ooff, da);
                }
                ooff += ist32 * ES;
            }
        };
        using I_0 = std::integral_constant<int, 0>;
        using I_A = std::integral_constant<int, NSTEP - HALO>;
        using I_N = std::integral_constant<int, NSTEP>;
        // The rows asked for above, taken when they are needed.  The first look stands outside the polling
        // loop, and the whole of it inside each of the two paths below: the compiler places its own waits
        // for those loads from what it knows of a path, and where paths meet it knows the least.
        auto take_rows = [&]() {
            const int gshift = (int)(threadIdx.x & 63) - lv;
            const unsigned long long gmask = (1ull << LPR) - 1ull;
            auto all_tagged = [&]() {      // valid when every lane of the group found all its tags
                bool mine = true;
#pragma unroll
                for (int r = 0; r < HALO; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) mine = mine && tagged_ok(xw[r][0][v], tag) && tagged_ok(xw[r][1][v], tag);
                return ((__ballot(mine) >> gshift) & gmask) == gmask;
            };
            bool ok = all_tagged();
            for (uint32_t spins = 0; !ok && spins < a.spin_limit; ++spins) {
                __builtin_amdgcn_s_sleep(1);
                ask_rows();
                wait_vm<0>();
                ok = all_tagged();
            }
            if (ok) {
#pragma unroll
                for (int r = 0; r < HALO; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        hm[r][v] = tagged_value(xw[r][0][v]);
                        ha[r][v] = tagged_value(xw[r][1][v]);
                    }
            } else if (lv == 0) {
                __hip_atomic_store(&a.hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        };
        // The tokens that need no row beyond my segment come first; by then the rows asked for have arrived
        // (their round trip ran beside the barrier and those tokens).  Only the last wave waits, for
        // everything but the stores it has issued since.  Both paths end with every load complete, so that
        // no wait for one of them can land behind the output stores (where it would drain them); the stores
        // themselves stay in flight.
        if (plain) {
            conv_t(std::true_type{}, I_0{}, I_A{});
            if (HALO > 0 && last_wave && chained) {
                wait_vm<2 * (NSTEP - HALO) * V>();
                if (want_rows) take_rows();
            }
            conv_t(std::true_type{}, I_A{}, I_N{});
            wait_vm<(2 * NSTEP < 63 ? 2 * NSTEP : 63)>();
        } else {
            conv_t(std::false_type{}, I_0{}, I_A{});
            if (HALO > 0 && last_wave && chained) {
                wait_vm<0>();
                if (want_rows) take_rows();
            }
            conv_t(std::false_type{}, I_A{}, I_N{});
            wait_vm<0>();
        }
        // gradient of the incoming conv history: rows r <-> time r - HALO
        if (HALO > 0 && a.dstate_in && tt == 0 && head && active) {
            float *dtail_in = a.dstate_in + (size_t)a.B * 2 * a.J;
#pragma unroll
            for (int r = 0; r < HALO; ++r) {
                float dm[V], da[V];
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float sm_ = 0.f, sa_ = 0.f;
#pragma unroll
                    for (int k = 0; k <= r; ++k) {
                        sm_ = __builtin_fmaf(wm[k][v], dzr[r - k][v], sm_);
                        sa_ = __builtin_fmaf(wa[k][v], dzi[r - k][v], sa_);
                    }
                    dm[v] = sm_;
                    da[v] = sa_;
                }
                const int rs = r - a.L;                    // history row that state_out copied straight from state_in
                if (dtail_out && rs >= 0) {
                    float xm_[V], xa_[V];
                    const size_t o = ((size_t)(b * HALO + rs) * 2) * a.J + j0;
                    BVec<V>::ld(xm_, dtail_out + o);
                    BVec<V>::ld(xa_, dtail_out + o + a.J);
#pragma unroll
                    for (int v = 0; v < V; ++v) { dm[v] += xm_[v]; da[v] += xa_[v]; }
                }
                const size_t o = ((size_t)(b * HALO + r) * 2) * a.J + j0;
                BVec<V>::st(dtail_in + o, dm);
                BVec<V>::st(dtail_in + o + a.J, da);
            }
        }
    }

    ARGS_AGAIN();
    // ---- parameter partials: my tokens, then the wave's two segments, then the waves in order
    if (PARAM) {
        float part[ROWS][V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            part[0][v] = acc_g[v];
            part[1][v] = acc_t[v];
#pragma unroll
            for (int r = 2; r < ROWS; ++r) part[r][v] = 0.f;
        }
        if (KC > 0) {
            const bool zero_hist = HALO > 0 && !tail_in && tt == 0 && seg == 0;
            float hm_[HALO1], ha_[HALO1];       // bf16: the fp32 history rows again (first segment of a call with history)
#pragma unroll
            for (int k = 0; k < HALO1; ++k) hm_[k] = ha_[k] = 0.f;
            if (BF && hist_bf) {
#pragma unroll
                for (int k = 0; k < HALO; ++k) {
                    hm_[k] = hist_row(k, 0);
                    ha_[k] = hist_row(k, 1);
                }
                wait_vm<0>();
            }
#pragma unroll
            for (int i = 0; i < NSTEP; ++i)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    part[2][v] += dzr[i][v];
                    part[3][v] += dzi[i][v];
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        const bool z = zero_hist && (i + k < HALO);
                        const bool hrow = BF && hist_bf && (i + k < HALO);
                        const float um_ = z ? 0.f : (hrow ? hm_[i + k < HALO ? i + k : 0] : su(seg * NSTEP + i + k, lv * V + v));
                        const float ua_ = z ? 0.f : (hrow ? ha_[i + k < HALO ? i + k : 0] : su(NRTP + seg * NSTEP + i + k, lv * V + v));
                        part[4 + k][v] = __builtin_fmaf(dzr[i][v], um_, part[4 + k][v]);
                        part[4 + KC + k][v] = __builtin_fmaf(dzi[i][v], ua_, part[4 + KC + k][v]);
                    }
                }
        }
        if constexpr (HC) {
#pragma unroll
            for (int q = 0; q < HC_PART_ROWS; ++q) part[4 + 2 * KC + q][0] = hacc[q];
        }
        if (PF) lds_barrier_raw();      // the staging below lies over the input rows: everybody has read them
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float other = __shfl_xor(part[r][v], 32, 64);    // the wave's other segment
                const float s = (seg & 1) ? other + part[r][v] : part[r][v] + other;
                if (!(seg & 1)) sRed[wave][r][lv * V + v] = s;
            }
        if (PF) lds_barrier_raw(); else lds_barrier();
    BWD_STAMP(9);
        for (int e = tid; e < ROWS * JB; e += NT) {
            const int row = e / JB, c = e % JB;
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += sRed[w][row][c];
            a.part[((size_t)ticket * ROWS + row) * JB + c] = s;
        }
    }

    // ---- the valve's gradient terms of the tile go out, token-contiguous per group
    if (VALVE && a.vpart) {
        lds_barrier();
        for (int e = tid; e < a.gpb * TILE_T; e += NT) {
            const int g = e / TILE_T, tok = e - g * TILE_T;
            const int t = tt * TILE_T + tok, grp = lb * a.gpb + g;
            if (t < a.L && grp < a.G) a.vpart[((size_t)b * a.G + grp) * a.L + t] = sVp[e];
        }
    }
    // ---- and the retention logits' in the same layout
    if (RET && a.rpart) {
        if (!(VALVE && a.vpart)) lds_barrier();
        for (int e = tid; e < a.gpb * TILE_T; e += NT) {
            const int g = e / TILE_T, tok = e - g * TILE_T;
            const int t = tt * TILE_T + tok, grp = lb * a.gpb + g;
            if (t < a.L && grp < a.G) a.rpart[((size_t)b * a.G + grp) * a.L + t] = sRp[e];
        }
    }

    // ---- LDS is reused by the next tile.  The ticket asked for above is parked where this tile's was
    //      (everything older than the output stores has completed: no further wait)
    if (!PF && tid == 0) sTicket[(it + 1) & 1] = ticket_ahead;
    if (PF) lds_barrier_raw(); else lds_barrier();
    BWD_STAMP(10);
    ticket = (uint32_t)__builtin_amdgcn_readfirstlane((int)sTicket[(it + 1) & 1]);
#undef a
#undef ARGS_AGAIN
    }

    // ---- the workgroup that leaves last resets the ticket and advances the epoch for the next call.
    //      Workgroups are counted, not tiles: every one of the grid has then drawn its last ticket.
    if (tid_ == 0) {
        const uint32_t old = __hip_atomic_fetch_add(&a.hdr->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sLast = (old + 1 == gridDim.x) ? 1u : 0u;
    }
    __syncthreads();
    if (sLast) finish_call(a.hdr, a.clear_from, epoch, tid_, blockDim.x);
}

// Persistent grid: what fits on the chip at once (asked once per kernel), never more than tiles.
template <int V, int KC, bool PARAM, bool VALVE, bool RET, bool BF, bool HC = false>
static hipError_t launch_bwd_vkp(const BwdArgs &a, hipStream_t s)
{
    static int per_cu = 0, cus = 0;
    if (per_cu == 0) {
        int dev = 0, n = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorUnknown;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, bwd_kernel<V, KC, PARAM, VALVE, RET, BF, HC>, BwdGeom::NSEG * BwdLPR, 0) != hipSuccess)
            return hipErrorUnknown;
        cus = prop.multiProcessorCount;
        per_cu = n > 0 ? n : 1;
    }
    long long g = (long long)per_cu * cus;
    if (g > (long long)a.total_tiles) g = a.total_tiles;
    hipLaunchKernelGGL((bwd_kernel<V, KC, PARAM, VALVE, RET, BF, HC>), dim3((unsigned)g), dim3(BwdGeom::NSEG * BwdLPR), 0, s, a);
    return hipGetLastError();
}

// The kernels of one family (gate mode x retention mode x harmonic convolution), one per conv_k.  Each family
// is instantiated in a translation unit of its own, so that the families compile side by side.
// Tuning aid: -DCAWN_DEV_KC=<k> compiles only the conv_k = k kernels and -DCAWN_DEV_PLAIN only the
// threshold-mode fp32 ones (a build for timing one variant in seconds; every other variant then
// fails to launch with hipErrorInvalidValue).  The library is always built without them.
template <bool PARAM, bool VALVE, bool RET, bool BF, bool HC>
static hipError_t launch_bwd_family(const BwdArgs &a, int conv_k, hipStream_t s)
{
#ifdef CAWN_DEV_PLAIN
    if constexpr (VALVE || RET || BF) return hipErrorInvalidValue; else
#endif
    switch (conv_k) {
#ifdef CAWN_DEV_KC
    case CAWN_DEV_KC: return launch_bwd_vkp<1, CAWN_DEV_KC, PARAM, VALVE, RET, BF, HC>(a, s);
#else
    case 0: return launch_bwd_vkp<1, 0, PARAM, VALVE, RET, BF, HC>(a, s);
    case 1: return launch_bwd_vkp<1, 1, PARAM, VALVE, RET, BF, HC>(a, s);
    case 2: return launch_bwd_vkp<1, 2, PARAM, VALVE, RET, BF, HC>(a, s);
    case 3: return launch_bwd_vkp<1, 3, PARAM, VALVE, RET, BF, HC>(a, s);
    case 4: return launch_bwd_vkp<1, 4, PARAM, VALVE, RET, BF, HC>(a, s);
#endif
    default: return hipErrorInvalidValue;
    }
}
// ... with the activation type chosen at run time
template <bool PARAM, bool VALVE, bool RET, bool HC>
static hipError_t launch_bwd_family_act(const BwdArgs &a, int conv_k, hipStream_t s)
{
    return a.bf16 ? launch_bwd_family<PARAM, VALVE, RET, true, HC>(a, conv_k, s)
                  : launch_bwd_family<PARAM, VALVE, RET, false, HC>(a, conv_k, s);
}

// the families' launchers, one translation unit each
hipError_t launch_bwd_plain(const BwdArgs &a, int conv_k, hipStream_t s);    // threshold gate, constant retention
hipError_t launch_bwd_valve(const BwdArgs &a, int conv_k, hipStream_t s);    // per-head valve, constant retention
hipError_t launch_bwd_ret(const BwdArgs &a, int conv_k, hipStream_t s);      // data-dependent retention, either gate
hipError_t launch_bwd_hconv(const BwdArgs &a, int conv_k, hipStream_t s);    // harmonic convolution, threshold gate
hipError_t launch_bwd_hconv_valve(const BwdArgs &a, int conv_k, hipStream_t s);    // ... per-head valve
hipError_t launch_bwd_hconv_ret(const BwdArgs &a, int conv_k, hipStream_t s);      // ... data-dependent retention, either gate

}  // namespace cawn
