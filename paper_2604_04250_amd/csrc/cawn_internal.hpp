// Internal definitions shared by the libcawn translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cawn.h"
#include "cawn_gate_host.hpp"

namespace cawn {

// ------------------------------------------------------------------------------------ geometry
// One tile = JB lanes x TILE_T tokens of one batch row, processed by one workgroup at a time.  A
// thread owns V adjacent lanes and NSTEP consecutive tokens ("segment"); NSEG segments make the
// tile.  The two kernels pick their own shape:
//   forward : long tiles.  Its tiles of one chain are joined by memory round trips, so the fewer
//             tiles a chain has the better; it keeps only 2 values per token-lane in registers,
//             which allows 32 tokens per thread.
//   backward: keeps ~10 values per token-lane, hence 8 tokens per thread and one lane per thread
//             (4 waves per SIMD).
// Checkpoints of the scan state are kept every CKPT_T tokens = one backward segment: a backward
// thread starts the forward state of its tokens from the checkpoint of its own segment (one more
// byte per token-lane each way; without it every tile had to join its segments' states in LDS).
#ifndef CAWN_FWD_TILE_T
#define CAWN_FWD_TILE_T 256
#endif
#ifndef CAWN_FWD_NSTEP
#define CAWN_FWD_NSTEP 32
#endif
#ifndef CAWN_FWD_V
#define CAWN_FWD_V 1
#endif
#ifndef CAWN_FWD_LPR
#define CAWN_FWD_LPR 32
#endif
#ifndef CAWN_BWD_TILE_T
#define CAWN_BWD_TILE_T 128
#endif
#ifndef CAWN_BWD_NSTEP
#define CAWN_BWD_NSTEP 8
#endif
#ifndef CAWN_BWD_V
#define CAWN_BWD_V 1
#endif
#ifndef CAWN_BWD_LPR
#define CAWN_BWD_LPR 32
#endif
#ifndef CAWN_FWD_WAVES
#define CAWN_FWD_WAVES 2      // waves per SIMD the forward kernel's register budget is set for
#endif
#ifndef CAWN_BWD_WAVES
#define CAWN_BWD_WAVES 4
#endif
struct FwdGeom {
    static constexpr int TILE_T = CAWN_FWD_TILE_T, NSTEP = CAWN_FWD_NSTEP, NSEG = TILE_T / NSTEP;
};
struct BwdGeom {
    static constexpr int TILE_T = CAWN_BWD_TILE_T, NSTEP = CAWN_BWD_NSTEP, NSEG = TILE_T / NSTEP;
};
constexpr int CKPT_T = BwdGeom::NSTEP;
static_assert(FwdGeom::NSTEP % CKPT_T == 0, "a forward segment spans whole checkpoint intervals");
static_assert(BwdGeom::TILE_T % CKPT_T == 0, "backward tiles start on checkpoints");
constexpr int FwdV = CAWN_FWD_V, FwdLPR = CAWN_FWD_LPR;  // lanes per thread, threads per row
constexpr int BwdV = CAWN_BWD_V, BwdLPR = CAWN_BWD_LPR;
constexpr int MAX_KC = 4;
constexpr uint32_t MAX_TILES = 1u << 18;   // most tiles one call may have (tile indices, tickets)

// ---------------------------------------------------------------------------------- lane table
// Per-lane constants, struct-of-arrays, each row Jp floats (Jp = J rounded up to 64), built in
// fp64 by a small kernel from gamma, theta, conv_w, conv_b.
enum LaneRow : int {
    R_COS = 0, R_SIN, R_GAMMA, // e^{i theta}, gamma
    R_PT_HR, R_PT_HI,          // lambda^(forward TILE_T), leading fp32 part
    R_PT_LR, R_PT_LI,          //                          remainder (double-float)
    R_PTB_HR, R_PTB_HI,        // the same for the backward tile length
    R_PTB_LR, R_PTB_LI,
    R_PSEGB,                   // R_PSEGB + 2*s (+1): re (im) of lambda^(NSTEP*s), backward segments
    // The rows below are what a forward tile's threads keep in registers; they are contiguous so
    // that a tile stages them in LDS with a few wide loads (R_LR .. R_W0 + 2*conv_k - 1).
    R_LR = R_PSEGB + 2 * BwdGeom::NSEG, R_LI,   // lambda = gamma e^{i theta}
    R_PSEG,                    // R_PSEG + 2*s (+1): the same powers for the forward segments
    R_BIAS_M = R_PSEG + 2 * FwdGeom::NSEG, R_BIAS_A,
    R_RBIAS,                   // ret_mode 1: the lane's static retention bias b_k (k = j mod F)
    R_W0                       // R_W0 + s*conv_k + i : tap i of stream s
};
// Harmonic convolution (Sec. 3.6): HC_ROWS more rows behind the temporal conv's taps, per lane the
// constants of its head's two channels: R_W0 + 2*conv_k + 3*plane + i = tap i, + 6 + plane = bias.
constexpr int HC_ROWS = 8;
inline __host__ __device__ int lane_rows(int conv_k, bool hconv = false) { return R_W0 + 2 * conv_k + (hconv ? HC_ROWS : 0); }

// ----------------------------------------------------------------------------------- workspace
// Workspace: [header 1 KiB][lane table][aggregates][prefixes][backward conv halo][backward parameter
// partials].  Everything tiles publish to each other (aggregates, prefixes, halo rows) is stored as
// 8-byte words {value, tag}: the tag is make_tag(epoch of the call), so a word is valid exactly
// when its tag matches -- no separate status words, no ordering between stores, one memory round trip
// from publication to use.  Words left by earlier calls (whatever their descriptor) carry other tags
// and read as "not published"; cawn_workspace_init zeroes the whole buffer (a zero word is never a tag).
// Region offsets depend on the descriptor, so a call may find fp32 data of an earlier call with another
// descriptor (lane-table rows, partial sums) where it expects published words.  Tags are therefore the
// bit patterns of negative NaNs with a non-zero payload (0xFF800001 .. 0xFFFFFFFF): no finite value,
// infinity or hardware-made NaN (0x7FC00000) an fp32 computation leaves behind equals one.
// Nothing is cleared per tile or per call: the workgroup that leaves last resets the tickets and
// advances the epoch.
constexpr int MAX_QUEUES = 64;
struct WsHeader {
    uint32_t ticket[MAX_QUEUES];   // ticket[0]: next tile to hand out (the other words are spare)
    uint32_t done;                 // tiles finished
    uint32_t error;                // sticky: a tile gave up waiting
    uint32_t epoch;                // calls completed on this workspace (mod EPOCH_MOD): make_tag() of it marks published words
    uint32_t bytes_lo, bytes_hi;   // size given to cawn_workspace_init (what an epoch wrap has to clear)
    uint32_t pad[256 - MAX_QUEUES - 5];
};
static_assert(sizeof(WsHeader) == 1024, "header size");

struct WsLayout {
    int J, Jp, Jp128, nT, nTc;     // nT: backward tiles per sequence, nTc: checkpoint intervals
    size_t off_table, off_agg, off_pre, off_halo, off_part, off_vpart, off_aggp, off_rpart, off_hpart, off_dbg, total;
};

constexpr uint32_t EPOCH_MOD = (1u << 23) - 1u;     // epochs 0 .. 2^23 - 2
typedef unsigned long long tagged_t;     // {fp32 value (low half), tag (high half)}
inline __host__ __device__ uint32_t make_tag(uint32_t epoch) { return 0xFF800001u + epoch; }

// (GateSet, the gate as a union of two closed fp32 intervals, comes from cawn_gate_host.hpp)

struct FwdArgs {
    const float *mag, *ang;
    const float *table;          // lane table
    const float *state_in;       // may be null
    float *z_re, *z_im;
    float *state_out;            // may be null
    float *ckpt;                 // may be null
    uint32_t *mask;              // may be null
    WsHeader *hdr;
    tagged_t *agg, *pre;
    int B, L, J, Jp, nT, nLB;    // nT: forward tiles per sequence
    int nTc;                     // checkpoint intervals per sequence
    int stage16;                 // input rows may be staged with 16-byte loads (alignment, J % 4 == 0)
    int amp_mode;
    int small_angle;             // angles are bounded (conv clamp): skip the two-term range reduction
    long long isb, ist, osb, ost;
    float conv_clamp, out_clamp;
    GateSet gs;
    uint32_t spin_limit;
    uint32_t total_tiles;
    size_t clear_from;           // byte offset of the first published word (cleared when the epoch wraps)
    unsigned long long *dbg;     // -DCAWN_TIMING builds only
    // (kept behind everything else: the kernels that do not use them fetch none of this)
    // gate_mode 1 (per-head input valve, Sec. 3.3): logits [B][L][H]; a lane block of 32 lanes
    // holds gpb = max(1, 32 / F) heads (groups); the valve is open when the logit >= valve_thr
    const float *valve;          // null: gate_mode 0
    int H, F, gpb;
    float valve_thr;
    // ret_mode 1 (data-dependent retention, Sec. 3.3 item 4): logits [B][L][H], staged like the valve's;
    // the lane table is then built with gamma = 1 (its powers are pure rotations) and a tile's
    // aggregate has a third chained word, the product of the tile's retentions: aggp [tile][JB]
    const float *ret;            // null: ret_mode 0
    tagged_t *aggp;
    // activations are bfloat16 in memory (mag, ang, z_re, z_im then point to 2-byte elements; strides
    // are in elements); J and the strides are even
    int bf16;
    // harmonic convolution of the output before it is stored (Sec. 3.6, three taps); hcG: 32-lane blocks
    // per head (1 when a head fits a block), whose tickets one workgroup draws together
    int hconv, hcG;
};

struct BwdArgs {
    const float *mag, *ang, *dz_re, *dz_im;
    const float *table;
    const float *state_in;       // may be null
    const float *ckpt;           // may be null when no dgamma/dtheta
    const float *dstate_out;     // may be null
    float *dmag, *dang;
    float *dstate_in;            // may be null
    WsHeader *hdr;
    tagged_t *agg, *pre, *halo;
    float *part;
    int B, L, J, Jp, nT, nLB;
    int nTc;                     // checkpoint intervals per sequence
    int small_angle;
    int stage16;                 // input rows may be staged with 16-byte loads (alignment, J % 4 == 0)
    int stage16z;                // the same for the upstream-gradient rows
    int amp_mode, want_param;
    long long isb, ist, osb, ost;
    float conv_clamp, grad_clamp;
    GateSet gs;
    uint32_t spin_limit;
    uint32_t total_tiles;
    size_t clear_from;           // byte offset of the first published word (cleared when the epoch wraps)
    unsigned long long *dbg;     // -DCAWN_TIMING builds only
    // (kept behind everything else: the kernels that do not use them fetch none of this)
    // gate_mode 1 (per-head input valve): see FwdArgs; vpart [B][G][L] receives, per valve group
    // (a head, or the 32-lane slice of a head) and token, the sum over the group's lanes of
    // a Re(conj(dp) e^{i phi}); G groups per token
    const float *valve;          // null: gate_mode 0
    float *vpart;                // null: no valve gradient wanted
    int H, F, gpb, G;
    float valve_thr;
    // ret_mode 1 (data-dependent retention): see FwdArgs; rpart like vpart, for the retention logits
    const float *ret;            // null: ret_mode 0
    float *rpart;                // null: no gradient of the retention logits wanted
    tagged_t *aggp;
    int bf16;                    // activations (mag, ang, dz_*, dmag, dang) are bfloat16 in memory: see FwdArgs
    // harmonic convolution behind the output clamp (Sec. 3.6): dz_re / dz_im are then the gradients of the
    // CONVOLVED output; the kernel applies the transposed convolution as it reads them and emits, per lane,
    // the terms of the tap and bias gradients (rows behind the conv front-end's in `part`)
    int hconv;
    float out_clamp;
};

// Number of per-lane partial sums a backward tile emits: dgamma, dtheta, dbias[2], dw[2][conv_k]; with the
// harmonic convolution 8 more: its taps' terms [2 planes][3], then its biases' [2 planes].
constexpr int HC_PART_ROWS = 8;
inline __host__ __device__ int part_rows(int conv_k, bool hconv = false) { return 4 + 2 * conv_k + (hconv ? HC_PART_ROWS : 0); }

hipError_t launch_fwd(const FwdArgs &a, int conv_k, bool vec4, hipStream_t s);
hipError_t launch_bwd(const BwdArgs &a, int conv_k, bool vec, hipStream_t s);

#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC__)
// ------------------------------------------------------------------------------ device helpers
__device__ __forceinline__ float clampf(float v, float c) { return __builtin_amdgcn_fmed3f(v, -c, c); }

// Streamed data -- the activations a call reads once and the outputs it writes once -- moves with the
// non-temporal cache policy: it does not displace what is read again (lane table, published words, halo rows,
// and the checkpoints, which the backward of the same step reads back: those keep the default policy).
// Measured on the training-step shape: backward 275 -> 258 us, a 4096-token chunk 25.3 -> 23.5 us.
__device__ __forceinline__ void st_stream(float *p, float v) { __builtin_nontemporal_store(v, p); }
constexpr int DMA_STREAM = 2;      // cache-policy operand of the direct-to-LDS loads of staged rows: nt

// bfloat16 in memory: the upper half of an fp32; to bf16 with the hardware's round-to-nearest-even.
__device__ __forceinline__ float from_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t to_bf16(float x)
{
    const __bf16 h = (__bf16)x;
    return __builtin_bit_cast(uint16_t, h);
}

// sigmoid(z) with the hardware exp2 / reciprocal (both ~1 ulp).
__device__ __forceinline__ float sigmoid_fast(float z)
{
    float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * z);
    return __builtin_amdgcn_rcpf(1.0f + e);
}

// sin and cos of an angle in radians: two-term Cody-Waite reduction to [-pi, pi] (exact products
// through fma), then the hardware sin/cos, which take revolutions.
__device__ __forceinline__ void sincos_fast(float phi, float &s, float &c)
{
    const float INV_2PI = 0.15915494309189535f;
    const float TWO_PI_HI = 6.2831854820251465f;      // fp32(2 pi)
    const float TWO_PI_LO = -1.7484555314695172e-07f; // 2 pi - TWO_PI_HI
    float k = __builtin_rintf(phi * INV_2PI);
    float r = __builtin_fmaf(-k, TWO_PI_HI, phi);
    r = __builtin_fmaf(-k, TWO_PI_LO, r);
    float x = r * INV_2PI;
    s = __builtin_amdgcn_sinf(x);
    c = __builtin_amdgcn_cosf(x);
}

// Same, for angles known to be small (a few revolutions): the hardware reduces the range itself.
__device__ __forceinline__ void sincos_small(float phi, float &s, float &c)
{
    const float x = phi * 0.15915494309189535f;
    s = __builtin_amdgcn_sinf(x);
    c = __builtin_amdgcn_cosf(x);
}
// The reduced angle in revolutions those two hand to the hardware (a caller short of registers
// keeps this one value and asks the hardware for sin and cos again).
__device__ __forceinline__ float revolutions_fast(float phi)
{
    const float INV_2PI = 0.15915494309189535f;
    const float TWO_PI_HI = 6.2831854820251465f;
    const float TWO_PI_LO = -1.7484555314695172e-07f;
    float k = __builtin_rintf(phi * INV_2PI);
    float r = __builtin_fmaf(-k, TWO_PI_HI, phi);
    r = __builtin_fmaf(-k, TWO_PI_LO, r);
    return r * INV_2PI;
}
__device__ __forceinline__ float revolutions_small(float phi) { return phi * 0.15915494309189535f; }

__device__ __forceinline__ float softplus_fast(float m)
{
    // log(1 + e^m) = max(m, 0) + log(1 + e^-|m|)
    float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * __builtin_fabsf(m));
    return __builtin_fmaxf(m, 0.0f) + 0.6931471805599453f * __builtin_amdgcn_logf(1.0f + e);
}

__device__ __forceinline__ bool in_gate(const GateSet &g, float x)
{
    // bitwise on purpose: short-circuit forms compile to divergent branches
    return (bool)(((int)(x >= g.a1) & (int)(x <= g.b1)) | ((int)(x >= g.a2) & (int)(x <= g.b2)));
}

// Cross-tile publication.  Tiles of one chain may run on different XCDs, whose L2 caches are not
// coherent with each other.  Payload and status words therefore move with agent-scope relaxed
// atomics (sc1 accesses, which go to the memory-side coherence point), and ordering is by waiting
// for the stores to complete (vmcnt) before the status word is written.  Acquire/release atomics
// are avoided on purpose: at agent scope they write back / invalidate the whole L2 on every use,
// which a spin loop next to streaming stores cannot afford.
__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }
// Wait until at most N of this wave's vector memory operations are outstanding.  They complete in
// issue order (loads, stores and direct-to-LDS loads alike), so this waits for everything except
// the N youngest.  The builtin (not inline assembly) lets the compiler's own wait insertion see it.
template <int N>
__device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    compiler_fence();
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);   // expcnt, lgkmcnt: no wait
    compiler_fence();
}
__device__ __forceinline__ void wait_stores_done() { wait_vm<0>(); }
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding
// global load and store of every wave, which would serialise a tile's output stores and the next
// tile's staging loads with the barrier; global data here is never exchanged inside a workgroup.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
// The same barrier for a point where direct-to-LDS loads are still in flight: there the compiler
// makes the fences above wait for those loads.  Hardware barrier only; LDS accesses of this wave
// are waited for explicitly and the compiler may not move memory accesses across.
__device__ __forceinline__ void lds_barrier_raw()
{
    compiler_fence();
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0); vmcnt, expcnt: no wait
    __builtin_amdgcn_s_barrier();
    compiler_fence();
}

// Stage the pre-conv input rows of one tile in LDS with direct global->LDS loads (no registers):
// rows tile_t0-HALO .. tile_t0+TT-1 of the magnitude stream, then the same rows of the angle
// stream, JB lanes each, row-major; each stream occupies staged_rows<TT, JB, HALO>() rows (padded
// to whole load instructions).  Called by `nwaves` waves (index `wave` among them).  Rows outside
// [0, L) and lanes beyond J read a clamped (valid) address: their values never reach a result (the
// scan is causal, a lane only reads its own LDS column; rows before a sequence start are zeroed at
// the point of use).  Rows before the call's first token come from the carried conv history when
// there is one.  LB: bytes per lane per load (16 needs 16-byte aligned rows).
template <int TT, int JB, int HALO>
__host__ __device__ constexpr int staged_rows()
{
    constexpr int g = 256 / JB > 0 ? 256 / JB : 1;      // rows per instruction of the widest load
    return (TT + HALO + g - 1) / g * g;
}
template <int TT, int JB, int HALO, int LB>
__device__ __forceinline__ void stage_rows(float *sU, const float *mag, const float *ang, const float *tail_in,
                                           int b, int tile_t0, int lb, int J, int L, long long isb, int ist,
                                           int wave, int nwaves, int lane)
{
    constexpr int NRT = TT + HALO;
    // rows whose segment fills a 128-byte line are streamed; half lines (bf16) keep the default policy, so that
    // the cache can serve the neighbouring lane block's half of the line
    [[maybe_unused]] constexpr int POL = JB * 4 >= 128 ? DMA_STREAM : 0;
    constexpr int NRTP = staged_rows<TT, JB, HALO>();
    constexpr int LR = JB * 4 / LB;                // lanes per row
    if constexpr (LR <= 64) {
        constexpr int RPI = 64 / LR;               // rows per wave instruction
        static_assert(NRTP % RPI == 0, "a stream is a whole number of load instructions");
        constexpr int NIS = NRTP / RPI;            // instructions per stream
        const int t_first = tile_t0 - HALO;
        // wave-uniform bases of the two streams at the first staged row
        const float *base_m = mag + (size_t)b * isb + (long long)t_first * ist;
        const float *base_a = ang + (size_t)b * isb + (long long)t_first * ist;
        const int r_in = lane / LR, c_in = (lane % LR) * (LB / 4);      // my row within an instruction, my lane
        if (t_first >= 0 && t_first + NRT <= L && (lb + 1) * JB <= J) {
            // every staged row exists: uniform base + one per-lane byte offset
            const uint32_t loff = (uint32_t)(r_in * ist + lb * JB + c_in) * 4u;
            for (int i = wave; i < 2 * NIS; i += nwaves) {
                const int sidx = i >= NIS ? 1 : 0, ii = i - sidx * NIS;
                const float *ub = (sidx ? base_a : base_m) + (long long)(ii * RPI) * ist;
                const float *src = reinterpret_cast<const float *>(reinterpret_cast<const char *>(ub) + loff);
                if (ii * RPI + r_in >= NRT) continue;      // padding rows of a stream's last instruction: not fetched
#if defined(__HIP_DEVICE_COMPILE__)
                if constexpr (LB == 16) __builtin_amdgcn_global_load_lds(src, sU + (size_t)(sidx * NRTP + ii * RPI) * JB, 16, 0, POL);
                else __builtin_amdgcn_global_load_lds(src, sU + (size_t)(sidx * NRTP + ii * RPI) * JB, 4, 0, POL);
#else
                (void)src;
#endif
            }
            return;
        }
        int j = lb * JB + c_in;
        if (j >= J) j = 0;
        const bool hist = HALO > 0 && tile_t0 == 0 && tail_in != nullptr;
        for (int i = wave; i < 2 * NIS; i += nwaves) {
            const int sidx = i >= NIS ? 1 : 0, ii = i - sidx * NIS;
            int rr = ii * RPI + r_in;
            if (rr >= NRT) rr = NRT - 1;
            const int t = t_first + rr;
            const int tc = t < 0 ? 0 : (t >= L ? L - 1 : t);
            const float *src = (sidx ? base_a : base_m) + ((tc - t_first) * ist + j);
            if (hist && t < 0) src = tail_in + ((size_t)(b * HALO + rr) * 2 + sidx) * J + j;
#if defined(__HIP_DEVICE_COMPILE__)
            if constexpr (LB == 16) __builtin_amdgcn_global_load_lds(src, sU + (size_t)(sidx * NRTP + ii * RPI) * JB, 16, 0, POL);
            else __builtin_amdgcn_global_load_lds(src, sU + (size_t)(sidx * NRTP + ii * RPI) * JB, 4, 0, POL);
#else
            (void)src;
#endif
        }
    }
}
// Stage the valve logits of one tile (gate_mode 1): entry (group, token) of the tile lands at
// sV[group * TT + token]; the lane block's groups are the heads (gpb = 32 / F of them) or the
// one head its 32 lanes lie in.  4 bytes per lane per load; called by one wave.
template <int TT, int JB>
__device__ __forceinline__ void stage_valve(float *sV, const float *valve, int b, int tile_t0, int lb, int L, int H,
                                            int F, int gpb, int lane)
{
    const int h0 = (lb * JB) / F;
    for (int i = 0; i < TT * gpb / 64; ++i) {
        const int idx = i * 64 + lane;
        int t = tile_t0 + idx % TT, h = h0 + idx / TT;
        t = t < L ? t : L - 1;          // rows past the end, heads past the last: a valid address,
        h = h < H ? h : H - 1;          // the value is never used
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_global_load_lds(valve + ((size_t)b * L + t) * H + h, sV + i * 64, 4, 0, 0);
#else
        (void)sV;
        (void)valve;
#endif
    }
}

__device__ __forceinline__ void flag_store(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t flag_load(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Published words.  One 8-byte relaxed agent-scope store carries a value and the call's tag; the
// reader takes the value only from a word whose tag matches.  8-byte naturally aligned accesses are
// single-copy atomic, so a reader sees either the whole new word or an old one.
__device__ __forceinline__ void tagged_store(tagged_t *p, float v, uint32_t tag)
{
    __hip_atomic_store(p, (tagged_t)__float_as_uint(v) | ((tagged_t)tag << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ tagged_t tagged_load(const tagged_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool tagged_ok(tagged_t w, uint32_t tag) { return (uint32_t)(w >> 32) == tag; }
__device__ __forceinline__ float tagged_value(tagged_t w) { return __uint_as_float((uint32_t)w); }

// End of a call, run by thread `tid` of the `nthreads` of the workgroup that left last: tickets and
// the finished-workgroup count return to zero and the epoch advances.  When the epoch wraps, words of
// EPOCH_MOD calls ago would become valid again: everything behind the lane table is cleared then
// (`clear_from`: byte offset of this call's first published word).
__device__ __forceinline__ void finish_call(WsHeader *hdr, size_t clear_from, uint32_t epoch, uint32_t tid,
                                            uint32_t nthreads)
{
    const uint32_t next = (epoch + 1) % EPOCH_MOD;
    if (next == 0) {
        const size_t bytes = (size_t)hdr->bytes_lo | ((size_t)hdr->bytes_hi << 32);
        tagged_t *base = reinterpret_cast<tagged_t *>(reinterpret_cast<char *>(hdr) + clear_from);
        const size_t n = bytes > clear_from ? (bytes - clear_from) / sizeof(tagged_t) : 0;
        for (size_t i = tid; i < n; i += nthreads)
            __hip_atomic_store(base + i, (tagged_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < (uint32_t)MAX_QUEUES) flag_store(&hdr->ticket[tid], 0u);
    if (tid == 0) {
        flag_store(&hdr->done, 0u);
        flag_store(&hdr->epoch, next);
    }
}

// One link of a tile chain: P = T + M c, with M = lambda^TILE_T held as a double-float (h + q) and
// conjugated for the adjoint chain.  Publication of a prefix and the look-back both go through
// this one function, so every tile's prefix has the value a strictly sequential chain would give,
// wherever the look-back happened to find its starting prefix: results do not depend on timing.
template <bool CONJ>
__device__ __forceinline__ void chain_step(float Tr, float Ti, float hr, float hi, float qr, float qi,
                                           float cr, float ci, float &Pr, float &Pi)
{
    if (!CONJ) {
        const float lo_r = __builtin_fmaf(qr, cr, -qi * ci);
        const float lo_i = __builtin_fmaf(qi, cr, qr * ci);
        Pr = __builtin_fmaf(hr, cr, __builtin_fmaf(-hi, ci, Tr + lo_r));
        Pi = __builtin_fmaf(hi, cr, __builtin_fmaf(hr, ci, Ti + lo_i));
    } else {
        const float lo_r = __builtin_fmaf(qr, cr, qi * ci);
        const float lo_i = __builtin_fmaf(qr, ci, -qi * cr);
        Pr = __builtin_fmaf(hr, cr, __builtin_fmaf(hi, ci, Tr + lo_r));
        Pi = __builtin_fmaf(hr, ci, __builtin_fmaf(-hi, cr, Ti + lo_i));
    }
}

// Decoupled look-back, run by one group of LPR consecutive threads of a wave (thread lv of the
// group owns V lanes at lane offset `lo` of the tile slots; a slot is [2][JB] tagged words).
// `pred` is the chain predecessor's tile index, `depth` the number of tiles before this one in the
// chain (the chain's first tile always publishes a prefix).
//   The group reads the prefixes AND aggregates of the next NB predecessors in one round trip; a
//   tile's words count only when all of the group's lanes found their tags valid.  It stops at the
//   nearest tile with a valid prefix, provided every nearer tile has a valid aggregate; it waits
//   (bounded, polling one word per lane) on the nearest tile that has published nothing yet.  Then it walks forward from that
//   prefix through the aggregates with chain_step(), from the registers of the last window and, for
//   nearer tiles seen in earlier windows, by reading them again (published words never change
//   within a call).  In the common case -- a prefix within NB tiles -- that is one round trip.
// Returns false if a wait gave up (the carry is then meaningless).
// RET (data-dependent retention): an aggregate has a third word per lane, the product of the tile's
// retentions (aggp, [tile][JB]); a link then is P = T + product * M c.
template <int V, bool CONJ, int LPR, int NB, bool RET = false>
__device__ __forceinline__ bool look_back(const tagged_t *agg, const tagged_t *pre, uint32_t pred, uint32_t stride,
                                          int depth, int JB, int lo, int lv, const float (&hr)[V],
                                          const float (&hi)[V], const float (&qr)[V], const float (&qi)[V],
                                          uint32_t spin_limit, uint32_t tag, float (&cr)[V], float (&ci)[V],
                                          const tagged_t *aggp = nullptr)
{
    const int gshift = (int)(threadIdx.x & 63) - lv;
    const unsigned long long gmask = LPR >= 64 ? ~0ull : ((1ull << LPR) - 1ull);
    auto group_all = [&](bool ok) { return ((__ballot(ok) >> gshift) & gmask) == gmask; };
    int base = 0;       // tiles at distance < base are known to hold aggregates
    uint32_t spins = 0;
    float ar[NB][V], ai[NB][V];      // aggregates of the current window
    float ap[RET ? NB : 1][V];
    int found = -1;                  // position of the prefix in the current window
    while (true) {
        const int w = depth - base < NB ? depth - base : NB;
        bool pok[NB], aok[NB];
        float pr_[NB][V], pi_[NB][V];
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            const int dd = n < w ? base + n : base;      // (positions past the chain's start repeat a valid one)
            const size_t slot = (size_t)(pred - (uint32_t)dd * stride) * 2 * JB + lo;
            pok[n] = aok[n] = true;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const tagged_t w0 = tagged_load(pre + slot + v), w1 = tagged_load(pre + slot + JB + v);
                const tagged_t w2 = tagged_load(agg + slot + v), w3 = tagged_load(agg + slot + JB + v);
                pok[n] = pok[n] && tagged_ok(w0, tag) && tagged_ok(w1, tag);
                aok[n] = aok[n] && tagged_ok(w2, tag) && tagged_ok(w3, tag);
                pr_[n][v] = tagged_value(w0); pi_[n][v] = tagged_value(w1);
                ar[n][v] = tagged_value(w2);  ai[n][v] = tagged_value(w3);
                if constexpr (RET) {
                    const tagged_t w4 = tagged_load(aggp + (size_t)(pred - (uint32_t)dd * stride) * JB + lo + v);
                    aok[n] = aok[n] && tagged_ok(w4, tag);
                    ap[n][v] = tagged_value(w4);
                }
            }
        }
        compiler_fence();
        int stall = -1;
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            if (found < 0 && stall < 0 && n < w) {
                if (group_all(pok[n])) {
                    found = n;
#pragma unroll
                    for (int v = 0; v < V; ++v) { cr[v] = pr_[n][v]; ci[v] = pi_[n][v]; }
                } else if (!group_all(aok[n])) {
                    stall = n;
                }
            }
        }
        if (found >= 0) break;
        if (stall >= 0) {           // the tile at base + stall has published nothing yet
            base += stall;
            // wait for it on one word per lane (a light poll), then read the window again.  The
            // chain's first tile publishes a prefix only; every other tile publishes its aggregate first.
            const tagged_t *probe = (base == depth - 1 ? pre : agg) + (size_t)(pred - (uint32_t)base * stride) * 2 * JB + lo;
            while (true) {
                if (++spins > spin_limit) return false;
                __builtin_amdgcn_s_sleep(1);
                if (group_all(tagged_ok(tagged_load(probe), tag))) break;
            }
        } else {
            base += w;              // aggregates only: look further back
            if (base >= depth) return false;   // cannot happen: the chain's first tile publishes a prefix
        }
    }
    // forward again: first the aggregates of the last window, nearest last
#pragma unroll
    for (int n = NB - 1; n >= 0; --n) {
        if (n < found) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float nr, ni;
                if constexpr (RET) { cr[v] *= ap[n][v]; ci[v] *= ap[n][v]; }
                chain_step<CONJ>(ar[n][v], ai[n][v], hr[v], hi[v], qr[v], qi[v], cr[v], ci[v], nr, ni);
                cr[v] = nr;
                ci[v] = ni;
            }
        }
    }
    // then the tiles of earlier windows (nearer than `base`)
    for (int d = base - 1; d >= 0; d -= NB) {
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            const int dd = d - n < 0 ? 0 : d - n;
            const size_t slot = (size_t)(pred - (uint32_t)dd * stride) * 2 * JB + lo;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                ar[n][v] = tagged_value(tagged_load(agg + slot + v));
                ai[n][v] = tagged_value(tagged_load(agg + slot + JB + v));
                if constexpr (RET)
                    ap[n][v] = tagged_value(tagged_load(aggp + (size_t)(pred - (uint32_t)dd * stride) * JB + lo + v));
            }
        }
#pragma unroll
        for (int n = 0; n < NB; ++n) {
            if (d - n >= 0) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float nr, ni;
                    if constexpr (RET) { cr[v] *= ap[n][v]; ci[v] *= ap[n][v]; }
                    chain_step<CONJ>(ar[n][v], ai[n][v], hr[v], hi[v], qr[v], qi[v], cr[v], ci[v], nr, ni);
                    cr[v] = nr;
                    ci[v] = ni;
                }
            }
        }
    }
    return true;
}
#endif

}  // namespace cawn
