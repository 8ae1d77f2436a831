// Host-only part of libcawn's gates: the fp32 breakpoints of the two gate decisions, found by bisection over
// the ordered fp32 values.  Plain C++ with no HIP in it, so that it also builds with a host compiler alone
// (the sanitizer build of the CPU tests includes this file and nothing else of the library).
#pragma once
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

namespace cawn {

// Gate as a union of two closed fp32 intervals on the quantity the decision is taken on (the
// fp32 conv pre-activation, or the raw magnitude input when there is no conv).
struct GateSet { float a1, b1, a2, b2; };

// ------------------------------------------------------------------------------------------ gate
// The gate decision |A(X(x))| >= tau is defined on an fp32 quantity x (the conv pre-activation, or
// the raw magnitude when there is no conv), evaluated in fp64.  It is piecewise monotone in x, so
// the open set is a union of at most two closed fp32 intervals, found by bisection over the
// ordered fp32 values.
struct GateFn {
    bool fused;
    int amp_mode;
    double cc;   // conv clamp
    double tau;
    double f(float x) const
    {
        double v = (double)x;
        if (fused) {
            v = v < -cc ? -cc : (v > cc ? cc : v);
            v = v / (1.0 + std::exp(-v));   // SiLU
        }
        if (amp_mode == 1) {
            double sp = v > 30.0 ? v + std::log1p(std::exp(-v)) : std::log1p(std::exp(v));
            v = sp < 10.0 ? sp : 10.0;
        }
        return std::fabs(v);
    }
    bool open(float x) const { return f(x) >= tau; }
};

inline int64_t ord(float x)
{
    int32_t b;
    std::memcpy(&b, &x, 4);
    return b >= 0 ? (int64_t)b : -(int64_t)(b & 0x7fffffff);
}
inline float unord(int64_t o)
{
    int32_t b = o >= 0 ? (int32_t)o : (int32_t)((uint32_t)(-o) | 0x80000000u);
    float x;
    std::memcpy(&x, &b, 4);
    return x;
}

struct Interval { float lo, hi; bool empty; };

// Open sub-interval of the monotone piece [l, r].
inline Interval piece(const GateFn &g, float l, float r, bool increasing)
{
    int64_t lo = ord(l), hi = ord(r);
    if (increasing) {
        if (!g.open(r)) return {0, 0, true};
        while (lo < hi) {   // smallest open value
            int64_t mid = lo + (hi - lo) / 2;
            if (g.open(unord(mid))) hi = mid; else lo = mid + 1;
        }
        return {unord(lo), r, false};
    }
    if (!g.open(l)) return {0, 0, true};
    while (lo < hi) {       // largest open value
        int64_t mid = lo + (hi - lo + 1) / 2;
        if (g.open(unord(mid))) lo = mid; else hi = mid - 1;
    }
    return {l, unord(lo), false};
}

inline bool make_gate_set(bool fused, int amp_mode, double conv_clamp, float gate_tau, GateSet *out)
{
    const float INF = std::numeric_limits<float>::infinity();
    const float FMAX = std::numeric_limits<float>::max();
    GateSet gs{INF, -INF, INF, -INF};
    const double tau = (double)gate_tau;
    if (std::isnan(tau)) { *out = gs; return true; }
    if (tau <= 0.0) { gs.a1 = -INF; gs.b1 = INF; *out = gs; return true; }
    GateFn g{fused, amp_mode, conv_clamp, tau};
    const float ZSTAR = -1.2784645f;   // argmin of SiLU
    Interval iv[3];
    int n = 0;
    if (g.fused && g.amp_mode == 0) {
        iv[n++] = piece(g, -FMAX, ZSTAR, true);
        iv[n++] = piece(g, ZSTAR, 0.0f, false);
        iv[n++] = piece(g, 0.0f, FMAX, true);
    } else if (g.fused) {
        iv[n++] = piece(g, -FMAX, ZSTAR, false);
        iv[n++] = piece(g, ZSTAR, FMAX, true);
    } else if (g.amp_mode == 0) {
        iv[n++] = piece(g, -FMAX, 0.0f, false);
        iv[n++] = piece(g, 0.0f, FMAX, true);
    } else {
        iv[n++] = piece(g, -FMAX, FMAX, true);
    }
    // merge pieces that meet, widen the outer ends to infinity
    Interval m[3];
    int k = 0;
    for (int i = 0; i < n; ++i) {
        if (iv[i].empty) continue;
        if (k > 0 && ord(iv[i].lo) <= ord(m[k - 1].hi) + 1) m[k - 1].hi = iv[i].hi;
        else m[k++] = iv[i];
    }
    if (k > 2) return false;
    for (int i = 0; i < k; ++i) {
        if (m[i].lo == -FMAX) m[i].lo = -INF;
        if (m[i].hi == FMAX) m[i].hi = INF;
    }
    if (k > 0) { gs.a1 = m[0].lo; gs.b1 = m[0].hi; }
    if (k > 1) { gs.a2 = m[1].lo; gs.b2 = m[1].hi; }
    *out = gs;
    return true;
}

// gate_mode 1: the valve of Sec. 3.3 is open when sigmoid(v - 3) >= eps, a decision defined on the
// fp32 logit v and evaluated in fp64.  sigmoid is increasing, so the open set is [thr, +inf): thr is
// found by bisection over the ordered fp32 values.  +inf: never open; -inf: always open.
inline float valve_threshold(float eps)
{
    const float INF = std::numeric_limits<float>::infinity();
    const float FMAX = std::numeric_limits<float>::max();
    const double e = (double)eps;
    auto open = [&](float v) { return 1.0 / (1.0 + std::exp(-((double)v - 3.0))) >= e; };
    if (std::isnan(e)) return INF;
    if (open(-FMAX)) return -INF;
    if (!open(FMAX)) return INF;
    int64_t lo = ord(-FMAX), hi = ord(FMAX);
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (open(unord(mid))) hi = mid; else lo = mid + 1;
    }
    return unord(lo);
}

}  // namespace cawn
