// Sanitizer run of the host side of libcawn's gates (test infrastructure): includes the library's host-only
// header, is built with g++ -fsanitize=address,undefined, and checks the fp32 breakpoints that the bisection
// returns against the decision evaluated directly: every returned interval end is open, its outer neighbour
// (one fp32 step away) is closed, and a sweep of sampled fp32 values falls on the right side.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_2604_04250_amd/csrc/cawn_gate_host.hpp"

using namespace cawn;

static int g_fail = 0;
#define CHECK(c, ...) do { if (!(c)) { ++g_fail; std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } } while (0)

static bool in_set(const GateSet &g, float x) { return (x >= g.a1 && x <= g.b1) || (x >= g.a2 && x <= g.b2); }

static void check_gate(bool fused, int amp, double cc, float tau)
{
    GateSet gs;
    const bool ok = make_gate_set(fused, amp, cc, tau, &gs);
    CHECK(ok, "make_gate_set(%d,%d,%g,%g) refused", (int)fused, amp, cc, (double)tau);
    if (!ok) return;
    GateFn fn{fused, amp, cc, (double)tau};
    const float INF = std::numeric_limits<float>::infinity(), FMAX = std::numeric_limits<float>::max();
    // the ends: open inside, closed one step outside
    const float ends[4] = {gs.a1, gs.b1, gs.a2, gs.b2};
    for (int i = 0; i < 4; i += 2) {
        const float a = ends[i], b = ends[i + 1];
        if (a > b) continue;   // empty interval
        const float af = a == -INF ? -FMAX : a, bf = b == INF ? FMAX : b;
        CHECK(tau <= 0 || fn.open(af), "lower end %g closed (tau %g fused %d amp %d)", (double)af, (double)tau, (int)fused, amp);
        CHECK(tau <= 0 || fn.open(bf), "upper end %g closed (tau %g fused %d amp %d)", (double)bf, (double)tau, (int)fused, amp);
        if (a != -INF) CHECK(!fn.open(unord(ord(a) - 1)), "value below %g open", (double)a);
        if (b != INF) CHECK(!fn.open(unord(ord(b) + 1)), "value above %g open", (double)b);
    }
    // a sweep: dense near zero and the SiLU minimum, sparse over the whole range
    std::vector<float> xs;
    for (int i = -4000; i <= 4000; ++i) xs.push_back((float)i * 0.0025f);
    for (int e = -120; e <= 120; e += 3) { xs.push_back(std::ldexp(1.0f, e)); xs.push_back(-std::ldexp(1.0f, e)); }
    xs.push_back(0.0f); xs.push_back(-0.0f); xs.push_back(FMAX); xs.push_back(-FMAX);
    for (float x : xs)
        CHECK(in_set(gs, x) == (tau <= 0 ? true : fn.open(x)), "x %g: set says %d (tau %g fused %d amp %d)", (double)x,
              (int)in_set(gs, x), (double)tau, (int)fused, amp);
}

int main()
{
    const float taus[] = {0.0f, -1.0f, 1e-30f, 0.05f, 0.1f, 0.25f, 0.2784f, 0.2785f, 0.5f, 0.6931f, 0.6932f, 1.0f, 5.0f, 9.99f,
                          10.0f, 10.5f, 49.0f, 50.0f, 51.0f, 1e30f, std::numeric_limits<float>::infinity()};
    for (float tau : taus)
        for (int fused = 0; fused < 2; ++fused)
            for (int amp = 0; amp < 2; ++amp)
                for (double cc : {50.0, 2.0, (double)std::numeric_limits<float>::infinity()})
                    check_gate(fused != 0, amp, cc, tau);
    GateSet gs;
    CHECK(make_gate_set(true, 0, 50.0, std::nanf(""), &gs) && gs.a1 > gs.b1 && gs.a2 > gs.b2, "NaN threshold: not the empty set");
    // the ordered-integer map is a bijection that keeps order
    const float vals[] = {-std::numeric_limits<float>::max(), -1.0f, -1e-45f, -0.0f, 0.0f, 1e-45f, 1.0f, std::numeric_limits<float>::max()};
    for (size_t i = 0; i < sizeof vals / sizeof vals[0]; ++i) {
        CHECK(unord(ord(vals[i])) == vals[i], "ord/unord round trip at %g", (double)vals[i]);
        if (i) CHECK(ord(vals[i - 1]) <= ord(vals[i]), "ord not monotone at %g", (double)vals[i]);
    }
    // the valve: sigmoid(v - 3) >= eps
    const float epss[] = {0.001f, 0.3f, 0.5f, 0.999f, 1e-30f};
    for (float eps : epss) {
        const float thr = valve_threshold(eps);
        auto open = [&](float v) { return 1.0 / (1.0 + std::exp(-((double)v - 3.0))) >= (double)eps; };
        CHECK(open(thr), "valve threshold %g closed (eps %g)", (double)thr, (double)eps);
        CHECK(!open(unord(ord(thr) - 1)), "value below the valve threshold %g open (eps %g)", (double)thr, (double)eps);
    }
    CHECK(valve_threshold(0.0f) == -std::numeric_limits<float>::infinity(), "eps 0: always open");
    CHECK(valve_threshold(1.5f) == std::numeric_limits<float>::infinity(), "eps > 1: never open");
    CHECK(valve_threshold(std::nanf("")) == std::numeric_limits<float>::infinity(), "eps NaN: never open");
    const float t001 = valve_threshold(0.001f);
    CHECK(std::fabs((double)t001 - (3.0 + std::log(0.001 / 0.999))) < 1e-5, "eps 0.001: threshold %g", (double)t001);
    if (g_fail) { std::printf("%d failure(s)\n", g_fail); return 1; }
    std::puts("gate sanitizer run: done");
    return 0;
}
