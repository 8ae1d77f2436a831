"""Pins for the fp64 oracle: what the paper and the mathematics fix, written with numpy complex
arithmetic / library routines that share nothing with the oracle's real-form loop.

Each test is chosen so that a plausible slip in the oracle (a dropped term, a sign, a transposed
tap, an off-by-one in time) fails it.  CPU only.
"""
import math

import numpy as np
import pytest

from oracle import cawn_oracle as O

INF = float("inf")


def rng_(seed):
    return np.random.Generator(np.random.PCG64(seed))


def lam(gamma, theta):
    return gamma.astype(np.float64) * np.exp(1j * theta.astype(np.float64))


def np_silu(v):
    return v / (1.0 + np.exp(-v))


def np_dsilu(v):
    s = 1.0 / (1.0 + np.exp(-v))
    return s * (1.0 + v * (1.0 - s))


def brute_scan(p, lmb, s_in=None):
    """O(L^2): S_t = lambda^(t+1) S_in + sum_{tau<=t} lambda^(t-tau) p_tau  (Sec. 3.4: a push
    injected at tau is rotated by (t-tau) theta and decayed by gamma^(t-tau))."""
    B, L, J = p.shape
    S = np.zeros((B, L, J), dtype=np.complex128)
    for t in range(L):
        for tau in range(t + 1):
            S[:, t] += np.power(lmb, t - tau)[None] * p[:, tau]
        if s_in is not None:
            S[:, t] += np.power(lmb, t + 1)[None] * s_in
    return S


def brute_adjoint(dS, lmb):
    """G_t = sum_{s>=t} conj(lambda)^(s-t) dS_s."""
    B, L, J = dS.shape
    G = np.zeros((B, L, J), dtype=np.complex128)
    for t in range(L):
        for s in range(t, L):
            G[:, t] += np.power(np.conj(lmb), s - t)[None] * dS[:, s]
    return G


def small(seed, B=2, L=24, H=2, F=3, Kc=0):
    r = rng_(seed)
    J = H * F
    d = dict(mag=r.standard_normal((B, L, J)).astype(np.float32),
             ang=(2.0 * r.standard_normal((B, L, J))).astype(np.float32),
             gamma=r.uniform(0.5, 0.999, J).astype(np.float32),
             theta=r.uniform(0, np.pi, J).astype(np.float32))
    if Kc:
        d["conv_w"] = (r.standard_normal((2, J, Kc)) / math.sqrt(Kc)).astype(np.float32)
        d["conv_b"] = (0.1 * r.standard_normal((2, J))).astype(np.float32)
    return d


# ----------------------------------------------------------------------------------- recurrence
def test_brute_force_sum_of_decayed_rotated_pushes():
    B, L, H, F = 2, 40, 2, 4
    d = small(1, B, L, H, F)
    tau = 0.3
    cfg = O.Cfg(B, L, H, F, gate_tau=tau, out_clamp=INF)
    s_in = rng_(2).standard_normal((B, 2, H * F))
    out = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], scan_in=s_in)
    a = d["mag"].astype(np.float64)
    g = np.abs(d["mag"]) >= np.float32(tau)
    p = g * a * np.exp(1j * d["ang"].astype(np.float64))
    S = brute_scan(p, lam(d["gamma"], d["theta"]), s_in[:, 0] + 1j * s_in[:, 1])
    np.testing.assert_allclose(out["z_re"], S.real, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["z_im"], S.imag, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(out["gate"], g.astype(np.uint8))
    np.testing.assert_allclose(out["scan_out"][:, 0], S[:, -1].real, atol=1e-12)
    np.testing.assert_allclose(out["scan_out"][:, 1], S[:, -1].imag, atol=1e-12)


def test_single_impulse_modulus_and_counter_clockwise_phase():
    # one push at t0: |S_t| = gamma^(t-t0) |p|, arg S_t = phi + (t-t0) theta  (Sec. 3.4)
    L, t0 = 30, 4
    gamma = np.array([0.97], np.float32)
    theta = np.array([0.11], np.float32)
    mag = np.zeros((1, L, 1), np.float32)
    ang = np.zeros((1, L, 1), np.float32)
    mag[0, t0, 0] = 1.5
    ang[0, t0, 0] = 0.4
    out = O.phase_fwd(O.Cfg(1, L, 1, 1), mag, ang, gamma, theta)
    S = out["z_re"][0, :, 0] + 1j * out["z_im"][0, :, 0]
    assert np.all(S[:t0] == 0)
    n = np.arange(L - t0)
    np.testing.assert_allclose(np.abs(S[t0:]), 1.5 * float(gamma[0]) ** n, rtol=1e-13)
    expect = float(ang[0, t0, 0]) + n * float(theta[0])
    np.testing.assert_allclose(np.angle(S[t0:] * np.exp(-1j * expect)), 0.0, atol=1e-13)


def test_constant_input_geometric_series():
    L, H, F = 200, 1, 5
    J = H * F
    gamma = np.array([0.9, 0.99, 0.999, 1.0, 0.5], np.float32)
    theta = np.array([0.0, 0.3, 1.0, 0.0, 3.0], np.float32)
    mag = np.full((1, L, J), 0.75, np.float32)
    ang = np.full((1, L, J), -0.6, np.float32)
    out = O.phase_fwd(O.Cfg(1, L, H, F, out_clamp=INF), mag, ang, gamma, theta)
    lmb = lam(gamma, theta)
    p = 0.75 * np.exp(1j * float(np.float32(-0.6)))
    t = np.arange(L)[:, None]
    with np.errstate(invalid="ignore", divide="ignore"):
        S = p * (1 - lmb[None] ** (t + 1)) / (1 - lmb[None])
    S[:, 3] = (t[:, 0] + 1) * p  # lambda = 1
    got = out["z_re"][0] + 1j * out["z_im"][0]
    np.testing.assert_allclose(got, S, rtol=1e-11, atol=1e-12)


def test_reduces_to_prefix_sum():
    B, L, H, F = 2, 100, 1, 4
    d = small(3, B, L, H, F)
    one = np.ones(H * F, np.float32)
    zero = np.zeros(H * F, np.float32)
    out = O.phase_fwd(O.Cfg(B, L, H, F, gate_tau=0.0, out_clamp=INF), d["mag"], d["ang"], one, zero)
    p = d["mag"].astype(np.float64) * np.exp(1j * d["ang"].astype(np.float64))
    np.testing.assert_allclose(out["z_re"], np.cumsum(p.real, axis=1), atol=1e-12)
    np.testing.assert_allclose(out["z_im"], np.cumsum(p.imag, axis=1), atol=1e-12)
    assert out["gate"].all()


@pytest.mark.parametrize("Kc", [0, 3, 4])
def test_chunked_equals_unchunked_bitwise(Kc):
    B, L, H, F = 2, 37, 2, 3
    d = small(4, B, L, H, F, Kc)
    kw = dict(conv_w=d.get("conv_w"), conv_b=d.get("conv_b"))
    full = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=0.1), d["mag"], d["ang"], d["gamma"],
                       d["theta"], **kw)
    for splits in ([1] * L, [2, 1, 1, 3, 30], [36, 1], [5, 32], [17, 20]):
        assert sum(splits) == L
        scan, tail, t0 = None, None, 0
        zr, zi, gt = [], [], []
        for n in splits:
            o = O.phase_fwd(O.Cfg(B, n, H, F, conv_k=Kc, gate_tau=0.1), d["mag"][:, t0:t0 + n],
                            d["ang"][:, t0:t0 + n], d["gamma"], d["theta"], scan_in=scan,
                            tail_in=tail, **kw)
            scan, tail = o["scan_out"], o["tail_out"]
            zr.append(o["z_re"]); zi.append(o["z_im"]); gt.append(o["gate"])
            t0 += n
        assert np.array_equal(np.concatenate(zr, 1), full["z_re"])
        assert np.array_equal(np.concatenate(zi, 1), full["z_im"])
        assert np.array_equal(np.concatenate(gt, 1), full["gate"])
        assert np.array_equal(scan, full["scan_out"])
        if Kc > 1:
            assert np.array_equal(tail, full["tail_out"])
            assert np.array_equal(tail[:, :, 0], d["mag"][:, L - (Kc - 1):])
            assert np.array_equal(tail[:, :, 1], d["ang"][:, L - (Kc - 1):])


# ----------------------------------------------------------------------------------------- conv
def test_conv_kernel1_is_silu():
    x = rng_(5).standard_normal((2, 9, 4)).astype(np.float32)
    y, _ = O.syntax_conv(x, np.ones((4, 1), np.float32))
    np.testing.assert_allclose(y, np_silu(x.astype(np.float64)), rtol=1e-14)


def test_conv_impulse_reads_taps_back_last_tap_on_current_token():
    Kc, L, t0 = 4, 12, 3
    w = np.array([[0.1, 0.2, 0.3, 0.4]], np.float32)
    x = np.zeros((1, L, 1), np.float32)
    x[0, t0, 0] = 1.0
    y, _ = O.syntax_conv(x, w, conv_clamp=INF)
    z = np.zeros(L)
    for d in range(Kc):
        z[t0 + d] = float(w[0, Kc - 1 - d])   # current token meets the LAST tap
    np.testing.assert_allclose(y[0, :, 0], np_silu(z), rtol=1e-14)


@pytest.mark.parametrize("Kc", [3, 4])
def test_conv_matches_numpy_convolve_with_history_and_clamp(Kc):
    r = rng_(6)
    B, L, Cc = 2, 20, 3
    x = (30 * r.standard_normal((B, L, Cc))).astype(np.float32)
    w = r.standard_normal((Cc, Kc)).astype(np.float32)
    bias = r.standard_normal(Cc).astype(np.float32)
    hist = r.standard_normal((B, Kc - 1, Cc)).astype(np.float32)
    y, hout = O.syntax_conv(x, w, bias, hist)
    for b in range(B):
        for c in range(Cc):
            seq = np.concatenate([hist[b, :, c], x[b, :, c]]).astype(np.float64)
            z = np.convolve(seq, w[c, ::-1].astype(np.float64), mode="valid") + float(bias[c])
            assert z.shape == (L,)
            np.testing.assert_allclose(y[b, :, c], np_silu(np.clip(z, -50, 50)), rtol=1e-12,
                                       atol=1e-15)
    assert (np.abs(y) <= 50).all() and np.abs(x).max() > 50
    np.testing.assert_array_equal(hout, x[:, L - (Kc - 1):])


def test_fused_front_end_equals_conv_then_scan():
    B, L, H, F, Kc = 2, 25, 2, 2, 4
    J = H * F
    d = small(7, B, L, H, F, Kc)
    _, tail = (None, rng_(8).standard_normal((B, Kc - 1, 2, J)).astype(np.float32))
    fused = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc), d["mag"], d["ang"], d["gamma"], d["theta"],
                        conv_w=d["conv_w"], conv_b=d["conv_b"], tail_in=tail)
    xcat = np.concatenate([d["mag"], d["ang"]], axis=2)                  # [B,L,2J]
    y, _ = O.syntax_conv(xcat, d["conv_w"].reshape(2 * J, Kc), d["conv_b"].reshape(2 * J),
                         tail.reshape(B, Kc - 1, 2 * J))
    p = y[..., :J] * np.exp(1j * y[..., J:])
    S = brute_scan(p, lam(d["gamma"], d["theta"]))
    np.testing.assert_allclose(fused["z_re"], S.real, atol=1e-12)
    np.testing.assert_allclose(fused["z_im"], S.imag, atol=1e-12)


# ----------------------------------------------------------------------------------------- gate
def test_gate_open_closed_and_fraction():
    B, L, H, F = 1, 4000, 2, 8
    J = H * F
    r = rng_(9)
    mag = r.standard_normal((B, L, J)).astype(np.float32)
    ang = r.standard_normal((B, L, J)).astype(np.float32)
    gamma = r.uniform(0.9, 0.99, J).astype(np.float32)
    theta = r.uniform(0, 3, J).astype(np.float32)
    s_in = r.standard_normal((B, 2, J))
    o0 = O.phase_fwd(O.Cfg(B, L, H, F, gate_tau=0.0), mag, ang, gamma, theta)
    assert o0["gate"].all()
    oc = O.phase_fwd(O.Cfg(B, 50, H, F, gate_tau=INF), mag[:, :50], ang[:, :50], gamma, theta,
                     scan_in=s_in)
    assert not oc["gate"].any()
    lmb = lam(gamma, theta)
    n = np.arange(1, 51)[:, None]
    free = (lmb[None] ** n) * (s_in[0, 0] + 1j * s_in[0, 1])[None]
    np.testing.assert_allclose(oc["z_re"][0], free.real, atol=1e-13)
    np.testing.assert_allclose(oc["z_im"][0], free.imag, atol=1e-13)
    for tau in (0.1, 0.25):
        o = O.phase_fwd(O.Cfg(B, L, H, F, gate_tau=tau), mag, ang, gamma, theta)
        closed = 1.0 - o["gate"].mean()
        expect = math.erf(tau / math.sqrt(2))        # P(|N(0,1)| < tau): 7.97 % / 19.74 %
        assert abs(closed - expect) < 4 * math.sqrt(expect * (1 - expect) / (L * J))
    # keep when equal to the threshold
    m2 = np.array([[[0.25], [np.nextafter(np.float32(0.25), np.float32(0))], [-0.25]]], np.float32)
    o = O.phase_fwd(O.Cfg(1, 3, 1, 1, gate_tau=0.25), m2, np.zeros_like(m2), gamma[:1], theta[:1])
    assert o["gate"][0, :, 0].tolist() == [1, 0, 1]


def test_fused_gate_is_taken_on_the_fp32_preactivation():
    # decision = |SiLU(clamp(z32))| >= tau with z32 the fp32 fma chain, bias first, taps in order
    B, L, H, F, Kc = 1, 300, 1, 4, 4
    d = small(10, B, L, H, F, Kc)
    tau = 0.1
    o = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=tau), d["mag"], d["ang"], d["gamma"],
                    d["theta"], conv_w=d["conv_w"], conv_b=d["conv_b"])
    J = H * F
    pad = np.concatenate([np.zeros((B, Kc - 1, J), np.float32), d["mag"]], axis=1)
    z32 = np.broadcast_to(d["conv_b"][0][None, None], (B, L, J)).astype(np.float32).copy()
    for i in range(Kc):
        prod = d["conv_w"][0][None, None, :, i].astype(np.float64) * pad[:, i:i + L].astype(np.float64)
        z32 = (prod + z32.astype(np.float64)).astype(np.float32)   # fp64 product+sum is exact enough: one rounding
    gate = np.abs(np_silu(np.clip(z32.astype(np.float64), -50, 50))) >= float(np.float32(tau))
    assert (o["gate"] == gate).mean() > 0.999   # numpy emulation of fma may differ by a double rounding
    # gated-off lanes contribute nothing: zero them by hand and compare with tau = 0 on masked input
    assert 0.02 < 1 - o["gate"].mean() < 0.6


# ---------------------------------------------------------------------------------------- clamp
def test_output_clamp_saturates_but_state_does_not():
    L = 400
    mag = np.full((1, L, 1), 5.0, np.float32)
    ang = np.zeros((1, L, 1), np.float32)
    one, zero = np.ones(1, np.float32), np.zeros(1, np.float32)
    o = O.phase_fwd(O.Cfg(1, L, 1, 1), mag, ang, one, zero)
    expect = np.minimum(5.0 * np.arange(1, L + 1), 100.0)
    np.testing.assert_allclose(o["z_re"][0, :, 0], expect)
    assert o["scan_out"][0, 0, 0] == 5.0 * L
    # the other reading (clamped value carried), offered only to quantify the difference
    of = O.phase_fwd(O.Cfg(1, L, 1, 1, clamp_feedback=1), mag, ang, one, zero)
    assert of["scan_out"][0, 0, 0] == 100.0


def test_amplitude_softplus_cap():
    m = np.array([[[0.0], [20.0], [-3.0]]], np.float32)
    z = np.zeros_like(m)
    o = O.phase_fwd(O.Cfg(1, 3, 1, 1, amp_mode=1), m, z, np.zeros(1, np.float32), np.zeros(1, np.float32))
    np.testing.assert_allclose(o["z_re"][0, :, 0], [math.log(2), 10.0, math.log1p(math.exp(-3))],
                               rtol=1e-14)


# ------------------------------------------------------------------------------------- backward
def test_adjoint_dot_product_identity():
    B, L, H, F = 2, 50, 2, 3
    d = small(11, B, L, H, F)
    r = rng_(12)
    dz_re = r.standard_normal((B, L, H * F)).astype(np.float32)
    dz_im = r.standard_normal((B, L, H * F)).astype(np.float32)
    cfg = O.Cfg(B, L, H, F, out_clamp=INF, grad_clamp=INF)
    f = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"])
    g = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], dz_re, dz_im)
    # <dZ, Scan(p)> = <Scan^T(dZ), p>, with Scan^T(dZ) recovered from (dmag, dang):
    # dmag = Re(conj(G) e^{i phi}), dang = a Im(conj(G) e^{i phi})... so sum(G . p) = sum(a * dmag)
    lhs = (dz_re * f["z_re"] + dz_im * f["z_im"]).sum()
    rhs = (d["mag"].astype(np.float64) * g["dmag"]).sum()
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)
    G = brute_adjoint(dz_re.astype(np.float64) + 1j * dz_im, lam(d["gamma"], d["theta"]))
    e = np.exp(1j * d["ang"].astype(np.float64))
    np.testing.assert_allclose(g["dmag"], (np.conj(G) * e).real, atol=1e-12)
    np.testing.assert_allclose(g["dang"], d["mag"] * (np.conj(G) * 1j * e).real, atol=1e-12)


def _loss(cfg, d, up, scan_in, tail_in):
    f = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], conv_w=d.get("conv_w"),
                    conv_b=d.get("conv_b"), scan_in=scan_in, tail_in=tail_in)
    v = (up["dz_re"] * f["z_re"]).sum() + (up["dz_im"] * f["z_im"]).sum()
    v += (up["dscan_out"] * f["scan_out"]).sum()
    if cfg.conv_k > 1:
        v += (up["dtail_out"] * f["tail_out"]).sum()
    return v


@pytest.mark.parametrize("Kc,amp_mode,L", [(0, 0, 9), (4, 0, 9), (3, 1, 7), (4, 0, 2), (0, 1, 5)])
def test_all_gradients_against_finite_differences(Kc, amp_mode, L):
    B, H, F = 2, 1, 3
    J = H * F
    d = small(13 + Kc, B, L, H, F, Kc)
    q = lambda a: (np.round(a * 1024) / 1024).astype(np.float32)     # leave room for exact +-h
    for k in d:
        d[k] = q(d[k])
    r = rng_(14)
    scan_in = np.round(r.standard_normal((B, 2, J)) * 1024) / 1024
    tail_in = q(r.standard_normal((B, Kc - 1, 2, J))) if Kc > 1 else None
    up = dict(dz_re=r.standard_normal((B, L, J)).astype(np.float32),
              dz_im=r.standard_normal((B, L, J)).astype(np.float32),
              dscan_out=r.standard_normal((B, 2, J)),
              dtail_out=r.standard_normal((B, max(Kc - 1, 0), 2, J)))
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=0.0, conv_clamp=INF,
                out_clamp=INF, grad_clamp=INF)
    g = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], up["dz_re"], up["dz_im"],
                    conv_w=d.get("conv_w"), conv_b=d.get("conv_b"), scan_in=scan_in,
                    tail_in=tail_in, dscan_out=up["dscan_out"],
                    dtail_out=up["dtail_out"] if Kc > 1 else None)

    def fd(name, arr, idx, is_state=False):
        def at(h):
            a2 = arr.copy()
            a2[idx] += h
            dd = dict(d)
            si, ti = scan_in, tail_in
            if name == "scan_in":
                si = a2
            elif name == "tail_in":
                ti = a2
            else:
                dd[name] = a2
            return _loss(cfg, dd, up, si, ti)
        h = 2.0 ** -7
        d1 = (at(h) - at(-h)) / (2 * h)
        d2 = (at(h / 2) - at(-h / 2)) / h
        return (4 * d2 - d1) / 3                                        # Richardson, O(h^4)

    checks = [("mag", d["mag"], g["dmag"]), ("ang", d["ang"], g["dang"]),
              ("gamma", d["gamma"], g["dgamma"]), ("theta", d["theta"], g["dtheta"]),
              ("scan_in", scan_in, g["dscan_in"])]
    if Kc > 0:
        checks += [("conv_w", d["conv_w"], g["dconv_w"]), ("conv_b", d["conv_b"], g["dconv_b"])]
    if Kc > 1:
        checks += [("tail_in", tail_in, g["dtail_in"])]
    r2 = rng_(15)
    for name, arr, grad in checks:
        assert grad.shape == arr.shape, name
        flat = r2.permutation(arr.size)[:10]
        for f in flat:
            idx = np.unravel_index(f, arr.shape)
            num = fd(name, arr, idx)
            assert abs(num - grad[idx]) <= 2e-7 * max(1.0, abs(num)), (name, idx, num, grad[idx])


def test_ste_gradient_ignores_gate_for_amplitude_and_masks_phase():
    B, L, H, F = 2, 30, 2, 3
    d = small(16, B, L, H, F)
    r = rng_(17)
    dz_re = r.standard_normal((B, L, H * F)).astype(np.float32)
    dz_im = r.standard_normal((B, L, H * F)).astype(np.float32)
    g0 = O.phase_bwd(O.Cfg(B, L, H, F, gate_tau=0.0), d["mag"], d["ang"], d["gamma"], d["theta"],
                     dz_re, dz_im)
    tau = 0.5
    g1 = O.phase_bwd(O.Cfg(B, L, H, F, gate_tau=tau), d["mag"], d["ang"], d["gamma"], d["theta"],
                     dz_re, dz_im)
    mask = np.abs(d["mag"]) >= np.float32(tau)
    assert 0.2 < mask.mean() < 0.8
    assert np.array_equal(g1["dmag"], g0["dmag"])              # gradient as if no threshold
    assert np.array_equal(g1["dang"], mask * g0["dang"])
    assert not np.array_equal(g1["dgamma"], g0["dgamma"])      # the state itself did change


@pytest.mark.parametrize("tau,amp_mode", [(0.0, 0), (0.15, 0), (0.0, 1), (0.75, 1)])
def test_fused_backward_equals_numpy_chain(tau, amp_mode):
    # conv backward + STE with the gate active: rebuild every gradient from brute-force pieces.
    # amp_mode 1 (Sec. 3.3 item 1): a = min(softplus(x), 10) on the conv's output x, the threshold is taken
    # on that amplitude, and the chain to x carries sigmoid(x) below the cap
    B, L, H, F, Kc = 2, 14, 1, 3, 4
    J = H * F
    d = small(18, B, L, H, F, Kc)
    r = rng_(19)
    tail = r.standard_normal((B, Kc - 1, 2, J)).astype(np.float32)
    dz_re = r.standard_normal((B, L, J)).astype(np.float32)
    dz_im = r.standard_normal((B, L, J)).astype(np.float32)
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=tau, out_clamp=INF, grad_clamp=INF)
    fwd = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], conv_w=d["conv_w"],
                      conv_b=d["conv_b"], tail_in=tail)
    g = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], dz_re, dz_im,
                    conv_w=d["conv_w"], conv_b=d["conv_b"], tail_in=tail)
    lmb = lam(d["gamma"], d["theta"])
    G = brute_adjoint(dz_re.astype(np.float64) + 1j * dz_im, lmb)
    w = d["conv_w"].astype(np.float64)
    useq = [np.concatenate([tail[:, :, s], (d["mag"], d["ang"])[s]], axis=1).astype(np.float64)
            for s in range(2)]                                         # [B, Kc-1+L, J]
    z = [sum(w[s][None, None, :, i] * useq[s][:, i:i + L] for i in range(Kc)) + d["conv_b"][s]
         for s in range(2)]
    x, phi = np_silu(z[0]), np_silu(z[1])
    a = np.minimum(np.logaddexp(0.0, x), 10.0) if amp_mode == 1 else x
    dadx = np.where(np.logaddexp(0.0, x) < 10.0, np_sigmoid(x), 0.0) if amp_mode == 1 else 1.0
    gate = fwd["gate"].astype(np.float64)
    clear = np.abs(np.abs(a) - tau) > 1e-5         # away from ties the fp32 decision is the fp64 one
    assert np.array_equal(gate[clear], (np.abs(a) >= tau)[clear].astype(np.float64))
    if tau > 0:
        assert 0.1 < gate.mean() < 0.9
    e = np.exp(1j * phi)
    np.testing.assert_allclose(fwd["z_re"] + 1j * fwd["z_im"], brute_scan(gate * a * e, lmb), atol=1e-12)
    da = (np.conj(G) * e).real
    dphi = gate * a * (np.conj(G) * 1j * e).real
    dzc = [da * dadx * np_dsilu(z[0]), dphi * np_dsilu(z[1])]
    S = brute_scan(gate * a * e, lmb)
    Sprev = np.concatenate([np.zeros((B, 1, J)), S[:, :-1]], axis=1)
    np.testing.assert_allclose(g["dgamma"], (np.conj(G) * np.exp(1j * d["theta"].astype(np.float64)) * Sprev).real.sum((0, 1)), atol=1e-11)
    np.testing.assert_allclose(g["dtheta"], (np.conj(G) * 1j * lmb * Sprev).real.sum((0, 1)), atol=1e-11)
    for s, name in ((0, "dmag"), (1, "dang")):
        du = np.zeros((B, Kc - 1 + L, J))
        dw = np.zeros((J, Kc))
        for i in range(Kc):
            du[:, i:i + L] += w[s][None, None, :, i] * dzc[s]
            dw[:, i] = (dzc[s] * useq[s][:, i:i + L]).sum((0, 1))
        np.testing.assert_allclose(g[name], du[:, Kc - 1:], atol=1e-12)
        np.testing.assert_allclose(g["dtail_in"][:, :, s], du[:, :Kc - 1], atol=1e-12)
        np.testing.assert_allclose(g["dconv_w"][s], dw, atol=1e-11)
        np.testing.assert_allclose(g["dconv_b"][s], dzc[s].sum((0, 1)), atol=1e-11)


def test_impulse_closed_forms_for_retention_and_rotation_gradients():
    # one push p at t0, one unit of upstream gradient at t1: S_t1 = lambda^n p, n = t1 - t0
    L, t0, t1 = 20, 3, 15
    n = t1 - t0
    gamma = np.array([0.93], np.float32)
    theta = np.array([0.37], np.float32)
    mag = np.zeros((1, L, 1), np.float32); ang = np.zeros((1, L, 1), np.float32)
    mag[0, t0, 0], ang[0, t0, 0] = 1.25, 0.8
    p = 1.25 * np.exp(1j * float(np.float32(0.8)))
    lmb = lam(gamma, theta)[0]
    cfg = O.Cfg(1, L, 1, 1, out_clamp=INF, grad_clamp=INF)
    for (ur, ui) in ((1.0, 0.0), (0.0, 1.0)):
        dz_re = np.zeros((1, L, 1), np.float32); dz_im = np.zeros((1, L, 1), np.float32)
        dz_re[0, t1, 0], dz_im[0, t1, 0] = ur, ui
        g = O.phase_bwd(cfg, mag, ang, gamma, theta, dz_re, dz_im)
        dS_dgamma = n * float(gamma[0]) ** (n - 1) * np.exp(1j * n * float(theta[0])) * p
        dS_dtheta = 1j * n * lmb ** n * p
        pick = (lambda c: c.real) if ur else (lambda c: c.imag)
        np.testing.assert_allclose(g["dgamma"][0], pick(dS_dgamma), rtol=1e-12)
        np.testing.assert_allclose(g["dtheta"][0], pick(dS_dtheta), rtol=1e-12)


def test_gradient_clamp_by_hand():
    # L=2, gamma=1, theta=0, phi=0: G_1 = 150, G_0 = 300 -> returned dp clamps to 100;
    # dgamma terms: t=1: G_1 * S_0 = 150 * 2 = 300 -> 100; t=0: S_-1 = 0.
    mag = np.array([[[2.0], [1.0]]], np.float32)
    ang = np.zeros_like(mag)
    dz_re = np.full((1, 2, 1), 150.0, np.float32)
    dz_im = np.zeros_like(dz_re)
    one, zero = np.ones(1, np.float32), np.zeros(1, np.float32)
    g = O.phase_bwd(O.Cfg(1, 2, 1, 1, grad_clamp=100.0), mag, ang, one, zero, dz_re, dz_im)
    assert g["dmag"][0, :, 0].tolist() == [100.0, 100.0]
    assert g["dgamma"][0] == 100.0
    assert g["dscan_in"][0, 0, 0] == 300.0           # the carried adjoint is not clamped
    g = O.phase_bwd(O.Cfg(1, 2, 1, 1, grad_clamp=INF), mag, ang, one, zero, dz_re, dz_im)
    assert g["dmag"][0, :, 0].tolist() == [300.0, 150.0]
    assert g["dgamma"][0] == 300.0


def test_output_clamp_passes_gradient_straight_through():
    L = 60
    mag = np.full((1, L, 1), 5.0, np.float32)
    ang = np.zeros_like(mag)
    one, zero = np.ones(1, np.float32), np.zeros(1, np.float32)
    dz = np.ones((1, L, 1), np.float32)
    g = O.phase_bwd(O.Cfg(1, L, 1, 1, grad_clamp=INF), mag, ang, one, zero, dz, np.zeros_like(dz))
    # saturated from t = 19 on, yet every upstream unit still flows back: dmag_t = L - t
    np.testing.assert_allclose(g["dmag"][0, :, 0], np.arange(L, 0, -1.0))


def test_conv_clamp_blocks_gradient_outside_range():
    Kc = 1
    mag = np.array([[[60.0], [1.0], [-70.0]]], np.float32)
    ang = np.zeros_like(mag)
    w = np.ones((2, 1, 1), np.float32)
    dz = np.ones((1, 3, 1), np.float32)
    g = O.phase_bwd(O.Cfg(1, 3, 1, 1, conv_k=Kc, grad_clamp=INF), mag, ang, np.zeros(1, np.float32),
                    np.zeros(1, np.float32), dz, np.zeros_like(dz), conv_w=w,
                    conv_b=np.zeros((2, 1), np.float32))
    assert g["dmag"][0, 0, 0] == 0.0 and g["dmag"][0, 2, 0] == 0.0
    np.testing.assert_allclose(g["dmag"][0, 1, 0], math.cos(np_silu(0.0)) * np_dsilu(1.0), rtol=1e-13)


# -------------------------------------------------------------------------------------- theta_j
def test_softplus_cap_blocks_the_amplitude_gradient():
    """amp_mode 1 (Sec. 3.3 item 1): a = min(softplus(m), 10).  d a / d m = sigmoid(m) while softplus(m) < 10
    and 0 once the cap holds (m = 10 already gives softplus = 10.0000454).  One token, phi = 0, dz = 1: the
    returned dmag is that derivative itself."""
    ms = np.array([0.0, -2.0, 9.0, 9.99, 10.0, 20.0], np.float32)
    want = [0.5, 1 / (1 + math.exp(2.0)), 1 / (1 + math.exp(-9.0)), 1 / (1 + math.exp(-float(np.float32(9.99)))), 0.0, 0.0]
    for m, w in zip(ms, want):
        one = np.full((1, 1, 1), m, np.float32)
        g = O.phase_bwd(O.Cfg(1, 1, 1, 1, amp_mode=1), one, np.zeros_like(one), np.zeros(1, np.float32),
                        np.zeros(1, np.float32), np.ones_like(one), np.zeros_like(one))
        assert g["dmag"][0, 0, 0] == pytest.approx(w, rel=1e-14, abs=0)
    # the phase keeps its gradient at the cap: d/dphi of a sin(phi) . dz_im = a cos(phi) = 10 at phi = 0
    one = np.full((1, 1, 1), 20.0, np.float32)
    g = O.phase_bwd(O.Cfg(1, 1, 1, 1, amp_mode=1), one, np.zeros_like(one), np.zeros(1, np.float32),
                    np.zeros(1, np.float32), np.zeros_like(one), np.ones_like(one))
    assert g["dang"][0, 0, 0] == 10.0 and g["dmag"][0, 0, 0] == 0.0


def test_paper_layer_all_gradients_against_finite_differences():
    """The layer with everything the paper states switched on at once: conv kernel 3 (Sec. 3.2), softplus
    amplitude, per-head valve and data-dependent retention (Sec. 3.3).  With eps = 0 the valve's forward is its
    sigmoid, so the straight-through gradient is the exact derivative and central differences apply to every
    input, parameter and carried state."""
    B, L, H, F, Kc = 2, 8, 2, 3, 3
    J = H * F
    d = small(301, B, L, H, F, Kc)
    q = lambda a: (np.round(np.asarray(a, np.float64) * 1024) / 1024).astype(np.float32)
    for k in d:
        d[k] = q(d[k])
    r = rng_(302)
    valve = q(3.0 + 2.0 * r.standard_normal((B, L, H)))
    ret = q(0.5 + 1.5 * r.standard_normal((B, L, H)))
    bias = np.linspace(3.0, 0.0, F).astype(np.float32)
    scan_in = np.round(r.standard_normal((B, 2, J)) * 1024) / 1024
    tail_in = q(r.standard_normal((B, Kc - 1, 2, J)))
    up = dict(dz_re=r.standard_normal((B, L, J)).astype(np.float32), dz_im=r.standard_normal((B, L, J)).astype(np.float32),
              dscan_out=r.standard_normal((B, 2, J)), dtail_out=r.standard_normal((B, Kc - 1, 2, J)))
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=1, gate_mode=1, valve_eps=0.0, ret_mode=1, conv_clamp=INF,
                out_clamp=INF, grad_clamp=INF)
    arrs = dict(mag=d["mag"], ang=d["ang"], theta=d["theta"], conv_w=d["conv_w"], conv_b=d["conv_b"], valve=valve,
                ret=ret, scan_in=scan_in, tail_in=tail_in)

    def loss(a):
        f = O.phase_fwd(cfg, a["mag"], a["ang"], None, a["theta"], conv_w=a["conv_w"], conv_b=a["conv_b"],
                        scan_in=a["scan_in"], tail_in=a["tail_in"], valve=a["valve"], ret=a["ret"], ret_bias=bias,
                        want_gate=False)
        return float((up["dz_re"] * f["z_re"]).sum() + (up["dz_im"] * f["z_im"]).sum()
                     + (up["dscan_out"] * f["scan_out"]).sum() + (up["dtail_out"] * f["tail_out"]).sum())

    g = O.phase_bwd(cfg, d["mag"], d["ang"], None, d["theta"], up["dz_re"], up["dz_im"], conv_w=d["conv_w"],
                    conv_b=d["conv_b"], scan_in=scan_in, tail_in=tail_in, dscan_out=up["dscan_out"],
                    dtail_out=up["dtail_out"], valve=valve, ret=ret, ret_bias=bias)
    assert "dgamma" not in g
    names = dict(mag="dmag", ang="dang", theta="dtheta", conv_w="dconv_w", conv_b="dconv_b", valve="dvalve", ret="dret",
                 scan_in="dscan_in", tail_in="dtail_in")
    r2 = rng_(303)
    for name, gname in names.items():
        arr, grad = arrs[name], g[gname]
        assert grad.shape == arr.shape, name
        for f in r2.permutation(arr.size)[:8]:
            idx = np.unravel_index(f, arr.shape)

            def at(h):
                a2 = dict(arrs)
                a2[name] = arr.copy()
                a2[name][idx] += h
                return loss(a2)
            h = 2.0 ** -7
            d1 = (at(h) - at(-h)) / (2 * h)
            d2 = (at(h / 2) - at(-h / 2)) / h
            num = (4 * d2 - d1) / 3
            assert abs(num - grad[idx]) <= 3e-7 * max(1.0, abs(num)), (name, idx, num, grad[idx])


# ------------------------------------------------------- harmonic convolution, backward (Sec. 3.6)
def test_harmonic_conv_bwd_by_hand():
    """One head of four harmonics, taps (10, 1, 0.125) on the real plane, upstream (1, 0, 0, 2): position 0
    fed outputs 0 (centre) and 1 (lower tap), position 3 fed outputs 3 (centre) and 2 (upper tap), so
    dZ = (1, 0.125, 20, 2); d tap_i = sum_k up[k] Z[k + i - 1]; the bias receives the sum of its channel."""
    z = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 4)
    w = np.zeros((2, 1, 3), np.float32)
    w[0, 0] = [10.0, 1.0, 0.125]
    w[1, 0] = [0.0, 0.0, 1.0]
    up_re = np.array([1.0, 0.0, 0.0, 2.0]).reshape(1, 1, 4)
    up_im = np.array([0.0, 1.0, 0.0, 0.5]).reshape(1, 1, 4)
    g = O.harmonic_conv_bwd(z, 2 * z, 1, 4, w, up_re, up_im)
    np.testing.assert_array_equal(g["dz_re"][0, 0], [1.0, 0.125, 20.0, 2.0])
    np.testing.assert_array_equal(g["dz_im"][0, 0], [0.0, 0.0, 1.0, 0.0])      # output 1 read position 2; output 3 read nothing
    np.testing.assert_array_equal(g["dw"][0, 0], [2.0 * 3.0, 1.0 * 1.0 + 2.0 * 4.0, 1.0 * 2.0])
    np.testing.assert_array_equal(g["dw"][1, 0], [1.0 * 2.0 + 0.5 * 6.0, 1.0 * 4.0 + 0.5 * 8.0, 1.0 * 6.0])
    np.testing.assert_array_equal(g["dbias"], [[3.0], [1.5]])


@pytest.mark.parametrize("Kh", [1, 3, 5])
def test_harmonic_conv_bwd_is_the_adjoint_and_matches_library_routines(Kh):
    """<up, conv(Z) - bias> = <dZ, Z> for any up and Z (the transposed map); dZ is the correlation of up with the
    reversed taps (scipy, zero fill); the tap gradient is numpy's full cross-correlation of up and Z read at lags
    -pad .. pad; heads and planes stay apart."""
    from scipy.ndimage import correlate1d
    r = rng_(950 + Kh)
    B, L, H, F = 2, 4, 3, 8
    pad = (Kh - 1) // 2
    z = r.standard_normal((2, B, L, H * F))
    up = r.standard_normal((2, B, L, H * F))
    w = r.standard_normal((2, H, Kh)).astype(np.float32)
    bias = r.standard_normal((2, H)).astype(np.float32)
    o = O.harmonic_conv(z[0], z[1], H, F, w, bias)
    o0 = O.harmonic_conv(np.zeros_like(z[0]), np.zeros_like(z[1]), H, F, w, bias)
    g = O.harmonic_conv_bwd(z[0], z[1], H, F, w, up[0], up[1])
    for p_ in range(2):
        lhs = (up[p_] * (o[p_] - o0[p_])).sum()
        rhs = (g[("dz_re", "dz_im")[p_]] * z[p_]).sum()
        assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
        for h in range(H):
            sl = slice(h * F, (h + 1) * F)
            ref = correlate1d(up[p_][:, :, sl], w[p_, h, ::-1].astype(np.float64), axis=2, mode="constant", cval=0.0)
            np.testing.assert_allclose(g[("dz_re", "dz_im")[p_]][:, :, sl], ref, rtol=0, atol=1e-13)
            dw = np.zeros(Kh)
            for b in range(B):
                for t in range(L):
                    full = np.correlate(z[p_][b, t, sl], up[p_][b, t, sl], mode="full")   # lag s at index s + F - 1
                    dw += full[F - 1 - pad:F + pad]
            np.testing.assert_allclose(g["dw"][p_, h], dw, rtol=0, atol=1e-12)
            np.testing.assert_allclose(g["dbias"][p_, h], up[p_][:, :, sl].sum(), rtol=0, atol=1e-12)


def test_harmonic_conv_bwd_against_finite_differences():
    """The map is linear in Z and in (taps, bias): central differences are exact up to rounding."""
    r = rng_(960)
    B, L, H, F = 1, 3, 2, 5
    z = r.standard_normal((2, B, L, H * F))
    up = r.standard_normal((2, B, L, H * F))
    w = (np.round(r.standard_normal((2, H, 3)) * 256) / 256).astype(np.float32)
    bias = (np.round(r.standard_normal((2, H)) * 256) / 256).astype(np.float32)
    g = O.harmonic_conv_bwd(z[0], z[1], H, F, w, up[0], up[1])

    def loss(z_=z, w_=w, b_=bias):
        o = O.harmonic_conv(z_[0], z_[1], H, F, w_, b_)
        return float((o[0] * up[0]).sum() + (o[1] * up[1]).sum())

    for idx in [(0, 0, 0, 0), (1, 0, 2, 9), (0, 0, 1, 4), (1, 0, 1, 5)]:
        zp, zm = z.copy(), z.copy()
        zp[idx] += 0.25
        zm[idx] -= 0.25
        assert g[("dz_re", "dz_im")[idx[0]]][idx[1:]] == pytest.approx((loss(z_=zp) - loss(z_=zm)) / 0.5, rel=1e-12, abs=1e-12)
    for idx in [(0, 0, 0), (0, 1, 2), (1, 0, 1), (1, 1, 0)]:
        wp, wm = w.copy(), w.copy()
        wp[idx] += np.float32(0.25)
        wm[idx] -= np.float32(0.25)
        assert g["dw"][idx] == pytest.approx((loss(w_=wp) - loss(w_=wm)) / 0.5, rel=1e-12, abs=1e-12)
    for idx in [(0, 1), (1, 0)]:
        bp, bm = bias.copy(), bias.copy()
        bp[idx] += np.float32(0.25)
        bm[idx] -= np.float32(0.25)
        assert g["dbias"][idx] == pytest.approx((loss(b_=bp) - loss(b_=bm)) / 0.5, rel=1e-12, abs=1e-12)


def test_training_step_through_the_harmonic_conv_against_finite_differences():
    """The whole step: conv front-end, scan, clamp (inactive here), harmonic convolution, loss = <up, C>.  Backward
    = harmonic_conv_bwd, then phase_bwd on its fp64 dZ (cfg.dz_f64).  Central differences through the composed
    forward check the hand-over between the two (a dZ rounded to fp32 on the way would still pass this bar, a
    swapped plane, a transposed tap window or a missing term would not)."""
    B, L, H, F, Kc = 2, 7, 2, 4, 3
    J = H * F
    d = small(970, B, L, H, F, Kc)
    q = lambda a: (np.round(np.asarray(a, np.float64) * 1024) / 1024).astype(np.float32)
    for k in d:
        d[k] = q(d[k])
    r = rng_(971)
    hw = q(r.standard_normal((2, H, 3)))
    hb = q(r.standard_normal((2, H)))
    up = r.standard_normal((2, B, L, J))
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=0.0, conv_clamp=INF, out_clamp=INF, grad_clamp=INF)

    def loss(dd, hw_=hw, hb_=hb):
        f = O.phase_fwd(cfg, dd["mag"], dd["ang"], dd["gamma"], dd["theta"], conv_w=dd["conv_w"], conv_b=dd["conv_b"],
                        want_gate=False)
        c = O.harmonic_conv(f["z_re"], f["z_im"], H, F, hw_, hb_)
        return float((c[0] * up[0]).sum() + (c[1] * up[1]).sum())

    f = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], conv_w=d["conv_w"], conv_b=d["conv_b"])
    gh = O.harmonic_conv_bwd(f["z_re"], f["z_im"], H, F, hw, up[0], up[1])
    cfg64 = O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=0.0, conv_clamp=INF, out_clamp=INF, grad_clamp=INF, dz_f64=1)
    g = O.phase_bwd(cfg64, d["mag"], d["ang"], d["gamma"], d["theta"], gh["dz_re"], gh["dz_im"], conv_w=d["conv_w"],
                    conv_b=d["conv_b"])
    # the fp64 hand-over differs from the fp32 one by rounding only
    g32 = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], gh["dz_re"].astype(np.float32),
                      gh["dz_im"].astype(np.float32), conv_w=d["conv_w"], conv_b=d["conv_b"])
    np.testing.assert_allclose(g["dmag"], g32["dmag"], rtol=0, atol=1e-5)
    assert not np.array_equal(g["dmag"], g32["dmag"])
    r2 = rng_(972)
    for name, gname in (("mag", "dmag"), ("ang", "dang"), ("gamma", "dgamma"), ("theta", "dtheta"),
                        ("conv_w", "dconv_w"), ("conv_b", "dconv_b")):
        arr, grad = d[name], g[gname]
        for fl in r2.permutation(arr.size)[:6]:
            idx = np.unravel_index(fl, arr.shape)

            def at(h):
                dd = dict(d)
                dd[name] = arr.copy()
                dd[name][idx] += h
                return loss(dd)
            h = 2.0 ** -7
            num = (4 * (at(h / 2) - at(-h / 2)) / h - (at(h) - at(-h)) / (2 * h)) / 3
            assert abs(num - grad[idx]) <= 3e-7 * max(1.0, abs(num)), (name, idx, num, grad[idx])
    hp, hm = hw.copy(), hw.copy()
    hp[1, 0, 2] += np.float32(0.125)
    hm[1, 0, 2] -= np.float32(0.125)
    assert gh["dw"][1, 0, 2] == pytest.approx((loss(d, hw_=hp) - loss(d, hw_=hm)) / 0.25, rel=1e-11)


def test_paper_layer_through_the_harmonic_conv_against_finite_differences():
    """Everything at once: conv kernel 3, softplus amplitude, per-head valve (eps = 0: the straight-through
    gradient is then the exact derivative), data-dependent retention (Sec. 3.2-3.4), the carried state, and the
    harmonic convolution of Sec. 3.6 behind it; loss = <up, C> + <dstate, state>.  Backward = harmonic_conv_bwd, then
    phase_bwd in the same modes on its fp64 dZ.  Central differences through the composed forward, on every input,
    parameter, logit and state."""
    B, L, H, F, Kc = 2, 7, 2, 4, 3
    J = H * F
    d = small(980, B, L, H, F, Kc)
    q = lambda a: (np.round(np.asarray(a, np.float64) * 1024) / 1024).astype(np.float32)
    for k in d:
        d[k] = q(d[k])
    r = rng_(981)
    valve = q(3.0 + 2.0 * r.standard_normal((B, L, H)))
    ret = q(0.5 + 1.5 * r.standard_normal((B, L, H)))
    bias = np.linspace(3.0, 0.0, F).astype(np.float32)
    scan_in = np.round(r.standard_normal((B, 2, J)) * 1024) / 1024
    tail_in = q(r.standard_normal((B, Kc - 1, 2, J)))
    hw = q(r.standard_normal((2, H, 3)))
    hb = q(r.standard_normal((2, H)))
    up = r.standard_normal((2, B, L, J))
    dscan_out, dtail_out = r.standard_normal((B, 2, J)), r.standard_normal((B, Kc - 1, 2, J))
    kw = dict(conv_k=Kc, amp_mode=1, gate_mode=1, valve_eps=0.0, ret_mode=1, conv_clamp=INF, out_clamp=INF, grad_clamp=INF)
    cfg = O.Cfg(B, L, H, F, **kw)
    arrs = dict(mag=d["mag"], ang=d["ang"], theta=d["theta"], conv_w=d["conv_w"], conv_b=d["conv_b"], valve=valve,
                ret=ret, scan_in=scan_in, tail_in=tail_in, hconv_w=hw)

    def fwd(a):
        return O.phase_fwd(cfg, a["mag"], a["ang"], None, a["theta"], conv_w=a["conv_w"], conv_b=a["conv_b"],
                           scan_in=a["scan_in"], tail_in=a["tail_in"], valve=a["valve"], ret=a["ret"], ret_bias=bias,
                           want_gate=False)

    def loss(a):
        f = fwd(a)
        c = O.harmonic_conv(f["z_re"], f["z_im"], H, F, a["hconv_w"], hb)
        return float((c[0] * up[0]).sum() + (c[1] * up[1]).sum() + (dscan_out * f["scan_out"]).sum()
                     + (dtail_out * f["tail_out"]).sum())

    f = fwd(arrs)
    gh = O.harmonic_conv_bwd(f["z_re"], f["z_im"], H, F, hw, up[0], up[1])
    g = O.phase_bwd(O.Cfg(B, L, H, F, dz_f64=1, **kw), d["mag"], d["ang"], None, d["theta"], gh["dz_re"], gh["dz_im"],
                    conv_w=d["conv_w"], conv_b=d["conv_b"], scan_in=scan_in, tail_in=tail_in, dscan_out=dscan_out,
                    dtail_out=dtail_out, valve=valve, ret=ret, ret_bias=bias)
    g["dhconv_w"] = gh["dw"]
    names = dict(mag="dmag", ang="dang", theta="dtheta", conv_w="dconv_w", conv_b="dconv_b", valve="dvalve", ret="dret",
                 scan_in="dscan_in", tail_in="dtail_in", hconv_w="dhconv_w")
    r2 = rng_(982)
    for name, gname in names.items():
        arr, grad = arrs[name], g[gname]
        assert grad.shape == arr.shape, name
        for fl in r2.permutation(arr.size)[:6]:
            idx = np.unravel_index(fl, arr.shape)

            def at(h):
                a2 = dict(arrs)
                a2[name] = arr.copy()
                a2[name][idx] += h
                return loss(a2)
            h = 2.0 ** -7
            num = (4 * (at(h / 2) - at(-h / 2)) / h - (at(h) - at(-h)) / (2 * h)) / 3
            assert abs(num - grad[idx]) <= 3e-7 * max(1.0, abs(num)), (name, idx, num, grad[idx])
    # the biases' gradient is the sum of their channel's upstream gradients
    np.testing.assert_allclose(gh["dbias"], up.reshape(2, B, L, H, F).sum(axis=(1, 2, 4)), rtol=1e-12)


# ------------------------------------------------------------------------- per-head valve (mode 1)
def np_sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def test_valve_brute_force_and_mask():
    """gate_mode 1 (Sec. 3.3 "Hard-Threshold Gating", Sec. 3.4 gated-push equations): every lane of
    head h pushes beta_hard[t,h] * a * e^{i phi}; beta_sig = sigmoid(v - 3), closed below eps."""
    B, L, H, F = 2, 30, 3, 4
    d = small(31, B, L, H, F)
    r = rng_(32)
    valve = (3.0 + 4.0 * r.standard_normal((B, L, H))).astype(np.float32)   # beta_sig from ~0 to ~1
    eps = 0.2                                                              # closes a good fraction
    cfg = O.Cfg(B, L, H, F, gate_mode=1, valve_eps=eps, gate_tau=5.0, out_clamp=INF)   # tau plays no part
    out = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], valve=valve)
    bsig = np_sigmoid(valve.astype(np.float64) - 3.0)
    opened = bsig >= np.float64(np.float32(eps))
    assert 0.2 < opened.mean() < 0.8
    beta = np.where(opened, bsig, 0.0)
    p = np.repeat(beta, F, axis=2) * d["mag"].astype(np.float64) * np.exp(1j * d["ang"].astype(np.float64))
    S = brute_scan(p, lam(d["gamma"], d["theta"]))
    np.testing.assert_allclose(out["z_re"], S.real, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["z_im"], S.imag, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(out["gate"], np.repeat(opened, F, axis=2).astype(np.uint8))


def test_valve_half_open_by_hand_and_threshold_edge():
    # v = 3 -> beta = sigmoid(0) = 1/2: one token, Z = a/2 e^{i phi}
    cfg = O.Cfg(1, 1, 1, 1, gate_mode=1, out_clamp=INF)
    one = lambda v: np.full((1, 1, 1), v, dtype=np.float32)
    out = O.phase_fwd(cfg, one(1.5), one(0.25), one(0.9)[0, 0], one(0.1)[0, 0], valve=one(3.0))
    assert out["z_re"][0, 0, 0] == pytest.approx(0.75 * math.cos(0.25), abs=1e-15)
    assert out["z_im"][0, 0, 0] == pytest.approx(0.75 * math.sin(0.25), abs=1e-15)
    # the paper's eps = 0.001 closes the valve exactly where sigmoid(v - 3) < 0.001, i.e. below
    # v* = 3 + ln(0.001 / 0.999); the fp32 neighbours of v* fall on either side (keep when >=)
    vstar = 3.0 + math.log(0.001 / 0.999)
    lo = np.nextafter(np.float32(vstar), np.float32(-INF))
    hi = np.nextafter(np.float32(vstar), np.float32(INF))
    assert float(lo) < vstar < float(hi) or float(lo) <= vstar <= float(hi)
    cfg = O.Cfg(1, 1, 1, 1, gate_mode=1, valve_eps=0.001, out_clamp=INF)
    z_lo = O.phase_fwd(cfg, one(1.0), one(0.0), one(0.9)[0, 0], one(0.1)[0, 0], valve=one(lo - np.float32(1e-4)))
    z_hi = O.phase_fwd(cfg, one(1.0), one(0.0), one(0.9)[0, 0], one(0.1)[0, 0], valve=one(hi + np.float32(1e-4)))
    assert z_lo["z_re"][0, 0, 0] == 0.0 and z_lo["gate"][0, 0, 0] == 0
    assert z_hi["z_re"][0, 0, 0] == pytest.approx(0.001, rel=2e-4) and z_hi["gate"][0, 0, 0] == 1


def test_valve_gradients_against_numpy_chain_and_finite_differences():
    """Backward of gate_mode 1: da carries beta_hard, dphi carries beta_hard a, and the valve logit
    receives beta_sig (1 - beta_sig) * sum_k a_k Re(conj(G_k) e^{i phi_k}) whatever the threshold did
    (Sec. 3.3: beta = beta_hard - sg(beta_sig) + beta_sig).  The adjoint G does not depend on
    beta, so that gradient equals the exact derivative of the un-thresholded forward: checked by
    central differences of the eps = 0 forward."""
    B, L, H, F = 2, 14, 2, 3
    J = H * F
    d = small(41, B, L, H, F)
    r = rng_(42)
    valve = (3.0 + 3.0 * r.standard_normal((B, L, H))).astype(np.float32)
    dz = r.standard_normal((2, B, L, J)).astype(np.float32)
    eps = 0.3
    cfg = O.Cfg(B, L, H, F, gate_mode=1, valve_eps=eps, out_clamp=INF, grad_clamp=INF)
    g = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], dz[0], dz[1], valve=valve)
    # numpy chain
    bsig = np_sigmoid(valve.astype(np.float64) - 3.0)
    beta = np.repeat(np.where(bsig >= np.float64(np.float32(eps)), bsig, 0.0), F, axis=2)
    G = brute_adjoint(dz[0].astype(np.float64) + 1j * dz[1].astype(np.float64), lam(d["gamma"], d["theta"]))
    a = d["mag"].astype(np.float64)
    e = np.exp(1j * d["ang"].astype(np.float64))
    re = (np.conj(G) * e).real            # Re(conj(G) e^{i phi})
    np.testing.assert_allclose(g["dmag"], beta * re, atol=1e-12)
    np.testing.assert_allclose(g["dang"], beta * a * (np.conj(G) * 1j * e).real, atol=1e-12)
    want = bsig * (1 - bsig) * (a * re).reshape(B, L, H, F).sum(axis=3)
    np.testing.assert_allclose(g["dvalve"], want, atol=1e-12)
    assert (np.abs(g["dvalve"][np.where(bsig < eps)]) > 1e-6).any()      # closed valves still learn
    # finite differences of the soft forward
    soft = O.Cfg(B, L, H, F, gate_mode=1, valve_eps=0.0, out_clamp=INF)

    def loss(v):
        o = O.phase_fwd(soft, d["mag"], d["ang"], d["gamma"], d["theta"], valve=v, want_gate=False)
        return float((o["z_re"] * dz[0]).sum() + (o["z_im"] * dz[1]).sum())

    h = 2.0 ** -6          # exactly representable steps around fp32 logits
    for (b, t, hh) in [(0, 0, 0), (1, 5, 1), (0, 13, 1), (1, 9, 0)]:
        vp = valve.copy(); vm = valve.copy()
        vp[b, t, hh] += np.float32(h); vm[b, t, hh] -= np.float32(h)
        fd = (loss(vp) - loss(vm)) / (float(vp[b, t, hh]) - float(vm[b, t, hh]))
        assert g["dvalve"][b, t, hh] == pytest.approx(fd, rel=2e-3, abs=1e-6)


def test_valve_full_open_reduces_to_the_ungated_path():
    # beta_sig -> 1 for a large logit (sigmoid(37) = 1 - 9e-17): same result as mode 0 with tau = 0
    B, L, H, F, Kc = 1, 20, 2, 4, 3
    d = small(51, B, L, H, F, Kc)
    valve = np.full((B, L, H), 40.0, dtype=np.float32)
    a = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc, gate_mode=1), d["mag"], d["ang"], d["gamma"], d["theta"],
                    d["conv_w"], d["conv_b"], valve=valve)
    b = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=0.0), d["mag"], d["ang"], d["gamma"], d["theta"],
                    d["conv_w"], d["conv_b"])
    np.testing.assert_allclose(a["z_re"], b["z_re"], rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(a["z_im"], b["z_im"], rtol=1e-14, atol=1e-14)


def _ret_inputs(seed, B, L, H, F):
    r = rng_(seed)
    ret = (-0.5 + 1.5 * r.standard_normal((B, L, H))).astype(np.float32)
    bias = np.linspace(3.0, 0.0, F).astype(np.float32)          # Sec. 3.3: b_k falls from +3 to 0
    gam = np_sigmoid(ret.astype(np.float64)[..., None] + bias.astype(np.float64)).reshape(B, L, H * F)
    return ret, bias, gam


def test_retention_brute_force_sum_with_per_token_decay():
    """ret_mode 1 (Sec. 3.3 item 4, accumulation equations with gamma_{t,j}):
    S_t = sum_{s<=t} p_s e^{i theta (t-s)} prod_{r=s+1..t} gamma_r: the retention of token r scales
    what arrives from r-1, so a push is never scaled by its own token's retention."""
    B, L, H, F = 2, 19, 2, 3
    J = H * F
    d = small(61, B, L, H, F)
    ret, bias, gam = _ret_inputs(62, B, L, H, F)
    s_in = rng_(63).standard_normal((B, 2, J))
    o = O.phase_fwd(O.Cfg(B, L, H, F, ret_mode=1, out_clamp=INF), d["mag"], d["ang"], None, d["theta"],
                    scan_in=s_in, ret=ret, ret_bias=bias)
    p = d["mag"].astype(np.float64) * np.exp(1j * d["ang"].astype(np.float64))
    th = d["theta"].astype(np.float64)
    want = np.zeros((B, L, J), dtype=complex)
    for t in range(L):
        for s in range(-1, t + 1):
            src = (s_in[:, 0] + 1j * s_in[:, 1]) if s < 0 else p[:, s]
            decay = np.ones((B, J))
            for r in range(s + 1, t + 1):
                decay = decay * gam[:, r]
            want[:, t] += src * decay * np.exp(1j * th * (t - s))
    np.testing.assert_allclose(o["z_re"], want.real, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o["z_im"], want.imag, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o["scan_out"][:, 0], want[:, -1].real, rtol=1e-12, atol=1e-12)


def test_retention_two_tokens_by_hand_and_bias_runs_over_harmonics():
    # one head, two harmonics, theta = 0, unit pushes: S_1 = 1 + sigmoid(r_1 + b_k), r_0 plays no role
    B, L, H, F = 1, 2, 1, 2
    mag = np.ones((B, L, 2), np.float32)
    ang = np.zeros((B, L, 2), np.float32)
    ret = np.array([[[5.0], [-1.0]]], np.float32)
    bias = np.array([3.0, 0.0], np.float32)
    o = O.phase_fwd(O.Cfg(B, L, H, F, ret_mode=1), mag, ang, None, np.zeros(2, np.float32), ret=ret, ret_bias=bias)
    assert o["z_re"][0, 0].tolist() == [1.0, 1.0]
    assert o["z_re"][0, 1, 0] == pytest.approx(1.0 + 1.0 / (1.0 + math.exp(-2.0)), rel=1e-15)   # 1.8807970779778824
    assert o["z_re"][0, 1, 1] == pytest.approx(1.0 + 1.0 / (1.0 + math.exp(1.0)), rel=1e-15)    # 1.2689414213699951
    # two heads: the bias index is the harmonic k = j mod F, the logit index the head h = j div F
    H = 2
    mag = np.ones((B, L, 4), np.float32); ang = np.zeros((B, L, 4), np.float32)
    ret = np.array([[[0.0, 0.0], [-1.0, 2.0]]], np.float32)
    o = O.phase_fwd(O.Cfg(B, L, H, F, ret_mode=1), mag, ang, None, np.zeros(4, np.float32), ret=ret, ret_bias=bias)
    want = [1 + 1 / (1 + math.exp(-2.0)), 1 + 1 / (1 + math.exp(1.0)), 1 + 1 / (1 + math.exp(-5.0)), 1 + 1 / (1 + math.exp(-2.0))]
    np.testing.assert_allclose(o["z_re"][0, 1], want, rtol=1e-15)


def test_retention_constant_logit_reduces_to_constant_gamma():
    # logits chosen so that sigmoid(r + b_k) is a dyadic number: the constant-gamma path gets it exactly
    B, L, H, F, Kc = 2, 40, 2, 2, 3
    d = small(71, B, L, H, F, Kc)
    bias = np.zeros(F, np.float32)
    ret = np.zeros((B, L, H), np.float32)                  # sigmoid(0) = 0.5 exactly
    gamma = np.full(H * F, 0.5, np.float32)
    a = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc, ret_mode=1), d["mag"], d["ang"], None, d["theta"], d["conv_w"],
                    d["conv_b"], ret=ret, ret_bias=bias)
    b = O.phase_fwd(O.Cfg(B, L, H, F, conv_k=Kc), d["mag"], d["ang"], gamma, d["theta"], d["conv_w"], d["conv_b"])
    assert np.array_equal(a["z_re"], b["z_re"]) and np.array_equal(a["z_im"], b["z_im"])
    dz = rng_(72).standard_normal((2, B, L, H * F)).astype(np.float32)
    ga = O.phase_bwd(O.Cfg(B, L, H, F, conv_k=Kc, ret_mode=1), d["mag"], d["ang"], None, d["theta"], dz[0], dz[1],
                     d["conv_w"], d["conv_b"], ret=ret, ret_bias=bias)
    gb = O.phase_bwd(O.Cfg(B, L, H, F, conv_k=Kc), d["mag"], d["ang"], gamma, d["theta"], dz[0], dz[1],
                     d["conv_w"], d["conv_b"])
    for k in ("dmag", "dang", "dtheta", "dconv_w", "dconv_b", "dscan_in"):
        assert np.array_equal(ga[k], gb[k]), k
    assert "dgamma" not in ga


def test_retention_chunked_equals_unchunked_bitwise():
    B, L, H, F = 2, 33, 2, 3
    d = small(81, B, L, H, F)
    ret, bias, _ = _ret_inputs(82, B, L, H, F)
    full = O.phase_fwd(O.Cfg(B, L, H, F, ret_mode=1), d["mag"], d["ang"], None, d["theta"], ret=ret, ret_bias=bias)
    st, outs = None, []
    for lo, hi in ((0, 7), (7, 8), (8, 33)):
        o = O.phase_fwd(O.Cfg(B, hi - lo, H, F, ret_mode=1), d["mag"][:, lo:hi], d["ang"][:, lo:hi], None, d["theta"],
                        scan_in=st, ret=ret[:, lo:hi], ret_bias=bias)
        st = o["scan_out"]
        outs.append(o["z_re"])
    assert np.array_equal(np.concatenate(outs, axis=1), full["z_re"])


def test_retention_gradients_numpy_chain_and_finite_differences():
    """Adjoint with per-token retention: G_t = dS_t + gamma_{t+1} conj(e^{i theta}) G_{t+1};
    d gamma_t = Re(conj(G_t) e^{i theta} S_{t-1}); d r[t][h] = sum_k d gamma_t gamma_t (1 - gamma_t);
    d S_in = gamma_0 conj(e^{i theta}) G_0.  Then every gradient against central differences."""
    B, L, H, F = 2, 12, 2, 3
    J = H * F
    d = small(91, B, L, H, F)
    ret, bias, gam = _ret_inputs(92, B, L, H, F)
    r = rng_(93)
    dz = r.standard_normal((2, B, L, J)).astype(np.float32)
    s_in = r.standard_normal((B, 2, J))
    ds_out = r.standard_normal((B, 2, J))
    cfg = O.Cfg(B, L, H, F, ret_mode=1, out_clamp=INF, grad_clamp=INF)
    g = O.phase_bwd(cfg, d["mag"], d["ang"], None, d["theta"], dz[0], dz[1], scan_in=s_in, dscan_out=ds_out,
                    ret=ret, ret_bias=bias)
    th = d["theta"].astype(np.float64)
    rot = np.exp(1j * th)
    p = d["mag"].astype(np.float64) * np.exp(1j * d["ang"].astype(np.float64))
    S = np.zeros((B, L + 1, J), dtype=complex)           # S[:, t+1] = S_t
    S[:, 0] = s_in[:, 0] + 1j * s_in[:, 1]
    for t in range(L):
        S[:, t + 1] = p[:, t] + gam[:, t] * rot * S[:, t]
    dS = dz[0].astype(np.float64) + 1j * dz[1].astype(np.float64)
    dS[:, L - 1] += ds_out[:, 0] + 1j * ds_out[:, 1]
    G = np.zeros((B, L, J), dtype=complex)
    for t in range(L - 1, -1, -1):
        G[:, t] = dS[:, t] + (gam[:, t + 1] * np.conj(rot) * G[:, t + 1] if t + 1 < L else 0.0)
    dgam = (np.conj(G) * rot * S[:, :L]).real
    np.testing.assert_allclose(g["dret"], (dgam * gam * (1 - gam)).reshape(B, L, H, F).sum(axis=3), atol=1e-11)
    np.testing.assert_allclose(g["dtheta"], (np.conj(G) * 1j * gam * rot * S[:, :L]).real.sum(axis=(0, 1)), atol=1e-10)
    m0 = gam[:, 0] * np.conj(rot) * G[:, 0]
    np.testing.assert_allclose(g["dscan_in"][:, 0], m0.real, atol=1e-12)
    np.testing.assert_allclose(g["dscan_in"][:, 1], m0.imag, atol=1e-12)
    np.testing.assert_allclose(g["dmag"], (np.conj(G) * np.exp(1j * d["ang"].astype(np.float64))).real, atol=1e-12)

    def loss(ret_=ret, mag_=d["mag"], theta_=d["theta"], s_in_=s_in):
        o = O.phase_fwd(O.Cfg(B, L, H, F, ret_mode=1, out_clamp=INF), mag_, d["ang"], None, theta_, scan_in=s_in_,
                        ret=ret_, ret_bias=bias, want_gate=False)
        return float((o["z_re"] * dz[0]).sum() + (o["z_im"] * dz[1]).sum()
                     + (o["scan_out"] * ds_out).sum())

    h = np.float32(2.0 ** -7)
    for (b, t, hh) in [(0, 0, 0), (1, 4, 1), (0, 11, 1), (1, 7, 0)]:
        rp = ret.copy(); rm = ret.copy()
        rp[b, t, hh] += h; rm[b, t, hh] -= h
        fd = (loss(ret_=rp) - loss(ret_=rm)) / (float(rp[b, t, hh]) - float(rm[b, t, hh]))
        assert g["dret"][b, t, hh] == pytest.approx(fd, rel=2e-3, abs=1e-6)
    for j in (0, 4):
        tp = d["theta"].copy(); tm = d["theta"].copy()
        tp[j] += h; tm[j] -= h
        fd = (loss(theta_=tp) - loss(theta_=tm)) / (float(tp[j]) - float(tm[j]))
        assert g["dtheta"][j] == pytest.approx(fd, rel=2e-3, abs=1e-6)
    sp = s_in.copy(); sp[1, 1, 2] += 1e-5
    sm = s_in.copy(); sm[1, 1, 2] -= 1e-5
    assert g["dscan_in"][1, 1, 2] == pytest.approx((loss(s_in_=sp) - loss(s_in_=sm)) / 2e-5, rel=1e-5, abs=1e-8)


def test_retention_gradient_term_is_clamped_before_the_sigmoid_chain():
    # one lane, one head: d gamma_1 = G_1 S_0 = 1000 * 1 -> clamped to 100, times gamma (1 - gamma)
    B, L, H, F = 1, 2, 1, 1
    mag = np.array([[[1.0], [0.0]]], np.float32)
    ang = np.zeros((B, L, 1), np.float32)
    dz_re = np.array([[[0.0], [1000.0]]], np.float32)
    ret = np.zeros((B, L, 1), np.float32)
    g = O.phase_bwd(O.Cfg(B, L, H, F, ret_mode=1, grad_clamp=100.0), mag, ang, None, np.zeros(1, np.float32), dz_re,
                    np.zeros_like(dz_re), ret=ret, ret_bias=np.zeros(1, np.float32))
    assert g["dret"][0, 1, 0] == 100.0 * 0.25
    assert g["dret"][0, 0, 0] == 0.0          # S_{-1} = 0


def test_theta_init_endpoints_and_ratio():
    H, F = 12, 64
    th = O.theta_init(H, F).astype(np.float64)
    assert th[0] == 1.0
    J = H * F
    np.testing.assert_allclose(th[1:] / th[:-1], 10000.0 ** (-2.0 / J), rtol=3e-7)
    np.testing.assert_allclose(th[-1], 10.0 ** (-8.0 * (J - 1) / J), rtol=1e-7)


# ---------------------------------------------------------------- harmonic convolution (Sec. 3.6)
def test_harmonic_conv_by_hand():
    """One head of four harmonics, taps (10, 1, 0.1): position k takes 10 x its lower neighbour, itself
    and 0.1 x its upper neighbour, zeros beyond both ends.  Flipped taps, a shifted window or a
    dropped bias each change the printed values."""
    z = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 4)
    w = np.zeros((2, 1, 3), np.float32)
    w[0, 0] = [10.0, 1.0, 0.125]
    w[1, 0] = [0.0, 0.0, 1.0]
    bias = np.array([[0.5], [-1.0]], np.float32)
    o_re, o_im = O.harmonic_conv(z, 2 * z, 1, 4, w, bias)
    np.testing.assert_array_equal(o_re[0, 0], [1.75, 12.875, 24.0, 34.5])
    np.testing.assert_array_equal(o_im[0, 0], [3.0, 5.0, 7.0, -1.0])


@pytest.mark.parametrize("Kh", [1, 3, 5])
def test_harmonic_conv_matches_library_correlation(Kh):
    """Against scipy's 1-D correlation with zero fill, channel by channel: every (plane, head) uses
    its own taps and bias, and nothing crosses from one head's harmonics into the next head's."""
    from scipy.ndimage import correlate1d
    r = rng_(900 + Kh)
    B, L, H, F = 2, 5, 3, 8
    z_re = r.standard_normal((B, L, H * F))
    z_im = r.standard_normal((B, L, H * F))
    w = r.standard_normal((2, H, Kh)).astype(np.float32)
    bias = r.standard_normal((2, H)).astype(np.float32)
    o_re, o_im = O.harmonic_conv(z_re, z_im, H, F, w, bias)
    for p_, (z, o) in enumerate(((z_re, o_re), (z_im, o_im))):
        for h in range(H):
            ref = correlate1d(z[:, :, h * F:(h + 1) * F], w[p_, h].astype(np.float64), axis=2,
                              mode="constant", cval=0.0) + float(bias[p_, h])
            np.testing.assert_allclose(o[:, :, h * F:(h + 1) * F], ref, rtol=0, atol=1e-13)


def test_harmonic_conv_is_numpy_convolution_with_flipped_taps():
    """The textbook convolution flips its kernel: np.convolve(z, taps reversed, 'same') is the same map."""
    r = rng_(911)
    F = 16
    z = r.standard_normal(F)
    w = r.standard_normal(3).astype(np.float32)
    o_re, o_im = O.harmonic_conv(z.reshape(1, 1, F), np.zeros((1, 1, F)), 1, F,
                                 np.stack([w, w]).reshape(2, 1, 3))
    np.testing.assert_allclose(o_re[0, 0], np.convolve(z, w[::-1].astype(np.float64), mode="same"), atol=1e-14)
    np.testing.assert_array_equal(o_im, 0.0)


def test_harmonic_conv_heads_and_planes_stay_apart():
    """An impulse on the last harmonic of head 0 (real plane) reaches harmonics F-2 and F-1 of head 0
    only; the centre tap alone is the identity; the bias shows on every position of its channel."""
    H, F = 2, 8
    z_re = np.zeros((1, 1, H * F))
    z_re[0, 0, F - 1] = 1.0
    w = np.zeros((2, H, 3), np.float32)
    w[0, 0] = [2.0, 3.0, 5.0]
    w[0, 1] = [7.0, 7.0, 7.0]
    w[1, :] = [9.0, 9.0, 9.0]
    o_re, o_im = O.harmonic_conv(z_re, np.zeros_like(z_re), H, F, w)
    want = np.zeros(H * F)
    want[F - 2], want[F - 1] = 5.0, 3.0       # position k sees the impulse at k+1 through tap 2
    np.testing.assert_array_equal(o_re[0, 0], want)
    np.testing.assert_array_equal(o_im, 0.0)
    ident = np.zeros((2, H, 3), np.float32)
    ident[:, :, 1] = 1.0
    bias = np.array([[1.0, 2.0], [3.0, 4.0]], np.float32)
    r = rng_(912)
    a, b = r.standard_normal((2, 3, H * F)), r.standard_normal((2, 3, H * F))
    o_re, o_im = O.harmonic_conv(a, b, H, F, ident, bias)
    np.testing.assert_array_equal(o_re, a + np.repeat(bias[0].astype(np.float64), F))
    np.testing.assert_array_equal(o_im, b + np.repeat(bias[1].astype(np.float64), F))


# ------------------------------------------------------------------------------- regression anchor
def test_oracle_matches_its_stored_samples():
    """tests/golden/cfg1_oracle_samples.txt was written by tests/golden/make_golden.py from the oracle
    alone (the paper prints no numeric example for this path).  It does not pin the oracle to the
    mathematics -- the tests above do -- it flags any later drift of the oracle's arithmetic."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = {(n, t, j): v for n, t, j, v in mod.samples()}
    stored = {}
    for line in open(os.path.join(here, "cfg1_oracle_samples.txt")):
        if line.startswith("#"):
            continue
        n, t, j, v = line.split()
        stored[(n, int(t), int(j))] = float(v)
    assert stored.keys() == now.keys()
    for k, v in stored.items():
        assert abs(now[k] - v) <= 1e-12 * max(1.0, abs(v)), (k, now[k], v)
