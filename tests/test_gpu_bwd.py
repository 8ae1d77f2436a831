"""GPU parity: libcawn backward (through the C ABI) against the fp64 oracle, element by element.

Bar: max relative error (rms-floored) <= 1e-4 for every returned gradient.  Parameter gradients are
sums in a fixed order: two runs must agree bitwise.
"""
import numpy as np
import pytest

from oracle import cawn_oracle as O
from paper_2604_04250_amd import workloads as WL

pytestmark = pytest.mark.gpu

TOL = 1e-4
INF = float("inf")


def _gpu():
    import gpu_util
    return gpu_util


def _inputs(B, L, H, F, Kc, seed, gamma=(0.9, 0.999), bias=True, dz_scale=1.0):
    r = np.random.Generator(np.random.PCG64(seed))
    J = H * F
    d = dict(mag=r.standard_normal((B, L, J), dtype=np.float32),
             ang=r.standard_normal((B, L, J), dtype=np.float32),
             gamma=r.uniform(gamma[0], gamma[1], J).astype(np.float32),
             theta=r.uniform(0, np.pi, J).astype(np.float32))
    kk = max(Kc, 1)
    d["conv_w"] = (r.standard_normal((2, J, kk)) / np.sqrt(kk)).astype(np.float32)
    d["conv_b"] = (0.1 * r.standard_normal((2, J))).astype(np.float32) if bias else np.zeros((2, J), np.float32)
    d["dz_re"] = (dz_scale * r.standard_normal((B, L, J))).astype(np.float32)
    d["dz_im"] = (dz_scale * r.standard_normal((B, L, J))).astype(np.float32)
    return d


def _check(B, L, H, F, Kc, d, tau=0.1, amp_mode=0, with_state=False, grad_clamp=100.0, conv_clamp=50.0, seed=1, **kw):
    G = _gpu()
    J = H * F
    scan_in = tail_in = blob = dscan = dtail = dblob = None
    if with_state:
        wl = WL.Workload("x", B, H, F, L, conv_k=Kc)
        scan_in, tail_in = WL.random_state(wl, seed=seed)
        dscan, dtail = WL.random_state(wl, seed=seed + 1)
        blob = G.pack_state(scan_in, tail_in if Kc > 1 else None)
        dblob = G.pack_state(dscan, dtail if Kc > 1 else None)
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=tau, grad_clamp=grad_clamp, conv_clamp=conv_clamp)
    ora = O.phase_bwd(cfg, d["mag"][:, :L], d["ang"][:, :L], d["gamma"], d["theta"], d["dz_re"][:, :L],
                      d["dz_im"][:, :L], conv_w=d["conv_w"], conv_b=d["conv_b"],
                      scan_in=None if scan_in is None else scan_in.astype(np.float64),
                      tail_in=tail_in if Kc > 1 else None,
                      dscan_out=None if dscan is None else dscan.astype(np.float64),
                      dtail_out=None if (dtail is None or Kc <= 1) else dtail.astype(np.float64))
    out = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=tau, grad_clamp=grad_clamp,
                        conv_clamp=conv_clamp, state_in=blob, dstate_out=dblob, **kw)
    errs = {}
    for k in ("dmag", "dang", "dgamma", "dtheta"):
        errs[k] = G.rel_err(out[k], ora[k])
    if Kc > 0:
        errs["dconv_w"] = G.rel_err(out["dconv_w"], ora["dconv_w"])
        errs["dconv_b"] = G.rel_err(out["dconv_b"], ora["dconv_b"])
    dsc, dtl = G.unpack_state(out["dstate_in"], B, J, Kc)
    errs["dscan_in"] = G.rel_err(dsc, ora["dscan_in"])
    if Kc > 1:
        errs["dtail_in"] = G.rel_err(dtl, ora["dtail_in"])
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, (bad, errs)
    return out, ora


def test_cfg1_tiny_fused_and_plain():
    wl = WL.CONFIGS["cfg1_tiny"]
    d = WL.make_inputs(wl)
    _check(wl.B, wl.L, wl.H, wl.F, wl.conv_k, d, tau=wl.gate_tau)
    _check(wl.B, wl.L, wl.H, wl.F, 0, d, tau=wl.gate_tau)
    _check(wl.B, wl.L, wl.H, wl.F, wl.conv_k, d, tau=wl.gate_tau, with_state=True)


@pytest.mark.parametrize("L", [1, 2, 3, 7, 8, 9, 63, 64, 65, 127, 128, 129, 257, 517, 1030])
@pytest.mark.parametrize("Kc", [0, 4])
def test_ragged_lengths_span_tiles(L, Kc):
    B, H, F = 2, 2, 16
    d = _inputs(B, L, H, F, Kc, 100 + L)
    _check(B, L, H, F, Kc, d, with_state=True)


@pytest.mark.parametrize("H,F", [(12, 64), (1, 100), (3, 11), (1, 1), (2, 130)])
def test_lane_counts_vector_and_scalar_paths(H, F):
    B, L, Kc = 2, 200, 4
    d = _inputs(B, L, H, F, Kc, 200 + H * F)
    _check(B, L, H, F, Kc, d, tau=0.25, with_state=True)


@pytest.mark.parametrize("Kc", [1, 2, 3])
def test_conv_tap_counts(Kc):
    B, L, H, F = 2, 150, 2, 32
    d = _inputs(B, L, H, F, Kc, 300 + Kc)
    _check(B, L, H, F, Kc, d, with_state=True)


def test_clamps_off_is_the_plain_adjoint():
    B, L, H, F, Kc = 2, 300, 2, 32, 4
    d = _inputs(B, L, H, F, Kc, 400)
    _check(B, L, H, F, Kc, d, grad_clamp=INF, conv_clamp=INF)


def test_gradient_clamp_active_on_most_terms():
    # upstream gradients large enough that the adjoint and the parameter terms exceed +-100
    B, L, H, F, Kc = 2, 400, 2, 32, 4
    d = _inputs(B, L, H, F, Kc, 500, gamma=(0.99, 0.9999), dz_scale=20.0)
    out, ora = _check(B, L, H, F, Kc, d)
    free = O.phase_bwd(O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=0.1, grad_clamp=INF), d["mag"], d["ang"], d["gamma"],
                       d["theta"], d["dz_re"], d["dz_im"], conv_w=d["conv_w"], conv_b=d["conv_b"])
    assert np.abs(free["dgamma"] - ora["dgamma"]).max() > 1e3      # the clamp really changed the answer


def test_long_chain_high_retention():
    B, L, H, F = 1, 8192, 2, 32
    d = _inputs(B, L, H, F, 4, 600, gamma=(0.99, 0.9999))
    _check(B, L, H, F, 4, d)


@pytest.mark.parametrize("Kc", [0, 3])
def test_amplitude_softplus_mode(Kc):
    B, L, H, F = 2, 130, 2, 32
    d = _inputs(B, L, H, F, Kc, 700 + Kc)
    d["mag"] *= 6.0
    _check(B, L, H, F, Kc, d, tau=0.6, amp_mode=1, with_state=True)


def test_ste_on_gpu_amplitude_gradient_ignores_gate():
    G = _gpu()
    B, L, H, F = 2, 200, 2, 32
    d = _inputs(B, L, H, F, 0, 800)
    a = G.run_fwd_bwd(d, B, L, H, F, gate_tau=0.0)
    b = G.run_fwd_bwd(d, B, L, H, F, gate_tau=0.5)
    assert np.array_equal(a["dmag"], b["dmag"])
    mask = np.abs(d["mag"]) >= np.float32(0.5)
    assert np.array_equal(b["dang"], np.where(mask, a["dang"], np.float32(0.0)))


def test_parameter_gradients_repeatable_accumulate_and_optional():
    G = _gpu()
    B, L, H, F, Kc = 2, 700, 4, 32, 4
    d = _inputs(B, L, H, F, Kc, 900)
    a = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1)
    b = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1)
    for k in ("dmag", "dang", "dgamma", "dtheta", "dconv_w", "dconv_b", "dstate_in"):
        assert np.array_equal(a[k], b[k]), k
    c = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1, accumulate=1, preset=2.0)
    for k in ("dgamma", "dtheta", "dconv_w", "dconv_b"):
        assert np.array_equal(c[k], a[k] + np.float32(2.0)), k
    e = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1, want_param=False, want_dstate=False)
    assert G.rel_err(e["dmag"], a["dmag"]) <= 1e-6 and G.rel_err(e["dang"], a["dang"]) <= 1e-6


def test_chunked_backward_through_state_matches_one_pass():
    # BPTT across two calls: gradients of the second chunk's state_in feed the first chunk's dstate_out
    G = _gpu()
    B, L, H, F, Kc = 2, 300, 2, 32, 4
    J = H * F
    d = _inputs(B, L, H, F, Kc, 1000)
    full = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1, grad_clamp=INF)
    n1 = 170
    first = {k: (v[:, :n1] if v.ndim == 3 and v.shape[1] == L else v) for k, v in d.items()}
    second = {k: (v[:, n1:] if v.ndim == 3 and v.shape[1] == L else v) for k, v in d.items()}
    f1 = G.run_fwd(first, B, n1, H, F, conv_k=Kc, gate_tau=0.1, want_mask=False)
    b2 = G.run_fwd_bwd(second, B, L - n1, H, F, conv_k=Kc, gate_tau=0.1, grad_clamp=INF, state_in=f1["state_out"])
    b1 = G.run_fwd_bwd(first, B, n1, H, F, conv_k=Kc, gate_tau=0.1, grad_clamp=INF, dstate_out=b2["dstate_in"])
    assert G.rel_err(np.concatenate([b1["dmag"], b2["dmag"]], 1), full["dmag"]) <= TOL
    assert G.rel_err(np.concatenate([b1["dang"], b2["dang"]], 1), full["dang"]) <= TOL
    for k in ("dgamma", "dtheta", "dconv_w", "dconv_b"):
        assert G.rel_err(b1[k] + b2[k], full[k]) <= TOL, k


def test_zero_length_backward_passes_state_gradient_through():
    import torch
    G = _gpu()
    from paper_2604_04250_amd import binding as K
    B, H, F, Kc = 2, 2, 16, 4
    J = H * F
    d = K.make_desc(B, 0, H, F, conv_k=Kc)
    n = K.cawn_state_bytes(d) // 4
    dso = torch.randn(n, device=G.DEV)
    dsi = torch.full((n,), float("nan"), device=G.DEV)
    dg = torch.full((J,), 3.0, device=G.DEV)
    K.check(K.cawn_phase_accumulate_bwd(d, None, None, None, None, None, None, None, None, None, None, dso,
                                        None, None, dg, None, None, None, dsi, None))
    torch.cuda.synchronize()
    assert torch.equal(dsi, dso) and not dg.any()


@pytest.mark.parametrize("H,F,Kc", [(2, 64, 4), (3, 32, 0), (1, 24, 3)])
def test_concat_layout_inputs_outputs_and_their_gradients(H, F, Kc):
    """Sec. 3.5: Z is the concatenation of the real and the imaginary plane.  Here every activation pair
    shares rows of 2 J elements ([mag | ang], [Z_re | Z_im], and the gradients likewise): strided rows
    in the staging of the inputs and of the upstream gradients and in every store, with state."""
    B, L = 2, 333
    d = _inputs(B, L, H, F, Kc, 2600 + H + F + Kc)
    _check(B, L, H, F, Kc, d, with_state=True, concat=True)


@pytest.mark.parametrize("paper_modes", [False, True])
def test_training_step_replayed_from_a_hip_graph_matches_eager(paper_modes):
    """Forward (with checkpoints) and backward (every gradient) of one step captured in a HIP graph -- with the valve
    and the retention: their kernels and the epilogue's logit sums as well; three replays with eager work and
    synchronisation in between, each compared with the eager step bit for bit (same kernels, fixed summation
    orders).  The eager step itself is held to the oracle by the parity tests."""
    G = _gpu()
    import torch
    K = G.K
    B, L, H, F, Kc = 2, 700, 2, 64, 3
    J = H * F
    d = _inputs(B, L, H, F, Kc, 990)
    r = np.random.Generator(np.random.PCG64(991))
    dev = G.dev
    mag, ang, theta, cw, cb = (dev(d[k]) for k in ("mag", "ang", "theta", "conv_w", "conv_b"))
    gamma = None if paper_modes else dev(d["gamma"])
    valve = dev((-3.9 + 3.0 * r.standard_normal((B, L, H))).astype(np.float32)) if paper_modes else None
    ret = dev((-2.0 + 1.5 * r.standard_normal((B, L, H))).astype(np.float32)) if paper_modes else None
    rb = dev(np.linspace(3.0, 0.0, F).astype(np.float32)) if paper_modes else None
    dz_re, dz_im = dev(d["dz_re"]), dev(d["dz_im"])
    desc = K.make_desc(B, L, H, F, conv_k=Kc, amp_mode=1 if paper_modes else 0, gate_tau=0.1,
                       gate_mode=1 if paper_modes else 0, ret_mode=1 if paper_modes else 0)
    ws = G.Workspaces.get(desc)
    new = lambda *s: torch.full(s, float("nan"), device=G.DEV)
    z_re, z_im, dmag, dang = new(B, L, J), new(B, L, J), new(B, L, J), new(B, L, J)
    ckpt = new(max(K.cawn_ckpt_bytes(desc) // 4, 1))
    dgamma = None if paper_modes else new(J)
    dtheta, dcw, dcb = new(J), new(2, J, Kc), new(2, J)
    dvalve = new(B, L, H) if paper_modes else None
    dret = new(B, L, H) if paper_modes else None
    outs = [t for t in (z_re, z_im, dmag, dang, dgamma, dtheta, dcw, dcb, dvalve, dret) if t is not None]

    def step():
        if paper_modes:
            K.check(K.cawn_phase_accumulate_ret_fwd(desc, mag, ang, valve, ret, rb, theta, cw, cb, None, z_re, z_im, None,
                                                    ckpt, None, ws))
            K.check(K.cawn_phase_accumulate_ret_bwd(desc, mag, ang, valve, ret, rb, theta, cw, cb, None, ckpt, dz_re, dz_im,
                                                    None, dmag, dang, dvalve, dret, dtheta, dcw, dcb, None, ws))
        else:
            K.check(K.cawn_phase_accumulate_fwd(desc, mag, ang, gamma, theta, cw, cb, None, z_re, z_im, None, ckpt, None,
                                                ws))
            K.check(K.cawn_phase_accumulate_bwd(desc, mag, ang, gamma, theta, cw, cb, None, ckpt, dz_re, dz_im, None, dmag,
                                                dang, dgamma, dtheta, dcw, dcb, None, ws))

    step()                                  # (the first call of a kernel asks the runtime how many workgroups fit)
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    ref = [t.clone() for t in outs]
    assert all(bool(torch.isfinite(t).all()) for t in ref)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(3):
        for t in outs:
            t.fill_(float("nan"))           # eager work between the replays
        ckpt.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(x, y) for x, y in zip(outs, ref)), f"replay {rep} differs from eager"
    K.check(K.cawn_workspace_status(ws))
