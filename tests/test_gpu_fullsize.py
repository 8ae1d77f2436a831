"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run the whole tensors in seconds, but lanes are independent: for a sample of
lanes (first, last, and a spread over every lane block) the oracle computes the complete sequences,
outputs, state and per-lane parameter gradients, and those are compared element by element with the
same lanes of the full-size GPU run.  Bar: max relative error <= 1e-4 (rms-floored).
"""
import numpy as np
import pytest

from oracle import cawn_oracle as O
from paper_2604_04250_amd import workloads as WL

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _sample_lanes(J, n=24, seed=0):
    r = np.random.Generator(np.random.PCG64(seed))
    lanes = set([0, 1, J - 1, J - 2, 127 % J, 128 % J, 63 % J, 64 % J])
    while len(lanes) < min(n, J):
        lanes.add(int(r.integers(0, J)))
    return np.array(sorted(lanes))


def _sub(inp, lanes):
    out = {}
    for k, v in inp.items():
        if k in ("mag", "ang", "dz_re", "dz_im"):
            out[k] = np.ascontiguousarray(v[..., lanes])
        elif k in ("gamma", "theta"):
            out[k] = np.ascontiguousarray(v[lanes])
        elif k in ("conv_w",):
            out[k] = np.ascontiguousarray(v[:, lanes])
        elif k in ("conv_b",):
            out[k] = np.ascontiguousarray(v[:, lanes])
    return out


def _run_full(name, do_bwd):
    import torch
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS[name]
    B, L, H, F, J, Kc = wl.B, wl.L, wl.H, wl.F, wl.J, wl.conv_k
    theta = K.cawn_theta_init(H, F)
    assert np.array_equal(theta, O.theta_init(H, F))
    inp = WL.make_inputs(wl, theta=theta, with_grads=do_bwd)
    lanes = _sample_lanes(J)
    sub = _sub(inp, lanes)
    n = len(lanes)
    cfg = O.Cfg(B, L, 1, n, conv_k=Kc, gate_tau=wl.gate_tau)
    of = O.phase_fwd(cfg, sub["mag"], sub["ang"], sub["gamma"], sub["theta"], conv_w=sub["conv_w"], conv_b=sub["conv_b"])
    # GPU, exactly as bench.py launches it
    d = K.make_desc(B, L, H, F, conv_k=Kc, gate_tau=wl.gate_tau)
    dev = G.DEV
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in inp}
    z_re, z_im = torch.empty((B, L, J), device=dev), torch.empty((B, L, J), device=dev)
    ws = K.alloc_workspace(d, dev)
    ckpt = torch.empty(K.cawn_ckpt_bytes(d) // 4, device=dev)
    state = torch.empty(K.cawn_state_bytes(d) // 4, device=dev)
    W = (J + 31) // 32
    mask = torch.zeros((B, L, W), dtype=torch.int32, device=dev)
    K.check(K.cawn_phase_accumulate_fwd(d, t["mag"], t["ang"], t["gamma"], t["theta"], t["conv_w"], t["conv_b"], None,
                                        z_re, z_im, state, ckpt, mask, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    li = torch.from_numpy(lanes).to(dev)
    e = max(G.rel_err(z_re[..., li].cpu().numpy(), of["z_re"]), G.rel_err(z_im[..., li].cpu().numpy(), of["z_im"]))
    assert e <= TOL, e
    scan, tail = G.unpack_state(state.cpu().numpy(), B, J, Kc)
    assert G.rel_err(scan[..., lanes], of["scan_out"]) <= TOL
    assert np.array_equal(tail[..., lanes], of["tail_out"])
    # gate bits of the sampled lanes, bit-exact
    m = mask.cpu().numpy().view(np.uint32)
    bits = (m[..., lanes // 32] >> (lanes % 32).astype(np.uint32)) & 1
    assert np.array_equal(bits.astype(np.uint8), of["gate"])
    closed = 1.0 - of["gate"].mean()
    if not do_bwd:
        return closed
    ob = O.phase_bwd(cfg, sub["mag"], sub["ang"], sub["gamma"], sub["theta"], sub["dz_re"], sub["dz_im"],
                     conv_w=sub["conv_w"], conv_b=sub["conv_b"])
    dmag, dang = torch.empty((B, L, J), device=dev), torch.empty((B, L, J), device=dev)
    dg, dt = torch.empty(J, device=dev), torch.empty(J, device=dev)
    dcw, dcb = torch.empty((2, J, Kc), device=dev), torch.empty((2, J), device=dev)
    dst = torch.empty(K.cawn_state_bytes(d) // 4, device=dev)
    d.lane_consts_cached = 1
    K.check(K.cawn_phase_accumulate_bwd(d, t["mag"], t["ang"], t["gamma"], t["theta"], t["conv_w"], t["conv_b"], None,
                                        ckpt, t["dz_re"], t["dz_im"], None, dmag, dang, dg, dt, dcw, dcb, dst, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    errs = dict(dmag=G.rel_err(dmag[..., li].cpu().numpy(), ob["dmag"]),
                dang=G.rel_err(dang[..., li].cpu().numpy(), ob["dang"]),
                dgamma=G.rel_err(dg.cpu().numpy()[lanes], ob["dgamma"]),
                dtheta=G.rel_err(dt.cpu().numpy()[lanes], ob["dtheta"]),
                dconv_w=G.rel_err(dcw.cpu().numpy()[:, lanes], ob["dconv_w"]),
                dconv_b=G.rel_err(dcb.cpu().numpy()[:, lanes], ob["dconv_b"]))
    dsc, dtl = G.unpack_state(dst.cpu().numpy(), B, J, Kc)
    errs["dscan_in"] = G.rel_err(dsc[..., lanes], ob["dscan_in"])
    errs["dtail_in"] = G.rel_err(dtl[..., lanes], ob["dtail_in"])
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, (bad, errs)
    return closed


def test_cfg2_layer_forward_full_size():
    closed = _run_full("cfg2_layer_fwd", do_bwd=False)
    assert 0.0 < closed < 0.5       # the fused SiLU front-end changes the 7.97 % of the raw-input gate


def test_cfg3_training_step_full_size():
    _run_full("cfg3_train", do_bwd=True)


def test_cfg5_wide_full_size():
    _run_full("cfg5_wide", do_bwd=True)


def test_cfg6_paper_lane_shape_full_size():
    # 4 heads of 64 harmonics (the paper's own 150M model), the training-step batch
    _run_full("cfg6_paper_heads", do_bwd=True)


def test_cfg5_shape_without_conv_gates_20_percent():
    # threshold 0.25 on raw N(0,1) magnitudes: P(|m| < 0.25) = 19.74 % of lanes gated off
    import torch
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS["cfg5_wide"].with_(L=2048)
    B, L, H, F, J = wl.B, wl.L, wl.H, wl.F, wl.J
    inp = WL.make_inputs(wl, theta=K.cawn_theta_init(H, F), with_grads=False)
    out = G.run_fwd(inp, B, L, H, F, conv_k=0, gate_tau=wl.gate_tau)
    bits = np.unpackbits(out["mask"].view(np.uint8), bitorder="little").reshape(B, L, -1)[..., :J]
    expect = np.abs(inp["mag"]) >= np.float32(wl.gate_tau)
    assert np.array_equal(bits.astype(bool), expect)
    assert abs((1 - bits.mean()) - 0.1974) < 0.002


def test_cfg4_streaming_two_million_tokens_constant_memory():
    """2,000,000 tokens in 4096-token chunks (+ a 1,152-token tail), state carried in place on the
    device, inputs from a rotating pool of chunks; oracle over the same 2 M tokens for sampled lanes."""
    import torch
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS["cfg4_stream"]
    B, H, F, J, Kc, Lc = wl.B, wl.H, wl.F, wl.J, wl.conv_k, wl.chunk
    P = 8
    theta = K.cawn_theta_init(H, F)
    pool = WL.make_inputs(wl, theta=theta, with_grads=False, L=P * Lc)        # P chunks, drawn once
    nfull, rem = divmod(wl.L, Lc)
    assert (nfull, rem) == (488, 1152)
    lanes = _sample_lanes(J, n=12)
    # the oracle's view: the pool chunks in the order the stream visits them
    order = [c % P for c in range(nfull + 1)]
    seq = lambda k: np.concatenate([pool[k][:, o * Lc:(o + 1) * Lc][..., lanes] for o in order], axis=1)[:, :wl.L]
    cfg = O.Cfg(B, wl.L, 1, len(lanes), conv_k=Kc, gate_tau=wl.gate_tau)
    ora = O.phase_fwd(cfg, seq("mag"), seq("ang"), pool["gamma"][lanes], theta[lanes],
                      conv_w=np.ascontiguousarray(pool["conv_w"][:, lanes]),
                      conv_b=np.ascontiguousarray(pool["conv_b"][:, lanes]), want_gate=False)
    dev = G.DEV
    t = {k: torch.from_numpy(pool[k]).to(dev) for k in ("mag", "ang", "gamma", "conv_w", "conv_b")}
    th = torch.from_numpy(theta).to(dev)
    zs = [(torch.empty((B, Lc, J), device=dev), torch.empty((B, Lc, J), device=dev)) for _ in range(P)]
    d = K.make_desc(B, Lc, H, F, conv_k=Kc, gate_tau=wl.gate_tau)
    d_tail = K.make_desc(B, rem, H, F, conv_k=Kc, gate_tau=wl.gate_tau, lane_consts_cached=1)
    ws = K.alloc_workspace(d, dev)
    state = torch.zeros(K.cawn_state_bytes(d) // 4, device=dev)
    li = torch.from_numpy(lanes).to(dev)
    keep = {0: None, nfull // 2: None, nfull - 1: None, nfull: None}
    torch.cuda.synchronize()
    mem0 = torch.cuda.memory_allocated()
    for c in range(nfull + 1):
        o = order[c]
        dd = d if c < nfull else d_tail
        n = Lc if c < nfull else rem
        zr, zi = zs[c % P]
        K.check(K.cawn_phase_accumulate_fwd(dd, t["mag"][:, o * Lc:o * Lc + n], t["ang"][:, o * Lc:o * Lc + n],
                                            t["gamma"], th, t["conv_w"], t["conv_b"], state, zr, zi, state, None,
                                            None, ws))
        d.lane_consts_cached = 1
        if c in keep:
            keep[c] = (zr[:, :n][..., li].cpu().numpy(), zi[:, :n][..., li].cpu().numpy())
        assert torch.cuda.memory_allocated() <= mem0 + (1 << 20)       # nothing grows with the stream
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    for c, (zr, zi) in keep.items():
        sl = slice(c * Lc, c * Lc + zr.shape[1])
        assert G.rel_err(zr, ora["z_re"][:, sl]) <= TOL, c
        assert G.rel_err(zi, ora["z_im"][:, sl]) <= TOL, c
    scan, tail = G.unpack_state(state.cpu().numpy(), B, J, Kc)
    assert G.rel_err(scan[..., lanes], ora["scan_out"]) <= TOL
    assert np.array_equal(tail[..., lanes], ora["tail_out"])


@pytest.mark.parametrize("valve,ret", [(True, False), (False, True), (True, True)])
def test_cfg3_training_step_full_size_valve_and_retention(valve, ret):
    """The training-step shape with the per-head valve (Sec. 3.3 "Hard-Threshold Gating"), the
    data-dependent retention (Sec. 3.3 item 4) and both, launched as bench.py --valve / --ret launches
    them.  Heads are independent: the oracle computes two whole heads (all their lanes, so that the
    per-head logit gradients are complete) over the full sequences."""
    import torch
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS["cfg3_train"]
    B, L, H, F, J, Kc = wl.B, wl.L, wl.H, wl.F, wl.J, wl.conv_k
    theta = K.cawn_theta_init(H, F)
    inp = WL.make_inputs(wl, theta=theta, with_grads=True)
    r = np.random.Generator(np.random.PCG64(4250 + 97))
    vlog = (-3.9 + 3.0 * r.standard_normal((B, L, H))).astype(np.float32)
    rlog = (-2.0 + 1.5 * r.standard_normal((B, L, H))).astype(np.float32)
    rbias = np.linspace(3.0, 0.0, F).astype(np.float32)
    dev = G.DEV
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in inp}
    tv, tr, tb = (torch.from_numpy(x).to(dev) for x in (vlog, rlog, rbias))
    d = K.make_desc(B, L, H, F, conv_k=Kc, gate_tau=wl.gate_tau, gate_mode=1 if valve else 0, ret_mode=1 if ret else 0)
    ws = K.alloc_workspace(d, dev)
    z_re, z_im = torch.empty((B, L, J), device=dev), torch.empty((B, L, J), device=dev)
    ckpt = torch.empty(K.cawn_ckpt_bytes(d) // 4, device=dev)
    dmag, dang = torch.empty((B, L, J), device=dev), torch.empty((B, L, J), device=dev)
    dg, dt = torch.empty(J, device=dev), torch.empty(J, device=dev)
    dcw, dcb = torch.empty((2, J, Kc), device=dev), torch.empty((2, J), device=dev)
    dvalve = torch.empty((B, L, H), device=dev) if valve else None
    dret = torch.empty((B, L, H), device=dev) if ret else None
    if ret:
        K.check(K.cawn_phase_accumulate_ret_fwd(d, t["mag"], t["ang"], tv if valve else None, tr, tb, t["theta"], t["conv_w"],
                                                t["conv_b"], None, z_re, z_im, None, ckpt, None, ws))
        d.lane_consts_cached = 1
        K.check(K.cawn_phase_accumulate_ret_bwd(d, t["mag"], t["ang"], tv if valve else None, tr, tb, t["theta"], t["conv_w"],
                                                t["conv_b"], None, ckpt, t["dz_re"], t["dz_im"], None, dmag, dang, dvalve,
                                                dret, dt, dcw, dcb, None, ws))
    else:
        K.check(K.cawn_phase_accumulate_valve_fwd(d, t["mag"], t["ang"], tv, t["gamma"], t["theta"], t["conv_w"], t["conv_b"],
                                                  None, z_re, z_im, None, ckpt, None, ws))
        d.lane_consts_cached = 1
        K.check(K.cawn_phase_accumulate_valve_bwd(d, t["mag"], t["ang"], tv, t["gamma"], t["theta"], t["conv_w"], t["conv_b"],
                                                  None, ckpt, t["dz_re"], t["dz_im"], None, dmag, dang, dvalve, dg, dt,
                                                  dcw, dcb, None, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    for h in (0, H - 1):
        lanes = np.arange(h * F, (h + 1) * F)
        sub = _sub(inp, lanes)
        cfg = O.Cfg(B, L, 1, F, conv_k=Kc, gate_tau=wl.gate_tau, gate_mode=1 if valve else 0, ret_mode=1 if ret else 0)
        kw = dict(conv_w=sub["conv_w"], conv_b=sub["conv_b"], valve=np.ascontiguousarray(vlog[:, :, h:h + 1]) if valve else None,
                  ret=np.ascontiguousarray(rlog[:, :, h:h + 1]) if ret else None, ret_bias=rbias if ret else None)
        of = O.phase_fwd(cfg, sub["mag"], sub["ang"], None if ret else sub["gamma"], sub["theta"], want_gate=False, **kw)
        ob = O.phase_bwd(cfg, sub["mag"], sub["ang"], None if ret else sub["gamma"], sub["theta"], sub["dz_re"], sub["dz_im"], **kw)
        sl = slice(h * F, (h + 1) * F)
        errs = dict(z_re=G.rel_err(z_re[..., sl].cpu().numpy(), of["z_re"]), z_im=G.rel_err(z_im[..., sl].cpu().numpy(), of["z_im"]),
                    dmag=G.rel_err(dmag[..., sl].cpu().numpy(), ob["dmag"]), dang=G.rel_err(dang[..., sl].cpu().numpy(), ob["dang"]),
                    dtheta=G.rel_err(dt.cpu().numpy()[sl], ob["dtheta"]),
                    dconv_w=G.rel_err(dcw.cpu().numpy()[:, sl], ob["dconv_w"]),
                    dconv_b=G.rel_err(dcb.cpu().numpy()[:, sl], ob["dconv_b"]))
        if valve:
            errs["dvalve"] = G.rel_err(dvalve[..., h].cpu().numpy(), ob["dvalve"][..., 0])
        if ret:
            errs["dret"] = G.rel_err(dret[..., h].cpu().numpy(), ob["dret"][..., 0])
        else:
            errs["dgamma"] = G.rel_err(dg.cpu().numpy()[sl], ob["dgamma"])
        bad = {k: v for k, v in errs.items() if not v <= TOL}
        assert not bad, (h, bad, errs)


def test_one_call_over_two_million_tokens_forward_and_backward():
    """A single call of 2^21 tokens on one 32-lane block: one chain of 8192 forward and 16384 backward
    tiles (1/16 of the most a call may span), retention up to 0.99999 so that the far past still weighs.
    All 32 lanes against the oracle: outputs, carried state, input and parameter gradients."""
    import torch
    import gpu_util as G
    B, L, H, F, Kc = 1, 1 << 21, 1, 32, 4
    J = H * F
    r = np.random.Generator(np.random.PCG64(4250 + 96))
    d = dict(mag=r.standard_normal((B, L, J), dtype=np.float32), ang=r.standard_normal((B, L, J), dtype=np.float32),
             gamma=r.uniform(0.999, 0.99999, J).astype(np.float32), theta=O.theta_init(H, F),
             conv_w=(r.standard_normal((2, J, Kc)) / 2).astype(np.float32), conv_b=np.zeros((2, J), np.float32),
             dz_re=r.standard_normal((B, L, J), dtype=np.float32), dz_im=r.standard_normal((B, L, J), dtype=np.float32))
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, gate_tau=0.1)
    of = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], conv_w=d["conv_w"], conv_b=d["conv_b"], want_gate=False)
    ob = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], d["dz_re"], d["dz_im"], conv_w=d["conv_w"],
                     conv_b=d["conv_b"])
    fw = G.run_fwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1, want_mask=False)
    assert max(G.rel_err(fw["z_re"], of["z_re"]), G.rel_err(fw["z_im"], of["z_im"])) <= TOL
    assert G.rel_err(G.unpack_state(fw["state_out"], B, J, Kc)[0], of["scan_out"]) <= TOL
    # the last stretch on its own terms (the rms floor of the whole tensor must not hide a drift)
    assert G.rel_err(fw["z_re"][:, -4096:], of["z_re"][:, -4096:]) <= TOL
    out = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1)
    errs = {k: G.rel_err(out[k], ob[k]) for k in ("dmag", "dang", "dgamma", "dtheta", "dconv_w", "dconv_b")}
    errs["dmag_head"] = G.rel_err(out["dmag"][:, :4096], ob["dmag"][:, :4096])
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, (bad, errs)
    del fw, out
    torch.cuda.empty_cache()


def _paper_inputs(wl):
    """The valve and retention logits exactly as bench.py --paper draws them."""
    B, L, H, F = wl.B, wl.L, wl.H, wl.F
    rr = np.random.Generator(np.random.PCG64(4250 + 98))
    ret = (-2.0 + 1.5 * rr.standard_normal((B, L, H))).astype(np.float32)
    ret_bias = np.linspace(3.0, 0.0, F).astype(np.float32)
    rv = np.random.Generator(np.random.PCG64(4250 + 99))
    valve = (-3.9 + 3.0 * rv.standard_normal((B, L, H))).astype(np.float32)
    return valve, ret, ret_bias


def test_paper_layer_training_step_full_size():
    """The descriptor bench.py --paper times: B=8, L=8192, 4 heads of 64 harmonics (Sec. 4.3), conv kernel 3
    (Sec. 3.2), softplus amplitude, per-head valve with eps = 0.001 and data-dependent retention (Sec. 3.3).
    The valve and the retention couple the lanes of a head, so whole heads are sampled: the oracle runs heads
    0 and 3 (all batch rows, all tokens) as a two-head problem of its own."""
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS["cfg6_paper_heads"].with_(name="paper_layer", conv_k=3)
    B, L, H, F, J, Kc = wl.B, wl.L, wl.H, wl.F, wl.J, wl.conv_k
    assert (B, L, H, F, Kc) == (8, 8192, 4, 64, 3)
    theta = K.cawn_theta_init(H, F)
    inp = WL.make_inputs(wl, theta=theta, with_grads=True)
    valve, ret, ret_bias = _paper_inputs(wl)
    out = G.run_fwd_bwd(inp, B, L, H, F, conv_k=Kc, amp_mode=1, valve=valve, valve_eps=0.001, ret=ret, ret_bias=ret_bias,
                        want_dstate=False)
    fw = G.run_fwd(inp, B, L, H, F, conv_k=Kc, amp_mode=1, valve=valve, valve_eps=0.001, ret=ret, ret_bias=ret_bias)
    heads = [0, 3]
    lanes = np.concatenate([np.arange(h * F, (h + 1) * F) for h in heads])
    sub = _sub(inp, lanes)
    cfg = O.Cfg(B, L, len(heads), F, conv_k=Kc, amp_mode=1, gate_mode=1, valve_eps=0.001, ret_mode=1, nthreads=O.max_threads())
    kw = dict(conv_w=sub["conv_w"], conv_b=sub["conv_b"], valve=np.ascontiguousarray(valve[:, :, heads]),
              ret=np.ascontiguousarray(ret[:, :, heads]), ret_bias=ret_bias)
    of = O.phase_fwd(cfg, sub["mag"], sub["ang"], None, sub["theta"], **kw)
    ob = O.phase_bwd(cfg, sub["mag"], sub["ang"], None, sub["theta"], sub["dz_re"], sub["dz_im"], **kw)
    errs = {"z_re": G.rel_err(fw["z_re"][..., lanes], of["z_re"]), "z_im": G.rel_err(fw["z_im"][..., lanes], of["z_im"]),
            "dmag": G.rel_err(out["dmag"][..., lanes], ob["dmag"]), "dang": G.rel_err(out["dang"][..., lanes], ob["dang"]),
            "dtheta": G.rel_err(out["dtheta"][lanes], ob["dtheta"]),
            "dconv_w": G.rel_err(out["dconv_w"][:, lanes], ob["dconv_w"]),
            "dconv_b": G.rel_err(out["dconv_b"][:, lanes], ob["dconv_b"]),
            "dvalve": G.rel_err(out["dvalve"][:, :, heads], ob["dvalve"]),
            "dret": G.rel_err(out["dret"][:, :, heads], ob["dret"])}
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, (bad, errs)
    # the valve mask of the sampled heads, bit for bit, and about half the valves shut
    bits = np.unpackbits(fw["mask"].view(np.uint8), bitorder="little").reshape(B, L, -1)[..., :J]
    assert np.array_equal(bits[..., lanes], of["gate"])
    assert 0.4 < 1.0 - bits.mean() < 0.6


def test_training_step_through_the_harmonic_conv_full_size():
    """bench.py --hconv: the training-step shape (B=8, L=8192, 12 heads of 64) with the harmonic convolution fused
    behind the clamp, forward and backward; heads 0, 5 and 11 against the oracle's composed step."""
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS["cfg3_train"]
    B, L, H, F, J, Kc = wl.B, wl.L, wl.H, wl.F, wl.J, wl.conv_k
    theta = K.cawn_theta_init(H, F)
    inp = WL.make_inputs(wl, theta=theta, with_grads=True)
    rh = np.random.Generator(np.random.PCG64(4250 + 97))
    inp["hconv_w"] = (rh.standard_normal((2, H, 3)) / np.sqrt(3.0)).astype(np.float32)
    inp["hconv_b"] = (0.1 * rh.standard_normal((2, H))).astype(np.float32)
    inp["dc_re"], inp["dc_im"] = inp["dz_re"], inp["dz_im"]
    out = G.run_hconv_fwd_bwd(inp, B, L, H, F, conv_k=Kc, gate_tau=wl.gate_tau)
    heads = [0, 5, 11]
    lanes = np.concatenate([np.arange(h * F, (h + 1) * F) for h in heads])
    sub = _sub(inp, lanes)
    n = len(heads)
    hw, hb = np.ascontiguousarray(inp["hconv_w"][:, heads]), np.ascontiguousarray(inp["hconv_b"][:, heads])
    kw = dict(conv_k=Kc, gate_tau=wl.gate_tau, nthreads=O.max_threads())
    f = O.phase_fwd(O.Cfg(B, L, n, F, **kw), sub["mag"], sub["ang"], sub["gamma"], sub["theta"], conv_w=sub["conv_w"],
                    conv_b=sub["conv_b"], want_gate=False)
    c = O.harmonic_conv(f["z_re"], f["z_im"], n, F, hw, hb)
    gh = O.harmonic_conv_bwd(f["z_re"], f["z_im"], n, F, hw, sub["dz_re"], sub["dz_im"])
    g = O.phase_bwd(O.Cfg(B, L, n, F, dz_f64=1, **kw), sub["mag"], sub["ang"], sub["gamma"], sub["theta"], gh["dz_re"],
                    gh["dz_im"], conv_w=sub["conv_w"], conv_b=sub["conv_b"])
    errs = {"c_re": G.rel_err(out["c_re"][..., lanes], c[0]), "c_im": G.rel_err(out["c_im"][..., lanes], c[1]),
            "dmag": G.rel_err(out["dmag"][..., lanes], g["dmag"]), "dang": G.rel_err(out["dang"][..., lanes], g["dang"]),
            "dgamma": G.rel_err(out["dgamma"][lanes], g["dgamma"]), "dtheta": G.rel_err(out["dtheta"][lanes], g["dtheta"]),
            "dconv_w": G.rel_err(out["dconv_w"][:, lanes], g["dconv_w"]),
            "dconv_b": G.rel_err(out["dconv_b"][:, lanes], g["dconv_b"]),
            "dhconv_w": G.rel_err(out["dhconv_w"][:, heads], gh["dw"]),
            "dhconv_b": G.rel_err(out["dhconv_b"][:, heads], gh["dbias"])}
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, (bad, errs)


def test_paper_layer_through_the_harmonic_conv_full_size():
    """bench.py --paper --hconv: the layer as the paper states it (B=8, L=8192, 4 heads of 64 harmonics, conv kernel 3,
    softplus amplitude, per-head valve, data-dependent retention: Sec. 3.2-3.4, Sec. 4.3) ending in the depth-wise
    harmonic convolution of Sec. 3.6, forward and backward; heads 0 and 3 against the oracle's composed step."""
    import gpu_util as G
    from paper_2604_04250_amd import binding as K
    wl = WL.CONFIGS["cfg6_paper_heads"].with_(name="paper_layer", conv_k=3)
    B, L, H, F, J, Kc = wl.B, wl.L, wl.H, wl.F, wl.J, wl.conv_k
    theta = K.cawn_theta_init(H, F)
    inp = WL.make_inputs(wl, theta=theta, with_grads=True)
    valve, ret, ret_bias = _paper_inputs(wl)
    rh = np.random.Generator(np.random.PCG64(4250 + 98))
    inp["hconv_w"] = (rh.standard_normal((2, H, 3)) / np.sqrt(3.0)).astype(np.float32)
    inp["hconv_b"] = (0.1 * rh.standard_normal((2, H))).astype(np.float32)
    inp["dc_re"], inp["dc_im"] = inp["dz_re"], inp["dz_im"]
    out = G.run_hconv_fwd_bwd(inp, B, L, H, F, conv_k=Kc, amp_mode=1, valve=valve, valve_eps=0.001, ret=ret,
                              ret_bias=ret_bias)
    heads = [0, 3]
    lanes = np.concatenate([np.arange(h * F, (h + 1) * F) for h in heads])
    sub = _sub(inp, lanes)
    n = len(heads)
    hw, hb = np.ascontiguousarray(inp["hconv_w"][:, heads]), np.ascontiguousarray(inp["hconv_b"][:, heads])
    kw = dict(conv_k=Kc, amp_mode=1, gate_mode=1, valve_eps=0.001, ret_mode=1, nthreads=O.max_threads())
    streams = dict(conv_w=sub["conv_w"], conv_b=sub["conv_b"], valve=np.ascontiguousarray(valve[:, :, heads]),
                   ret=np.ascontiguousarray(ret[:, :, heads]), ret_bias=ret_bias)
    f = O.phase_fwd(O.Cfg(B, L, n, F, **kw), sub["mag"], sub["ang"], None, sub["theta"], want_gate=False, **streams)
    c = O.harmonic_conv(f["z_re"], f["z_im"], n, F, hw, hb)
    gh = O.harmonic_conv_bwd(f["z_re"], f["z_im"], n, F, hw, sub["dz_re"], sub["dz_im"])
    g = O.phase_bwd(O.Cfg(B, L, n, F, dz_f64=1, **kw), sub["mag"], sub["ang"], None, sub["theta"], gh["dz_re"], gh["dz_im"],
                    **streams)
    errs = {"c_re": G.rel_err(out["c_re"][..., lanes], c[0]), "c_im": G.rel_err(out["c_im"][..., lanes], c[1]),
            "dmag": G.rel_err(out["dmag"][..., lanes], g["dmag"]), "dang": G.rel_err(out["dang"][..., lanes], g["dang"]),
            "dtheta": G.rel_err(out["dtheta"][lanes], g["dtheta"]),
            "dconv_w": G.rel_err(out["dconv_w"][:, lanes], g["dconv_w"]),
            "dconv_b": G.rel_err(out["dconv_b"][:, lanes], g["dconv_b"]),
            "dvalve": G.rel_err(out["dvalve"][:, :, heads], g["dvalve"]),
            "dret": G.rel_err(out["dret"][:, :, heads], g["dret"]),
            "dhconv_w": G.rel_err(out["dhconv_w"][:, heads], gh["dw"]),
            "dhconv_b": G.rel_err(out["dhconv_b"][:, heads], gh["dbias"])}
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, (bad, errs)
