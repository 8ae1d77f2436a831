"""GPU parity of the forward with the depth-wise harmonic convolution fused behind the output clamp
(Sec. 3.6: channel = (plane, head), three taps along the harmonics of the head, zero padding) against
the fp64 oracle (its forward followed by its harmonic convolution), through the C ABI.  Bar as for the
other parity tests: rms-floored relative error <= 1e-4, gate masks bit-exact; with bfloat16
activations the rounding allowance of the bf16 tests on the stored outputs."""
import numpy as np
import pytest

from oracle import cawn_oracle as O

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _gpu():
    import gpu_util
    return gpu_util


def _inputs(B, L, H, F, Kc, seed):
    r = np.random.Generator(np.random.PCG64(seed))
    J = H * F
    d = dict(mag=r.standard_normal((B, L, J), dtype=np.float32),
             ang=r.standard_normal((B, L, J), dtype=np.float32),
             gamma=r.uniform(0.9, 0.9999, J).astype(np.float32),
             theta=r.uniform(0, np.pi, J).astype(np.float32),
             ret=(-2.0 + 1.5 * r.standard_normal((B, L, H))).astype(np.float32),
             ret_bias=np.linspace(3.0, 0.0, F).astype(np.float32),
             valve=(-3.9 + 3.0 * r.standard_normal((B, L, H))).astype(np.float32),
             # taps of every size and sign, different in every channel; a bias on every channel
             hconv_w=r.standard_normal((2, H, 3)).astype(np.float32),
             hconv_b=r.standard_normal((2, H)).astype(np.float32))
    kk = max(Kc, 1)
    d["conv_w"] = (r.standard_normal((2, J, kk)) / np.sqrt(kk)).astype(np.float32)
    d["conv_b"] = (0.1 * r.standard_normal((2, J))).astype(np.float32)
    return d


def _oracle(B, L, H, F, Kc, d, amp_mode=0, valve=False, ret=False, tau=0.0, state=None, out_clamp=100.0):
    scan_in = tail_in = None
    if state is not None:
        scan_in, tail_in = state
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_mode=1 if valve else 0, gate_tau=tau,
                ret_mode=1 if ret else 0, out_clamp=out_clamp)
    ora = O.phase_fwd(cfg, d["mag"][:, :L], d["ang"][:, :L], None if ret else d["gamma"], d["theta"],
                      conv_w=d["conv_w"], conv_b=d["conv_b"], valve=d["valve"][:, :L] if valve else None,
                      ret=d["ret"][:, :L] if ret else None, ret_bias=d["ret_bias"] if ret else None,
                      scan_in=None if scan_in is None else scan_in.astype(np.float64),
                      tail_in=tail_in if Kc > 1 else None)
    ora["c_re"], ora["c_im"] = O.harmonic_conv(ora["z_re"], ora["z_im"], H, F, d["hconv_w"], d["hconv_b"])
    return ora


def _check(B, L, H, F, Kc, d, amp_mode=0, valve=False, ret=False, tau=0.0, state=None, bf16=False,
           out_clamp=100.0, **kw):
    G = _gpu()
    J = H * F
    blob = None
    if state is not None:
        blob = G.pack_state(state[0], state[1] if Kc > 1 else None)
    if bf16:
        d = dict(d, mag=G.bf16_exact(d["mag"]), ang=G.bf16_exact(d["ang"]))
    ora = _oracle(B, L, H, F, Kc, d, amp_mode, valve, ret, tau, state, out_clamp)
    out = G.run_fwd(d, B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=tau, state_in=blob, out_clamp=out_clamp,
                    valve=d["valve"] if valve else None, ret=d["ret"] if ret else None,
                    ret_bias=d["ret_bias"] if ret else None, hconv_w=d["hconv_w"], hconv_b=d["hconv_b"],
                    bf16=bf16, **kw)
    if bf16:
        e = max(G.bf16_err(out["z_re"], ora["c_re"]), G.bf16_err(out["z_im"], ora["c_im"]))
        assert e <= 1.0, e
    else:
        e = max(G.rel_err(out["z_re"], ora["c_re"]), G.rel_err(out["z_im"], ora["c_im"]))
        assert e <= TOL, e
    assert np.array_equal(out["mask"], G.mask_from_gate(ora["gate"])), "gate mask differs"
    scan, tail = G.unpack_state(out["state_out"], B, J, Kc)
    assert G.rel_err(scan, ora["scan_out"]) <= TOL          # the state is that of the unconvolved recurrence
    return out, ora


# heads inside a 32-lane block (8, 16, 32), of two, four and eight blocks (64, 128, 256); odd head counts
@pytest.mark.parametrize("H,F", [(4, 64), (3, 64), (2, 32), (5, 32), (4, 16), (3, 16), (8, 8), (3, 8), (1, 128),
                                 (3, 128), (1, 256), (12, 4)])
@pytest.mark.parametrize("Kc", [0, 3, 4])
def test_hconv_forward_head_widths(H, F, Kc):
    B, L = 2, 700                      # three forward tiles, ragged tail
    d = _inputs(B, L, H, F, Kc, 5100 + H * 131 + F + Kc)
    _check(B, L, H, F, Kc, d, tau=0.25)


@pytest.mark.parametrize("L", [17, 31, 255, 256, 257, 513])
def test_hconv_forward_lengths(L):
    B, H, F, Kc = 3, 2, 64, 3
    d = _inputs(B, L, H, F, Kc, 5200 + L)
    _check(B, L, H, F, Kc, d, tau=0.1)


@pytest.mark.parametrize("valve,ret", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("H,F", [(4, 64), (2, 32), (1, 128)])
def test_hconv_forward_valve_and_retention(valve, ret, H, F):
    B, L, Kc = 2, 600, 3
    d = _inputs(B, L, H, F, Kc, 5300 + H + F + 2 * valve + ret)
    _check(B, L, H, F, Kc, d, amp_mode=1, valve=valve, ret=ret)


@pytest.mark.parametrize("H,F", [(4, 64), (2, 32), (4, 16), (1, 128)])
@pytest.mark.parametrize("Kc", [0, 3])
def test_hconv_forward_bf16(H, F, Kc):
    B, L = 2, 700
    d = _inputs(B, L, H, F, Kc, 5400 + H + F + Kc)
    _check(B, L, H, F, Kc, d, tau=0.25, bf16=True)


def test_hconv_forward_bf16_paper_layer():
    B, L, H, F, Kc = 2, 600, 4, 64, 3
    d = _inputs(B, L, H, F, Kc, 5450)
    _check(B, L, H, F, Kc, d, amp_mode=1, valve=True, ret=True, bf16=True)


@pytest.mark.parametrize("bf16", [False, True])
def test_hconv_forward_concat_layout(bf16):
    """Both convolved planes share rows of 2 J elements (Sec. 3.5): the deferred last lane of a block
    is stored one element before the next block's first lane in either plane."""
    B, L, H, F, Kc = 2, 520, 3, 64, 3
    d = _inputs(B, L, H, F, Kc, 5500 + bf16)
    _check(B, L, H, F, Kc, d, tau=0.25, bf16=bf16, concat=True)


def test_hconv_forward_tight_clamp():
    """The convolution reads the clamped state: with a clamp that binds often, convolving the
    unclamped state would differ."""
    B, L, H, F, Kc = 2, 600, 2, 64, 3
    d = _inputs(B, L, H, F, Kc, 5600)
    out, ora = _check(B, L, H, F, Kc, d, out_clamp=2.0)
    assert np.mean(np.abs(ora["z_re"]) >= 2.0) > 0.05


@pytest.mark.parametrize("H,F", [(4, 64), (4, 16)])
def test_hconv_forward_chunked_state(H, F):
    """Two calls joined by state_out -> state_in give the convolved output of one call."""
    G = _gpu()
    B, L, Kc = 2, 900, 3
    J = H * F
    d = _inputs(B, L, H, F, Kc, 5700 + F)
    ora = _oracle(B, L, H, F, Kc, d, tau=0.25)
    n1 = 389
    o1 = G.run_fwd(d, B, n1, H, F, conv_k=Kc, gate_tau=0.25, hconv_w=d["hconv_w"], hconv_b=d["hconv_b"])
    d2 = dict(d, mag=d["mag"][:, n1:], ang=d["ang"][:, n1:])
    o2 = G.run_fwd(d2, B, L - n1, H, F, conv_k=Kc, gate_tau=0.25, state_in=o1["state_out"],
                   hconv_w=d["hconv_w"], hconv_b=d["hconv_b"])
    c_re = np.concatenate([o1["z_re"], o2["z_re"]], 1)
    c_im = np.concatenate([o1["z_im"], o2["z_im"]], 1)
    assert max(G.rel_err(c_re, ora["c_re"]), G.rel_err(c_im, ora["c_im"])) <= TOL
    scan, _ = G.unpack_state(o2["state_out"], B, J, Kc)
    assert G.rel_err(scan, ora["scan_out"]) <= TOL


@pytest.mark.parametrize("H,F", [(4, 64), (8, 8), (1, 256), (3, 128)])
@pytest.mark.parametrize("L", [1, 5, 16])
def test_hconv_decode_steps(H, F, L):
    """Short calls (the sequential per-lane kernel): token by token with the state carried."""
    B, Kc = 3, 3
    d = _inputs(B, L, H, F, Kc, 5800 + F + L)
    _check(B, L, H, F, Kc, d, tau=0.1)
    _check(B, L, H, F, Kc, d, tau=0.1, bf16=True)


def test_hconv_cached_lane_constants():
    """A second call with lane_consts_cached = 1 reuses the taps staged by the first."""
    G = _gpu()
    B, L, H, F, Kc = 2, 300, 2, 64, 3
    d = _inputs(B, L, H, F, Kc, 5900)
    ora = _oracle(B, L, H, F, Kc, d, tau=0.25)
    import torch
    from paper_2604_04250_amd import binding as K
    dsc = K.make_desc(B, L, H, F, conv_k=Kc, gate_tau=0.25, hconv_k=3)
    ws = torch.empty((K.cawn_workspace_bytes(dsc) + 3) // 4, dtype=torch.int32, device="cuda")
    K.check(K.cawn_workspace_init(ws))
    G.run_fwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.25, hconv_w=d["hconv_w"], hconv_b=d["hconv_b"], ws=ws)
    other = dict(d, hconv_w=np.zeros_like(d["hconv_w"]), hconv_b=np.zeros_like(d["hconv_b"]))
    out = G.run_fwd(other, B, L, H, F, conv_k=Kc, gate_tau=0.25, hconv_w=other["hconv_w"],
                    hconv_b=other["hconv_b"], ws=ws, cached=1)
    assert max(G.rel_err(out["z_re"], ora["c_re"]), G.rel_err(out["z_im"], ora["c_im"])) <= TOL


def test_hconv_unsupported_shapes_are_refused():
    import torch
    from paper_2604_04250_amd import binding as K
    G = _gpu()
    for H, F, gate_mode, want in [(2, 96, 0, K.CAWN_EUNSUPPORTED), (2, 24, 0, K.CAWN_EUNSUPPORTED),
                                  (4, 16, 1, K.CAWN_EUNSUPPORTED)]:
        B, L = 1, 64
        J = H * F
        dsc = K.make_desc(B, L, H, F, hconv_k=3, gate_mode=gate_mode)
        x = torch.zeros((B, L, J), device="cuda")
        p = torch.ones((J,), device="cuda")
        w = torch.zeros((2, H, 3), device="cuda")
        v = torch.zeros((B, L, H), device="cuda")
        ws = G.Workspaces.get(dsc)
        st = K.cawn_phase_accumulate_hconv_fwd(dsc, x, x, v, None, None, p, p, None, None, w, None, None,
                                               torch.empty_like(x), torch.empty_like(x), None, None, None, ws)
        assert st == want, (H, F, st)


@pytest.mark.parametrize("name,bf16", [("cfg2_layer_fwd", False), ("cfg2_layer_fwd", True), ("cfg6_paper_heads", False)])
def test_hconv_full_size_sampled_heads(name, bf16):
    """A benchmark configuration at full size, launched as bench.py --hconv launches it; whole heads are
    sampled (the convolution needs every harmonic of a head) and compared with the oracle on those heads."""
    import torch
    from paper_2604_04250_amd import binding as K
    from paper_2604_04250_amd import workloads as WL
    G = _gpu()
    wl = WL.CONFIGS[name]
    B, L, H, F, J, Kc = wl.B, wl.L, wl.H, wl.F, wl.J, wl.conv_k
    inp = WL.make_inputs(wl, theta=K.cawn_theta_init(H, F), with_grads=False)
    if bf16:
        inp = dict(inp, mag=G.bf16_exact(inp["mag"]), ang=G.bf16_exact(inp["ang"]))
    r = np.random.Generator(np.random.PCG64(6100))
    hw = (r.standard_normal((2, H, 3)) / np.sqrt(3.0)).astype(np.float32)
    hb = (0.1 * r.standard_normal((2, H))).astype(np.float32)
    heads = sorted({0, H - 1, int(r.integers(0, H))})
    lanes = np.concatenate([np.arange(h * F, (h + 1) * F) for h in heads])
    n = len(heads)
    cfg = O.Cfg(B, L, n, F, conv_k=Kc, gate_tau=wl.gate_tau)
    of = O.phase_fwd(cfg, np.ascontiguousarray(inp["mag"][..., lanes]), np.ascontiguousarray(inp["ang"][..., lanes]),
                     inp["gamma"][lanes], inp["theta"][lanes], conv_w=np.ascontiguousarray(inp["conv_w"][:, lanes]),
                     conv_b=np.ascontiguousarray(inp["conv_b"][:, lanes]))
    c_re, c_im = O.harmonic_conv(of["z_re"], of["z_im"], n, F, hw[:, heads], hb[:, heads])
    d = K.make_desc(B, L, H, F, conv_k=Kc, gate_tau=wl.gate_tau, hconv_k=3)
    dev = G.DEV
    adt = torch.bfloat16 if bf16 else torch.float32
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in inp}
    mag, ang = t["mag"].to(adt), t["ang"].to(adt)
    z_re, z_im = torch.empty((B, L, J), device=dev, dtype=adt), torch.empty((B, L, J), device=dev, dtype=adt)
    ws = K.alloc_workspace(d, dev)
    K.check(K.cawn_phase_accumulate_hconv_fwd(d, mag, ang, None, None, None, t["gamma"], t["theta"], t["conv_w"],
                                              t["conv_b"], torch.from_numpy(hw).to(dev), torch.from_numpy(hb).to(dev),
                                              None, z_re, z_im, None, None, None, ws,
                                              activations_bf16=1 if bf16 else 0))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    li = torch.from_numpy(lanes).to(dev)
    g_re, g_im = z_re[..., li].float().cpu().numpy(), z_im[..., li].float().cpu().numpy()
    if bf16:
        assert max(G.bf16_err(g_re, c_re), G.bf16_err(g_im, c_im)) <= 1.0
    else:
        assert max(G.rel_err(g_re, c_re), G.rel_err(g_im, c_im)) <= TOL
