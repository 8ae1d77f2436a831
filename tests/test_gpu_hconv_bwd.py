"""GPU parity of the backward through the fused harmonic convolution (Sec. 3.6) against the fp64 oracle, through
the C ABI.  The oracle's step is its forward, its harmonic convolution, the convolution's adjoint
(harmonic_conv_bwd) and its backward on the fp64 gradient that adjoint returns; the GPU does all of it in one
kernel from the gradients of the convolved output.  Bar as for the other parity tests: rms-floored relative error
<= 1e-4 on every returned tensor."""
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
    d = dict(mag=r.standard_normal((B, L, J), dtype=np.float32), ang=r.standard_normal((B, L, J), dtype=np.float32),
             gamma=r.uniform(0.9, 0.9999, J).astype(np.float32), theta=r.uniform(0, np.pi, J).astype(np.float32),
             hconv_w=r.standard_normal((2, H, 3)).astype(np.float32), hconv_b=r.standard_normal((2, H)).astype(np.float32),
             dc_re=r.standard_normal((B, L, J), dtype=np.float32), dc_im=r.standard_normal((B, L, J), dtype=np.float32))
    kk = max(Kc, 1)
    d["conv_w"] = (r.standard_normal((2, J, kk)) / np.sqrt(kk)).astype(np.float32)
    d["conv_b"] = (0.1 * r.standard_normal((2, J))).astype(np.float32)
    return d


def _oracle(B, L, H, F, Kc, d, amp_mode=0, tau=0.0, out_clamp=100.0, grad_clamp=100.0, scan_in=None, tail_in=None,
            dscan_out=None, dtail_out=None):
    kw = dict(conv_k=Kc, amp_mode=amp_mode, gate_tau=tau, out_clamp=out_clamp, grad_clamp=grad_clamp)
    st = dict(scan_in=scan_in, tail_in=tail_in if Kc > 1 else None)
    f = O.phase_fwd(O.Cfg(B, L, H, F, **kw), d["mag"][:, :L], d["ang"][:, :L], d["gamma"], d["theta"], conv_w=d["conv_w"],
                    conv_b=d["conv_b"], **st)
    c = O.harmonic_conv(f["z_re"], f["z_im"], H, F, d["hconv_w"], d["hconv_b"])
    gh = O.harmonic_conv_bwd(f["z_re"], f["z_im"], H, F, d["hconv_w"], d["dc_re"][:, :L], d["dc_im"][:, :L])
    g = O.phase_bwd(O.Cfg(B, L, H, F, dz_f64=1, **kw), d["mag"][:, :L], d["ang"][:, :L], d["gamma"], d["theta"],
                    gh["dz_re"], gh["dz_im"], conv_w=d["conv_w"], conv_b=d["conv_b"], dscan_out=dscan_out,
                    dtail_out=dtail_out if Kc > 1 else None, **st)
    g.update(c_re=c[0], c_im=c[1], dhconv_w=gh["dw"], dhconv_b=gh["dbias"])
    return g


def _compare(out, ora, Kc, names=None):
    G = _gpu()
    names = names or ["c_re", "c_im", "dmag", "dang", "dgamma", "dtheta", "dhconv_w", "dhconv_b"] + \
        (["dconv_w", "dconv_b"] if Kc > 0 else [])
    errs = {k: G.rel_err(out[k], ora[k]) for k in names}
    assert max(errs.values()) <= TOL, errs
    return errs


# heads inside a 32-lane block (4, 8, 16, 32), of two, four and eight blocks (64, 128, 256); odd head counts
@pytest.mark.parametrize("H,F", [(4, 64), (3, 64), (2, 32), (5, 32), (4, 16), (8, 8), (1, 128), (3, 128), (1, 256), (12, 4)])
@pytest.mark.parametrize("Kc", [0, 3, 4])
def test_hconv_backward_head_widths(H, F, Kc):
    B, L = 2, 300                      # three backward tiles, ragged tail
    d = _inputs(B, L, H, F, Kc, 6100 + H * 131 + F + Kc)
    out = _gpu().run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.25)
    _compare(out, _oracle(B, L, H, F, Kc, d, tau=0.25), Kc)


@pytest.mark.parametrize("L", [1, 7, 127, 128, 129, 257, 640])
def test_hconv_backward_lengths(L):
    B, H, F, Kc = 3, 2, 64, 3
    d = _inputs(B, L, H, F, Kc, 6200 + L)
    out = _gpu().run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1)
    _compare(out, _oracle(B, L, H, F, Kc, d, tau=0.1), Kc)


@pytest.mark.parametrize("Kc", [1, 2])
def test_hconv_backward_other_kernel_sizes_and_softplus_amplitude(Kc):
    B, L, H, F = 2, 200, 2, 64
    d = _inputs(B, L, H, F, Kc, 6300 + Kc)
    out = _gpu().run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, amp_mode=1, gate_tau=0.8)
    _compare(out, _oracle(B, L, H, F, Kc, d, amp_mode=1, tau=0.8), Kc)


def test_hconv_backward_tap_gradients_use_the_clamped_state():
    """With an output clamp that bites (|S| reaches a few units here), the tap gradients pair the upstream
    gradients with the CLAMPED state while the recurrence's own gradients pass the clamp."""
    B, L, H, F, Kc = 2, 260, 2, 64, 3
    d = _inputs(B, L, H, F, Kc, 6400)
    out = _gpu().run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, out_clamp=0.75, grad_clamp=2.0)
    ora = _oracle(B, L, H, F, Kc, d, out_clamp=0.75, grad_clamp=2.0)
    _compare(out, ora, Kc)
    free = _oracle(B, L, H, F, Kc, d, out_clamp=100.0, grad_clamp=2.0)
    assert _gpu().rel_err(free["dhconv_w"], ora["dhconv_w"]) > 0.05        # the clamp does bite in this case


def test_hconv_backward_state_gradients_and_chunks():
    """Carried state in, gradient of the carried state out: the state is that of the unconvolved recurrence."""
    G = _gpu()
    B, L, H, F, Kc = 2, 333, 2, 64, 4
    J = H * F
    d = _inputs(B, L, H, F, Kc, 6500)
    r = np.random.Generator(np.random.PCG64(6501))
    scan_in = r.standard_normal((B, 2, J)).astype(np.float32)
    tail_in = r.standard_normal((B, Kc - 1, 2, J)).astype(np.float32)
    dscan = r.standard_normal((B, 2, J)).astype(np.float32)
    dtail = r.standard_normal((B, Kc - 1, 2, J)).astype(np.float32)
    out = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1, state_in=G.pack_state(scan_in, tail_in),
                              dstate_out=G.pack_state(dscan, dtail))
    ora = _oracle(B, L, H, F, Kc, d, tau=0.1, scan_in=scan_in.astype(np.float64), tail_in=tail_in,
                  dscan_out=dscan.astype(np.float64), dtail_out=dtail.astype(np.float64))
    _compare(out, ora, Kc)
    dscan_in, dtail_in = G.unpack_state(out["dstate_in"], B, J, Kc)
    assert G.rel_err(dscan_in, ora["dscan_in"]) <= TOL
    assert G.rel_err(dtail_in, ora["dtail_in"]) <= TOL


def test_hconv_backward_concat_layout_and_accumulation():
    G = _gpu()
    B, L, H, F, Kc = 2, 200, 1, 256, 3
    d = _inputs(B, L, H, F, Kc, 6600)
    ora = _oracle(B, L, H, F, Kc, d, tau=0.2)
    out = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.2, concat=True)
    _compare(out, ora, Kc)
    acc = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.2, accumulate=1, preset=2.0)
    for k in ("dgamma", "dtheta", "dconv_w", "dconv_b", "dhconv_w", "dhconv_b"):
        assert G.rel_err(acc[k] - 2.0, ora[k]) <= 2 * TOL, k


@pytest.mark.parametrize("H,F", [(4, 64), (2, 32), (4, 16), (1, 128), (1, 256)])
@pytest.mark.parametrize("Kc", [0, 3, 4])
def test_hconv_backward_bf16(H, F, Kc):
    """bfloat16 activations: inputs and the gradients of the convolved output are bf16-exact, what the kernels store
    as bf16 (convolved output, input gradients) may differ from the oracle by 1e-4 and is then rounded; every other
    gradient stays fp32 and keeps the plain bar."""
    G = _gpu()
    B, L = 2, 300
    d = _inputs(B, L, H, F, Kc, 6700 + H * 131 + F + Kc)
    for k in ("mag", "ang", "dc_re", "dc_im"):
        d[k] = G.bf16_exact(d[k])
    out = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.25, bf16=True)
    ora = _oracle(B, L, H, F, Kc, d, tau=0.25)
    for k in ("c_re", "c_im", "dmag", "dang"):
        assert G.bf16_err(out[k], ora[k]) <= 1.0, k
    _compare(out, ora, Kc, names=["dgamma", "dtheta", "dhconv_w", "dhconv_b"] + (["dconv_w", "dconv_b"] if Kc > 0 else []))


def test_hconv_backward_bf16_ragged_and_concat():
    G = _gpu()
    B, L, H, F, Kc = 3, 257, 2, 64, 3
    d = _inputs(B, L, H, F, Kc, 6800)
    for k in ("mag", "ang", "dc_re", "dc_im"):
        d[k] = G.bf16_exact(d[k])
    ora = _oracle(B, L, H, F, Kc, d, tau=0.1)
    for concat in (False, True):
        out = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, gate_tau=0.1, bf16=True, concat=concat)
        for k in ("c_re", "c_im", "dmag", "dang"):
            assert G.bf16_err(out[k], ora[k]) <= 1.0, (k, concat)
        _compare(out, ora, Kc, names=["dgamma", "dtheta", "dhconv_w", "dhconv_b", "dconv_w", "dconv_b"])


def test_hconv_backward_refusals():
    import torch
    from paper_2604_04250_amd import binding as K
    B, L, H, F = 1, 64, 2, 64
    J = H * F
    z = lambda *s: torch.zeros(s, device="cuda")
    d = K.make_desc(B, L, H, F, conv_k=0, hconv_k=3)
    ws = K.alloc_workspace(d)
    ck = z(K.cawn_ckpt_bytes(d) // 4)
    args = lambda dd, hw, ckpt, valve=None: K.cawn_phase_accumulate_hconv_bwd(
        dd, z(B, L, J), z(B, L, J), valve, None, None, z(J), z(J), None, None, hw, None, None, ckpt, z(B, L, J), z(B, L, J),
        None, z(B, L, J), z(B, L, J), None, None, None, None, None, None, z(2, H, 3), z(2, H), None, ws)
    assert args(d, z(2, H, 3), ck) == K.CAWN_OK
    assert args(d, None, ck) == K.CAWN_EINVAL                                        # no taps
    assert args(d, z(2, H, 3), None) == K.CAWN_EINVAL                                # the state rebuild needs checkpoints
    assert args(K.make_desc(B, L, H, F, hconv_k=0), z(2, H, 3), ck) == K.CAWN_EINVAL
    # the valve and the retention behind the harmonic convolution: heads of at least 32 harmonics, as in the forward
    assert args(K.make_desc(B, L, 8, 16, hconv_k=3, gate_mode=1), z(2, 8, 3), ck, z(B, L, 8)) == K.CAWN_EUNSUPPORTED
    assert args(K.make_desc(B, L, 8, 16, hconv_k=3, ret_mode=1), z(2, 8, 3), ck) == K.CAWN_EUNSUPPORTED
    assert args(K.make_desc(B, L, H, F, hconv_k=3, gate_mode=1), z(2, H, 3), ck) == K.CAWN_EINVAL      # no valve logits
    assert args(K.make_desc(B, L, H, F, hconv_k=3, ret_mode=1), z(2, H, 3), ck) == K.CAWN_EINVAL       # no retention logits
    assert args(K.make_desc(B, L, 3, 48, hconv_k=3), z(2, 3, 3), ck) in (K.CAWN_EUNSUPPORTED, K.CAWN_EWORKSPACE)
    # the plain backward does not take gradients of a convolved output
    st = K.cawn_phase_accumulate_bwd(d, z(B, L, J), z(B, L, J), z(J), z(J), None, None, None, ck, z(B, L, J), z(B, L, J), None,
                                     z(B, L, J), z(B, L, J), None, None, None, None, None, ws)
    assert st == K.CAWN_EINVAL
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))


# ---- the harmonic convolution behind the per-head valve and the data-dependent retention (Sec. 3.3, Sec. 3.6: the
#      layer as the paper states it, trained end to end)

def _inputs_modes(B, L, H, F, Kc, seed):
    d = _inputs(B, L, H, F, Kc, seed)
    r = np.random.Generator(np.random.PCG64(seed + 77))
    d["valve"] = (-3.9 + 3.0 * r.standard_normal((B, L, H))).astype(np.float32)
    d["ret"] = (-2.0 + 1.5 * r.standard_normal((B, L, H))).astype(np.float32)
    d["ret_bias"] = np.linspace(3.0, 0.0, F).astype(np.float32)
    return d


def _oracle_modes(B, L, H, F, Kc, d, valve, ret, amp_mode=0, tau=0.0, scan_in=None, tail_in=None, dscan_out=None,
                  dtail_out=None):
    kw = dict(conv_k=Kc, amp_mode=amp_mode, gate_tau=tau, gate_mode=1 if valve else 0, ret_mode=1 if ret else 0)
    st = dict(scan_in=scan_in, tail_in=tail_in if Kc > 1 else None)
    streams = dict(conv_w=d["conv_w"], conv_b=d["conv_b"], valve=d["valve"][:, :L] if valve else None,
                   ret=d["ret"][:, :L] if ret else None, ret_bias=d["ret_bias"] if ret else None)
    gamma = None if ret else d["gamma"]
    f = O.phase_fwd(O.Cfg(B, L, H, F, **kw), d["mag"][:, :L], d["ang"][:, :L], gamma, d["theta"], **streams, **st)
    c = O.harmonic_conv(f["z_re"], f["z_im"], H, F, d["hconv_w"], d["hconv_b"])
    gh = O.harmonic_conv_bwd(f["z_re"], f["z_im"], H, F, d["hconv_w"], d["dc_re"][:, :L], d["dc_im"][:, :L])
    g = O.phase_bwd(O.Cfg(B, L, H, F, dz_f64=1, **kw), d["mag"][:, :L], d["ang"][:, :L], gamma, d["theta"],
                    gh["dz_re"], gh["dz_im"], dscan_out=dscan_out, dtail_out=dtail_out if Kc > 1 else None, **streams, **st)
    g.update(c_re=c[0], c_im=c[1], dhconv_w=gh["dw"], dhconv_b=gh["dbias"])
    return g


def _names_modes(Kc, valve, ret):
    return ["c_re", "c_im", "dmag", "dang", "dtheta", "dhconv_w", "dhconv_b"] + (["dconv_w", "dconv_b"] if Kc > 0 else []) + \
        (["dvalve"] if valve else []) + (["dret"] if ret else ["dgamma"])


@pytest.mark.parametrize("valve,ret", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("H,F", [(4, 64), (3, 32), (1, 128), (1, 256)])
@pytest.mark.parametrize("Kc", [0, 3, 4])
def test_hconv_backward_with_valve_and_retention(valve, ret, H, F, Kc):
    B, L = 2, 300
    d = _inputs_modes(B, L, H, F, Kc, 6900 + H * 131 + F + Kc)
    out = _gpu().run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, amp_mode=1, valve=d["valve"] if valve else None,
                                   ret=d["ret"] if ret else None, ret_bias=d["ret_bias"] if ret else None)
    _compare(out, _oracle_modes(B, L, H, F, Kc, d, valve, ret, amp_mode=1), Kc, names=_names_modes(Kc, valve, ret))


@pytest.mark.parametrize("L", [1, 127, 129, 640])
def test_hconv_backward_paper_layer_lengths_and_state(L):
    """The paper's layer (4 heads of 64 harmonics, conv kernel 3, softplus amplitude, valve, retention) behind the
    harmonic convolution, with a carried state in and the gradient of the carried state out."""
    G = _gpu()
    B, H, F, Kc = 2, 4, 64, 3
    J = H * F
    d = _inputs_modes(B, L, H, F, Kc, 7000 + L)
    r = np.random.Generator(np.random.PCG64(7001 + L))
    scan_in = r.standard_normal((B, 2, J)).astype(np.float32)
    tail_in = r.standard_normal((B, Kc - 1, 2, J)).astype(np.float32)
    dscan = r.standard_normal((B, 2, J)).astype(np.float32)
    dtail = r.standard_normal((B, Kc - 1, 2, J)).astype(np.float32)
    out = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, amp_mode=1, valve=d["valve"], ret=d["ret"], ret_bias=d["ret_bias"],
                              state_in=G.pack_state(scan_in, tail_in), dstate_out=G.pack_state(dscan, dtail))
    ora = _oracle_modes(B, L, H, F, Kc, d, True, True, amp_mode=1, scan_in=scan_in.astype(np.float64), tail_in=tail_in,
                        dscan_out=dscan.astype(np.float64), dtail_out=dtail.astype(np.float64))
    _compare(out, ora, Kc, names=_names_modes(Kc, True, True))
    dscan_in, dtail_in = G.unpack_state(out["dstate_in"], B, J, Kc)
    assert G.rel_err(dscan_in, ora["dscan_in"]) <= TOL
    assert G.rel_err(dtail_in, ora["dtail_in"]) <= TOL


@pytest.mark.parametrize("valve,ret", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("H,F,Kc", [(4, 64, 3), (2, 32, 4), (1, 128, 0)])
def test_hconv_backward_with_valve_and_retention_bf16(valve, ret, H, F, Kc):
    G = _gpu()
    B, L = 2, 300
    d = _inputs_modes(B, L, H, F, Kc, 7100 + H * 131 + F + Kc)
    for k in ("mag", "ang", "dc_re", "dc_im"):
        d[k] = G.bf16_exact(d[k])
    out = G.run_hconv_fwd_bwd(d, B, L, H, F, conv_k=Kc, amp_mode=1, bf16=True, valve=d["valve"] if valve else None,
                              ret=d["ret"] if ret else None, ret_bias=d["ret_bias"] if ret else None)
    ora = _oracle_modes(B, L, H, F, Kc, d, valve, ret, amp_mode=1)
    for k in ("c_re", "c_im", "dmag", "dang"):
        assert G.bf16_err(out[k], ora[k]) <= 1.0, k
    _compare(out, ora, Kc, names=[n for n in _names_modes(Kc, valve, ret) if n not in ("c_re", "c_im", "dmag", "dang")])
