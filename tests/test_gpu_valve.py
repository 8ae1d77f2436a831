"""GPU parity of the per-head input valve (gate_mode 1, Sec. 3.3 "Hard-Threshold Gating") against
the fp64 oracle, through the C ABI.  Bar as for the other parity tests: rms-floored relative error
<= 1e-4, valve masks bit-exact."""
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
             gamma=r.uniform(0.9, 0.999, J).astype(np.float32),
             theta=r.uniform(0, np.pi, J).astype(np.float32),
             # logits around the paper's closing point 3 + ln(0.001/0.999) = -3.907 and well above it
             valve=(-3.9 + 3.0 * r.standard_normal((B, L, H))).astype(np.float32),
             dz_re=r.standard_normal((B, L, J), dtype=np.float32),
             dz_im=r.standard_normal((B, L, J), dtype=np.float32))
    kk = max(Kc, 1)
    d["conv_w"] = (r.standard_normal((2, J, kk)) / np.sqrt(kk)).astype(np.float32)
    d["conv_b"] = (0.1 * r.standard_normal((2, J))).astype(np.float32)
    return d


def _check_fwd(B, L, H, F, Kc, d, amp_mode=0, eps=0.001, state=None, **kw):
    G = _gpu()
    J = H * F
    scan_in = tail_in = blob = None
    if state is not None:
        scan_in, tail_in = state
        blob = G.pack_state(scan_in, tail_in if Kc > 1 else None)
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_mode=1, valve_eps=eps)
    ora = O.phase_fwd(cfg, d["mag"][:, :L], d["ang"][:, :L], d["gamma"], d["theta"], conv_w=d["conv_w"],
                      conv_b=d["conv_b"], valve=d["valve"][:, :L],
                      scan_in=None if scan_in is None else scan_in.astype(np.float64),
                      tail_in=tail_in if Kc > 1 else None)
    out = G.run_fwd(d, B, L, H, F, conv_k=Kc, amp_mode=amp_mode, state_in=blob, valve=d["valve"], valve_eps=eps, **kw)
    assert G.rel_err(out["z_re"], ora["z_re"]) <= TOL and G.rel_err(out["z_im"], ora["z_im"]) <= TOL
    assert np.array_equal(out["mask"], G.mask_from_gate(ora["gate"])), "valve mask differs"
    scan, tail = G.unpack_state(out["state_out"], B, J, Kc)
    assert G.rel_err(scan, ora["scan_out"]) <= TOL
    return out, ora


@pytest.mark.parametrize("H,F", [(3, 64), (2, 32), (4, 16), (8, 8), (1, 128), (5, 32), (3, 16), (5, 8)])
@pytest.mark.parametrize("Kc", [0, 4])
def test_valve_forward_head_widths(H, F, Kc):
    B, L = 2, 700                      # three forward tiles, ragged tail
    d = _inputs(B, L, H, F, Kc, 700 + H * 131 + F + Kc)
    out, ora = _check_fwd(B, L, H, F, Kc, d)
    closed = 1.0 - ora["gate"].mean()
    assert 0.3 < closed < 0.7          # logits straddle the closing point


@pytest.mark.parametrize("L", [1, 5, 16, 17, 255, 256, 257])
def test_valve_forward_lengths_and_short_calls(L):
    B, H, F, Kc = 3, 2, 64, 3
    d = _inputs(B, 300, H, F, Kc, 900 + L)
    _check_fwd(B, L, H, F, Kc, d, amp_mode=1, eps=0.01)


def test_valve_forward_chunked_state_matches_one_pass():
    G = _gpu()
    B, L, H, F, Kc = 2, 1000, 2, 64, 4
    J = H * F
    d = _inputs(B, L, H, F, Kc, 1234)
    one, _ = _check_fwd(B, L, H, F, Kc, d)
    blob = None
    zs = []
    for lo, hi in ((0, 300), (300, 310), (310, 1000)):     # a long, a short (step kernel) and a long call
        part = {k: (v[:, lo:hi] if k in ("mag", "ang", "valve") else v) for k, v in d.items()}
        o = G.run_fwd(part, B, hi - lo, H, F, conv_k=Kc, state_in=blob, valve=part["valve"])
        blob = o["state_out"]
        zs.append(o["z_re"])
    z = np.concatenate(zs, axis=1)
    assert G.rel_err(z, one["z_re"]) <= TOL
    assert G.rel_err(G.unpack_state(blob, B, J, Kc)[0], G.unpack_state(one["state_out"], B, J, Kc)[0]) <= TOL


def test_valve_unsupported_head_width_and_wrong_entry_point():
    import torch
    from paper_2604_04250_amd import binding as K
    x = torch.zeros(8, device="cuda:0")
    d = K.make_desc(1, 8, 2, 12, gate_mode=1)        # F = 12: heads do not tile the 32-lane blocks
    assert K.cawn_phase_accumulate_valve_fwd(d, x, x, x, x, x, None, None, None, x, x, None, None, None, x) == K.CAWN_EUNSUPPORTED
    d = K.make_desc(1, 8, 2, 32, gate_mode=0)
    assert K.cawn_phase_accumulate_valve_fwd(d, x, x, x, x, x, None, None, None, x, x, None, None, None, x) == K.CAWN_EINVAL
    d = K.make_desc(1, 8, 2, 32, gate_mode=1)
    assert K.cawn_phase_accumulate_fwd(d, x, x, x, x, None, None, None, x, x, None, None, None, x) == K.CAWN_EINVAL      # a mode at an entry point that is not its own


def _check_bwd(B, L, H, F, Kc, d, amp_mode=0, eps=0.001, state=None, dstate=None, tol=TOL, **kw):
    G = _gpu()
    J = H * F
    scan_in = tail_in = blob = None
    if state is not None:
        scan_in, tail_in = state
        blob = G.pack_state(scan_in, tail_in if Kc > 1 else None)
    cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_mode=1, valve_eps=eps)
    ora = O.phase_bwd(cfg, d["mag"][:, :L], d["ang"][:, :L], d["gamma"], d["theta"], d["dz_re"][:, :L],
                      d["dz_im"][:, :L], conv_w=d["conv_w"], conv_b=d["conv_b"], valve=d["valve"][:, :L],
                      scan_in=None if scan_in is None else scan_in.astype(np.float64),
                      tail_in=tail_in if Kc > 1 else None)
    out = G.run_fwd_bwd(d, B, L, H, F, conv_k=Kc, amp_mode=amp_mode, state_in=blob, valve=d["valve"],
                        valve_eps=eps, **kw)
    names = ["dmag", "dang", "dvalve", "dgamma", "dtheta"] + (["dconv_w", "dconv_b"] if Kc > 0 else [])
    for n in names:
        if n in out:
            e = G.rel_err(out[n], ora[n])
            assert e <= tol, (n, e)
    return out, ora


@pytest.mark.parametrize("H,F", [(3, 64), (2, 32), (4, 16), (8, 8), (1, 128), (3, 16), (5, 8)])
@pytest.mark.parametrize("Kc", [0, 2, 4])
def test_valve_backward_head_widths(H, F, Kc):
    B, L = 2, 333                      # three backward tiles, ragged tail
    d = _inputs(B, L, H, F, Kc, 1700 + H * 131 + F + Kc)
    out, ora = _check_bwd(B, L, H, F, Kc, d)
    closed = ora["dvalve"][d["valve"][:, :L] < -3.95]      # logits below the closing point still learn
    assert closed.size > 0 and np.abs(closed).max() > 0


def test_valve_backward_without_parameter_gradients_and_softplus_amplitude():
    B, L, H, F, Kc = 2, 400, 2, 64, 4
    d = _inputs(B, L, H, F, Kc, 2100)
    _check_bwd(B, L, H, F, Kc, d, amp_mode=1, eps=0.01, want_param=False)
    _check_bwd(B, L, H, F, Kc, d, amp_mode=1, eps=0.01, want_dvalve=False)


def test_valve_backward_training_shape_sampled():
    """B=4 H=12 F=64 L=2048 (the layer shape of the benchmark configurations), valve mode."""
    B, L, H, F, Kc = 4, 2048, 12, 64, 4
    d = _inputs(B, L, H, F, Kc, 2200)
    d["gamma"] = np.random.Generator(np.random.PCG64(5)).uniform(0.95, 0.9999, H * F).astype(np.float32)
    _check_bwd(B, L, H, F, Kc, d)
