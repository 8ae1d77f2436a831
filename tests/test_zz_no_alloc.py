"""The allocation-free forward entry point (cawn_phase_accumulate_fwd_static: its workspace is a static
device array inside the library) against cawn_phase_accumulate_fwd on a caller workspace, through the
C ABI: two calls in a row on the shared array, the second with a smaller input, then a chunked pair with
the state carried in place; and the host-side refusal of descriptors beyond the array's size."""
import ctypes as C

import numpy as np
import pytest

TOL = 1e-4


def _inputs(B, L, H, F, Kc, seed):
    r = np.random.Generator(np.random.PCG64(seed))
    J = H * F
    return dict(mag=r.standard_normal((B, L, J), dtype=np.float32), ang=r.standard_normal((B, L, J), dtype=np.float32),
                gamma=r.uniform(0.95, 0.9999, J).astype(np.float32), theta=r.uniform(0, np.pi, J).astype(np.float32),
                conv_w=(r.standard_normal((2, J, Kc)) / np.sqrt(Kc)).astype(np.float32),
                conv_b=(0.1 * r.standard_normal((2, J))).astype(np.float32))


def _static_fwd(K, G, torch, inp, B, L, H, F, Kc, tau, state_in=None, want_ckpt=True):
    J = H * F
    d = K.make_desc(B, L, H, F, conv_k=Kc, gate_tau=tau)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(G.DEV)
    z_re = torch.full((B, L, J), float("nan"), device=G.DEV)
    z_im = torch.full((B, L, J), float("nan"), device=G.DEV)
    st_out = torch.full((K.cawn_state_bytes(d) // 4,), float("nan"), device=G.DEV)
    mask = torch.zeros((B, L, (J + 31) // 32), dtype=torch.int32, device=G.DEV)
    ckpt = torch.full((K.cawn_ckpt_bytes(d) // 4,), float("nan"), device=G.DEV) if want_ckpt else None
    st_in = t(state_in) if state_in is not None else None
    K.check(K.cawn_phase_accumulate_fwd_static(d, t(inp["mag"][:, :L]), t(inp["ang"][:, :L]), t(inp["gamma"]),
                                               t(inp["theta"]), t(inp["conv_w"]), t(inp["conv_b"]), st_in, z_re, z_im,
                                               st_out, ckpt, mask))
    torch.cuda.synchronize()
    out = dict(z_re=z_re.cpu().numpy(), z_im=z_im.cpu().numpy(), state_out=st_out.cpu().numpy(),
               mask=mask.cpu().numpy().view(np.uint32))
    if want_ckpt:
        out["ckpt"] = ckpt.cpu().numpy()
    return out


def _same(G, a, b, keys):
    for k in keys:
        if k == "mask":
            assert np.array_equal(a[k], b[k]), k
        else:
            assert np.all(np.isfinite(a[k])), k
            assert G.rel_err(a[k], b[k]) <= TOL, (k, G.rel_err(a[k], b[k]))


@pytest.mark.gpu
def test_static_scratch_forward_matches_the_workspace_forward_twice_in_a_row():
    import torch
    import gpu_util as G
    from paper_2604_04250_amd import binding as K

    H, F, Kc, tau = 12, 64, 4, 0.1
    big = _inputs(3, 1500, H, F, Kc, 7001)         # six tiles per chain with a ragged tail, 72 chains
    small = _inputs(2, 333, H, F, Kc, 7002)        # a smaller call on the same array right behind it
    keys = ("z_re", "z_im", "state_out", "mask", "ckpt")
    for inp, B, L in ((big, 3, 1500), (small, 2, 333)):
        ref = G.run_fwd(inp, B, L, H, F, conv_k=Kc, gate_tau=tau, want_ckpt=True)
        got = _static_fwd(K, G, torch, inp, B, L, H, F, Kc, tau)
        _same(G, got, ref, keys)
    # chunked: the state leaves one call of the static entry point and enters the next
    whole = G.run_fwd(big, 3, 1500, H, F, conv_k=Kc, gate_tau=tau)
    c1 = _static_fwd(K, G, torch, big, 3, 1000, H, F, Kc, tau, want_ckpt=False)
    rest = {k: (v[:, 1000:] if k in ("mag", "ang") else v) for k, v in big.items()}
    c2 = _static_fwd(K, G, torch, rest, 3, 500, H, F, Kc, tau, state_in=c1["state_out"], want_ckpt=False)
    got = dict(z_re=np.concatenate([c1["z_re"], c2["z_re"]], 1), z_im=np.concatenate([c1["z_im"], c2["z_im"]], 1),
               state_out=c2["state_out"], mask=np.concatenate([c1["mask"], c2["mask"]], 1))
    _same(G, got, whole, ("z_re", "z_im", "state_out", "mask"))
    # a single-token call (the decode kernel) on the same array
    one = _inputs(2, 1, H, F, Kc, 7003)
    _same(G, _static_fwd(K, G, torch, one, 2, 1, H, F, Kc, tau, want_ckpt=False),
          G.run_fwd(one, 2, 1, H, F, conv_k=Kc, gate_tau=tau), ("z_re", "z_im", "state_out", "mask"))


def test_static_scratch_forward_refuses_what_does_not_fit():
    """Host-side checks only: nothing is launched (fake pointers are never dereferenced)."""
    from paper_2604_04250_amd import binding as K

    L_ = K.lib()
    fake, null = C.c_void_p(0x1000), C.c_void_p(None)
    args = [fake] * 6 + [null, fake, fake, null, null, null]
    too_long = K.make_desc(8, 1 << 16, 12, 64, conv_k=4)          # 8 x 256 tiles x 768 lanes x 32 B = 50 MiB
    assert L_.cawn_phase_accumulate_fwd_static(C.byref(too_long), *args, null) == K.CAWN_EWORKSPACE
    wide = K.make_desc(2, 32768, 32, 128, conv_k=4)
    assert L_.cawn_phase_accumulate_fwd_static(C.byref(wide), *args, null) == K.CAWN_EWORKSPACE
    for bad in (K.make_desc(2, 128, 2, 32, gate_mode=1), K.make_desc(2, 128, 2, 32, ret_mode=1),
                K.make_desc(2, 128, 2, 32, hconv_k=3), K.make_desc(0, 128, 2, 32)):
        assert L_.cawn_phase_accumulate_fwd_static(C.byref(bad), *args, null) == K.CAWN_EINVAL
