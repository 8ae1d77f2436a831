"""Helpers for the GPU parity tests: run libcawn through its C ABI on numpy inputs."""
from __future__ import annotations

import numpy as np
import torch

from paper_2604_04250_amd import binding as K

DEV = "cuda:0"


def rel_err(gpu, ora):
    """max_i |gpu_i - ora_i| / max(|ora_i|, rms(ora)): element-wise relative error with an rms
    floor, because interference cancels some outputs to ~0."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    if ora.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ora * ora)))
    den = np.maximum(np.abs(ora), max(rms, 1e-30))
    return float(np.max(np.abs(gpu - ora) / den))


def dev(a):
    if a is None or isinstance(a, torch.Tensor):
        return a
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def pack_state(scan, tail):
    """[B,2,J] and [B,Kc-1,2,J] float32 -> flat state blob."""
    parts = [np.asarray(scan, np.float32).ravel()]
    if tail is not None and tail.size:
        parts.append(np.asarray(tail, np.float32).ravel())
    return np.concatenate(parts)


def unpack_state(blob, B, J, Kc):
    blob = np.asarray(blob)
    scan = blob[:B * 2 * J].reshape(B, 2, J)
    tail = blob[B * 2 * J:].reshape(B, max(Kc - 1, 0), 2, J) if Kc > 1 else None
    return scan, tail


class Workspaces:
    """One workspace per size, initialised once and reused across calls (as a caller would)."""
    _cache = {}

    @classmethod
    def get(cls, d):
        n = K.cawn_workspace_bytes(d)
        ws = cls._cache.get("ws")
        if ws is None or ws.numel() * 4 < n:
            ws = torch.empty((max(n, 8 << 20) + 3) // 4, dtype=torch.int32, device=DEV)
            K.check(K.cawn_workspace_init(ws))
            cls._cache["ws"] = ws
        return ws


def run_fwd(inp, B, L, H, F, conv_k=0, amp_mode=0, gate_tau=0.0, conv_clamp=50.0, out_clamp=100.0,
            state_in=None, want_mask=True, want_ckpt=False, concat=False, in_place_state=False,
            cached=0, ws=None, valve=None, valve_eps=0.001, ret=None, ret_bias=None, hconv_w=None,
            hconv_b=None, bf16=False):
    """inp: dict with mag, ang [B,L,J], gamma, theta, conv_w, conv_b (numpy float32).
    Returns dict(z_re, z_im, state_out (flat blob), mask [B,L,W] uint32, ckpt).
    hconv_w [2,H,3] (and hconv_b [2,H]): the harmonic convolution's entry point, z_re / z_im are then
    the convolved planes; with bf16 the inputs (bf16-exact fp32 arrays) and outputs are bfloat16 in memory."""
    J = H * F
    if hconv_w is not None:
        return _run_fwd_hconv(inp, B, L, H, F, conv_k, amp_mode, gate_tau, conv_clamp, out_clamp, state_in, want_mask,
                              want_ckpt, concat, cached, ws, valve, valve_eps, ret, ret_bias, hconv_w, hconv_b, bf16)
    assert not bf16
    d = K.make_desc(B, L, H, F, conv_k=conv_k, amp_mode=amp_mode, gate_tau=gate_tau,
                    conv_clamp=conv_clamp, out_clamp=out_clamp, lane_consts_cached=cached,
                    gate_mode=0 if valve is None else 1, valve_eps=valve_eps, ret_mode=0 if ret is None else 1)
    mag, ang = dev(inp["mag"][:, :L]), dev(inp["ang"][:, :L])
    gamma, theta = dev(inp.get("gamma")), dev(inp["theta"])
    cw = dev(inp["conv_w"]) if conv_k > 0 else None
    cb = dev(inp["conv_b"]) if conv_k > 0 and inp.get("conv_b") is not None else None
    if concat:
        z = torch.full((B, max(L, 1), 2 * J), float("nan"), device=DEV)
        z_re, z_im = z[:, :, :J], z[:, :, J:]
        d.out_stride_t, d.out_stride_b = 2 * J, max(L, 1) * 2 * J
    else:
        z_re = torch.full((B, max(L, 1), J), float("nan"), device=DEV)
        z_im = torch.full((B, max(L, 1), J), float("nan"), device=DEV)
    nstate = K.cawn_state_bytes(d) // 4
    st_in = dev(state_in) if state_in is not None else None
    if in_place_state:
        assert st_in is not None
        st_out = st_in
    else:
        st_out = torch.full((nstate,), float("nan"), device=DEV)
    W = (J + 31) // 32
    mask = torch.zeros((B, max(L, 1), W), dtype=torch.int32, device=DEV) if want_mask else None
    ckpt = torch.full((max(K.cawn_ckpt_bytes(d) // 4, 1),), float("nan"), device=DEV) if want_ckpt else None
    ws = ws if ws is not None else Workspaces.get(d)
    if ret is not None:
        vl = None if valve is None else dev(np.ascontiguousarray(valve[:, :L]))
        K.check(K.cawn_phase_accumulate_ret_fwd(d, mag, ang, vl, dev(np.ascontiguousarray(ret[:, :L])), dev(ret_bias),
                                                theta, cw, cb, st_in, z_re, z_im, st_out, ckpt, mask, ws))
    elif valve is None:
        K.check(K.cawn_phase_accumulate_fwd(d, mag, ang, gamma, theta, cw, cb, st_in, z_re, z_im, st_out,
                                            ckpt, mask, ws))
    else:
        K.check(K.cawn_phase_accumulate_valve_fwd(d, mag, ang, dev(np.ascontiguousarray(valve[:, :L])), gamma,
                                                  theta, cw, cb, st_in, z_re, z_im, st_out, ckpt, mask, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    out = dict(z_re=z_re[:, :L].cpu().numpy(), z_im=z_im[:, :L].cpu().numpy(),
               state_out=st_out.cpu().numpy())
    if want_mask:
        out["mask"] = mask[:, :L].cpu().numpy().view(np.uint32)
    if want_ckpt:
        out["ckpt"] = ckpt.cpu().numpy()
    return out


def _run_fwd_hconv(inp, B, L, H, F, conv_k, amp_mode, gate_tau, conv_clamp, out_clamp, state_in, want_mask,
                   want_ckpt, concat, cached, ws, valve, valve_eps, ret, ret_bias, hconv_w, hconv_b, bf16):
    J = H * F
    d = K.make_desc(B, L, H, F, conv_k=conv_k, amp_mode=amp_mode, gate_tau=gate_tau,
                    conv_clamp=conv_clamp, out_clamp=out_clamp, lane_consts_cached=cached,
                    gate_mode=0 if valve is None else 1, valve_eps=valve_eps, ret_mode=0 if ret is None else 1,
                    hconv_k=3)
    dt = torch.bfloat16 if bf16 else torch.float32
    mag, ang = dev(inp["mag"][:, :L]).to(dt), dev(inp["ang"][:, :L]).to(dt)
    gamma, theta = dev(inp.get("gamma")), dev(inp["theta"])
    cw = dev(inp["conv_w"]) if conv_k > 0 else None
    cb = dev(inp["conv_b"]) if conv_k > 0 and inp.get("conv_b") is not None else None
    Lr = max(L, 1)
    if concat:
        z = torch.full((B, Lr, 2 * J), float("nan"), device=DEV, dtype=dt)
        z_re, z_im = z[:, :, :J], z[:, :, J:]
        d.out_stride_t, d.out_stride_b = 2 * J, Lr * 2 * J
    else:
        z_re = torch.full((B, Lr, J), float("nan"), device=DEV, dtype=dt)
        z_im = torch.full((B, Lr, J), float("nan"), device=DEV, dtype=dt)
    nstate = K.cawn_state_bytes(d) // 4
    st_in = dev(state_in) if state_in is not None else None
    st_out = torch.full((nstate,), float("nan"), device=DEV)
    W = (J + 31) // 32
    mask = torch.zeros((B, Lr, W), dtype=torch.int32, device=DEV) if want_mask else None
    ckpt = torch.full((max(K.cawn_ckpt_bytes(d) // 4, 1),), float("nan"), device=DEV) if want_ckpt else None
    ws = ws if ws is not None else Workspaces.get(d)
    vl = None if valve is None else dev(np.ascontiguousarray(valve[:, :L]))
    rt = None if ret is None else dev(np.ascontiguousarray(ret[:, :L]))
    K.check(K.cawn_phase_accumulate_hconv_fwd(d, mag, ang, vl, rt, dev(ret_bias), gamma, theta, cw, cb,
                                              dev(np.ascontiguousarray(hconv_w, dtype=np.float32)),
                                              dev(hconv_b), st_in, z_re, z_im, st_out, ckpt, mask, ws,
                                              activations_bf16=1 if bf16 else 0))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    out = dict(z_re=z_re[:, :L].float().cpu().numpy(), z_im=z_im[:, :L].float().cpu().numpy(),
               state_out=st_out.cpu().numpy())
    if want_mask:
        out["mask"] = mask[:, :L].cpu().numpy().view(np.uint32)
    if want_ckpt:
        out["ckpt"] = ckpt.cpu().numpy()
    return out


def mask_from_gate(gate):
    """oracle gate bytes [B,L,J] -> packed uint32 words [B,L,ceil(J/32)], bit j%32 of word j/32."""
    B, L, J = gate.shape
    W = (J + 31) // 32
    g = np.zeros((B, L, W * 32), dtype=np.uint8)
    g[..., :J] = gate
    bits = np.packbits(g.reshape(B, L, W, 32), axis=-1, bitorder="little")   # 4 bytes, little endian
    return bits.view("<u4").reshape(B, L, W)


def run_fwd_bwd(inp, B, L, H, F, conv_k=0, amp_mode=0, gate_tau=0.0, conv_clamp=50.0, out_clamp=100.0,
                grad_clamp=100.0, state_in=None, dstate_out=None, want_param=True, want_dstate=True,
                accumulate=0, preset=None, ws=None, valve=None, valve_eps=0.001, want_dvalve=True,
                ret=None, ret_bias=None, want_dret=True, concat=False):
    """Forward (to get the checkpoints) then backward through the C ABI.  inp additionally holds
    dz_re, dz_im [B,L,J].  Returns dict of numpy arrays: dmag, dang, dgamma, dtheta, dconv_w, dconv_b,
    dstate_in (flat blob)."""
    J = H * F
    d = K.make_desc(B, L, H, F, conv_k=conv_k, amp_mode=amp_mode, gate_tau=gate_tau, conv_clamp=conv_clamp,
                    out_clamp=out_clamp, grad_clamp=grad_clamp, accumulate_param_grads=accumulate,
                    gate_mode=0 if valve is None else 1, valve_eps=valve_eps, ret_mode=0 if ret is None else 1)
    vlv = None if valve is None else dev(np.ascontiguousarray(valve[:, :L]))
    rt = None if ret is None else dev(np.ascontiguousarray(ret[:, :L]))
    rbias = dev(ret_bias)
    mag, ang = dev(inp["mag"][:, :L]), dev(inp["ang"][:, :L])
    gamma, theta = dev(inp.get("gamma")), dev(inp["theta"])
    cw = dev(inp["conv_w"]) if conv_k > 0 else None
    cb = dev(inp["conv_b"]) if conv_k > 0 and inp.get("conv_b") is not None else None
    z_re = torch.empty((B, max(L, 1), J), device=DEV)
    z_im = torch.empty((B, max(L, 1), J), device=DEV)
    if concat:
        # Concat layout (Sec. 3.5): the two planes of every activation pair share rows of 2 J elements,
        # inputs [mag | ang], outputs [Z_re | Z_im], and their gradients likewise
        Lr = max(L, 1)
        xin = torch.cat([mag, ang], dim=2).contiguous()
        mag, ang = xin[:, :, :J], xin[:, :, J:]
        zc = torch.empty((B, Lr, 2 * J), device=DEV)
        z_re, z_im = zc[:, :, :J], zc[:, :, J:]
        d.in_stride_t, d.in_stride_b = 2 * J, Lr * 2 * J
        d.out_stride_t, d.out_stride_b = 2 * J, Lr * 2 * J
    st_in = dev(state_in)
    ckpt = torch.full((max(K.cawn_ckpt_bytes(d) // 4, 1),), float("nan"), device=DEV)
    ws = ws if ws is not None else Workspaces.get(d)
    if ret is not None:
        K.check(K.cawn_phase_accumulate_ret_fwd(d, mag, ang, vlv, rt, rbias, theta, cw, cb, st_in, z_re, z_im, None,
                                                ckpt, None, ws))
    elif valve is None:
        K.check(K.cawn_phase_accumulate_fwd(d, mag, ang, gamma, theta, cw, cb, st_in, z_re, z_im, None, ckpt, None, ws))
    else:
        K.check(K.cawn_phase_accumulate_valve_fwd(d, mag, ang, vlv, gamma, theta, cw, cb, st_in, z_re, z_im, None,
                                                  ckpt, None, ws))
    dz_re, dz_im = dev(inp["dz_re"][:, :L]), dev(inp["dz_im"][:, :L])
    dmag = torch.full((B, max(L, 1), J), float("nan"), device=DEV)
    dang = torch.full((B, max(L, 1), J), float("nan"), device=DEV)
    if concat:
        dzc = torch.cat([dz_re, dz_im], dim=2).contiguous()
        dz_re, dz_im = dzc[:, :, :J], dzc[:, :, J:]
        dxc = torch.full((B, max(L, 1), 2 * J), float("nan"), device=DEV)
        dmag, dang = dxc[:, :, :J], dxc[:, :, J:]
    nstate = K.cawn_state_bytes(d) // 4
    fill = float("nan") if preset is None else preset
    dgamma = torch.full((J,), fill, device=DEV) if want_param and ret is None else None
    dtheta = torch.full((J,), fill, device=DEV) if want_param else None
    dcw = torch.full((2, J, conv_k), fill, device=DEV) if want_param and conv_k > 0 else None
    dcb = torch.full((2, J), fill, device=DEV) if want_param and conv_k > 0 else None
    dst_in = torch.full((nstate,), float("nan"), device=DEV) if want_dstate else None
    d.lane_consts_cached = 1
    dvalve = dret = None
    if ret is not None:
        dvalve = torch.full((B, max(L, 1), H), float("nan"), device=DEV) if want_dvalve and valve is not None else None
        dret = torch.full((B, max(L, 1), H), float("nan"), device=DEV) if want_dret else None
        K.check(K.cawn_phase_accumulate_ret_bwd(d, mag, ang, vlv, rt, rbias, theta, cw, cb, st_in, ckpt, dz_re, dz_im,
                                                dev(dstate_out), dmag, dang, dvalve, dret, dtheta, dcw, dcb,
                                                dst_in, ws))
    elif valve is None:
        K.check(K.cawn_phase_accumulate_bwd(d, mag, ang, gamma, theta, cw, cb, st_in, ckpt, dz_re, dz_im,
                                            dev(dstate_out), dmag, dang, dgamma, dtheta, dcw, dcb, dst_in, ws))
    else:
        dvalve = torch.full((B, max(L, 1), H), float("nan"), device=DEV) if want_dvalve else None
        K.check(K.cawn_phase_accumulate_valve_bwd(d, mag, ang, vlv, gamma, theta, cw, cb, st_in, ckpt, dz_re, dz_im,
                                                  dev(dstate_out), dmag, dang, dvalve, dgamma, dtheta, dcw, dcb,
                                                  dst_in, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    out = dict(dmag=dmag[:, :L].cpu().numpy(), dang=dang[:, :L].cpu().numpy())
    if dvalve is not None:
        out["dvalve"] = dvalve[:, :L].cpu().numpy()
    if dret is not None:
        out["dret"] = dret[:, :L].cpu().numpy()
    for k, v in (("dgamma", dgamma), ("dtheta", dtheta), ("dconv_w", dcw), ("dconv_b", dcb), ("dstate_in", dst_in)):
        if v is not None:
            out[k] = v.cpu().numpy()
    return out


# ---------------------------------------------------------------- bfloat16 activations
def to_bf16(x):
    """float32 array -> uint16 bfloat16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def from_bf16(h):
    return (np.asarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def bf16_exact(x):
    """float32 array rounded to values bfloat16 holds exactly."""
    return from_bf16(to_bf16(x))


def dev_bf16(a):
    """float32 numpy array of bf16-exact values -> torch.bfloat16 device tensor."""
    return torch.from_numpy(to_bf16(a).view(np.int16)).to(DEV).view(torch.bfloat16)


def host_bf16(t):
    return from_bf16(t.view(torch.int16).cpu().numpy().view(np.uint16))


def bf16_err(gpu, ora, tol=1e-4):
    """Worst excess over the bar for an output stored as bfloat16: the kernel's fp32 value may differ from
    the oracle by tol (rms-floored, as everywhere) and is then rounded to nearest: bf16 keeps 8 significant
    bits, so half a unit in the last place is at most 2^-8 relative.  Returns max(|gpu - ora| / bound); <= 1 passes."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    if ora.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ora * ora)))
    den = np.maximum(np.abs(ora), max(rms, 1e-30))
    bound = 2.0 ** -8 * np.abs(ora) * (1 + tol) + tol * den * (1 + 2.0 ** -8)
    return float(np.max(np.abs(gpu - ora) / bound))


def run_fwd_bf16(inp, B, L, H, F, conv_k=0, amp_mode=0, gate_tau=0.0, state_in=None, valve=None, ret=None,
                 ret_bias=None, want_ckpt=False, concat=False, valve_eps=0.001):
    """Forward with bfloat16 activations; inp["mag"], inp["ang"] hold bf16-exact float32 values.
    Returns z_re, z_im as float32 (widened from what the kernel stored), state_out, mask."""
    J = H * F
    d = K.make_desc(B, L, H, F, conv_k=conv_k, amp_mode=amp_mode, gate_tau=gate_tau,
                    gate_mode=0 if valve is None else 1, valve_eps=valve_eps, ret_mode=0 if ret is None else 1)
    mag, ang = dev_bf16(inp["mag"][:, :L]), dev_bf16(inp["ang"][:, :L])
    gamma, theta = dev(inp.get("gamma")), dev(inp["theta"])
    cw = dev(inp["conv_w"]) if conv_k > 0 else None
    cb = dev(inp["conv_b"]) if conv_k > 0 and inp.get("conv_b") is not None else None
    if concat:
        z = torch.full((B, max(L, 1), 2 * J), float("nan"), device=DEV, dtype=torch.bfloat16)
        z_re, z_im = z[:, :, :J], z[:, :, J:]
        d.out_stride_t, d.out_stride_b = 2 * J, max(L, 1) * 2 * J
    else:
        z_re = torch.full((B, max(L, 1), J), float("nan"), device=DEV, dtype=torch.bfloat16)
        z_im = torch.full((B, max(L, 1), J), float("nan"), device=DEV, dtype=torch.bfloat16)
    nstate = K.cawn_state_bytes(d) // 4
    st_in = dev(state_in) if state_in is not None else None
    st_out = torch.full((nstate,), float("nan"), device=DEV)
    W = (J + 31) // 32
    mask = torch.zeros((B, max(L, 1), W), dtype=torch.int32, device=DEV)
    ckpt = torch.full((max(K.cawn_ckpt_bytes(d) // 4, 1),), float("nan"), device=DEV) if want_ckpt else None
    ws = Workspaces.get(d)
    vl = None if valve is None else dev(np.ascontiguousarray(valve[:, :L]))
    rt = None if ret is None else dev(np.ascontiguousarray(ret[:, :L]))
    K.check(K.cawn_phase_accumulate_bf16_fwd(d, mag, ang, vl, rt, dev(ret_bias), gamma, theta, cw, cb, st_in, z_re, z_im,
                                             st_out, ckpt, mask, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    out = dict(z_re=host_bf16(z_re[:, :L].contiguous()), z_im=host_bf16(z_im[:, :L].contiguous()),
               state_out=st_out.cpu().numpy(), mask=mask[:, :L].cpu().numpy().view(np.uint32))
    if want_ckpt:
        out["ckpt"] = ckpt.cpu().numpy()
    return out


def run_hconv_fwd_bwd(inp, B, L, H, F, conv_k=0, amp_mode=0, gate_tau=0.0, out_clamp=100.0, grad_clamp=100.0,
                      state_in=None, dstate_out=None, accumulate=0, preset=None, concat=False, want_hgrads=True,
                      bf16=False, valve=None, ret=None, ret_bias=None, valve_eps=0.001):
    """Forward with the harmonic convolution (for the checkpoints and the convolved output), then its backward,
    through the C ABI.  inp holds hconv_w [2,H,3], hconv_b [2,H] and dc_re, dc_im [B,L,J] (gradients of the
    convolved output).  Returns numpy arrays: c_re, c_im, dmag, dang, dgamma, dtheta, dconv_w, dconv_b, dhconv_w,
    dhconv_b, dstate_in (flat blob).  bf16: mag, ang, dc_re, dc_im (bf16-exact fp32 arrays) go in as bfloat16, c_re,
    c_im, dmag, dang come back widened from what the kernels stored.  valve [B,L,H] selects gate_mode 1 (dvalve
    comes back), ret [B,L,H] with ret_bias [H,F] ret_mode 1 (dret comes back, no dgamma)."""
    J = H * F
    d = K.make_desc(B, L, H, F, conv_k=conv_k, amp_mode=amp_mode, gate_tau=gate_tau, out_clamp=out_clamp,
                    grad_clamp=grad_clamp, accumulate_param_grads=accumulate, hconv_k=3,
                    gate_mode=0 if valve is None else 1, valve_eps=valve_eps, ret_mode=0 if ret is None else 1)
    vl = None if valve is None else dev(np.ascontiguousarray(valve[:, :L]))
    rt = None if ret is None else dev(np.ascontiguousarray(ret[:, :L]))
    rb = dev(ret_bias)
    up = dev_bf16 if bf16 else dev
    adt = torch.bfloat16 if bf16 else torch.float32
    mag, ang = up(inp["mag"][:, :L]), up(inp["ang"][:, :L])
    gamma, theta = dev(inp.get("gamma")), dev(inp["theta"])
    cw = dev(inp["conv_w"]) if conv_k > 0 else None
    cb = dev(inp["conv_b"]) if conv_k > 0 and inp.get("conv_b") is not None else None
    hw, hb = dev(inp["hconv_w"]), dev(inp.get("hconv_b"))
    Lr = max(L, 1)
    c_re, c_im = torch.empty((B, Lr, J), device=DEV, dtype=adt), torch.empty((B, Lr, J), device=DEV, dtype=adt)
    dc_re, dc_im = up(inp["dc_re"][:, :L]), up(inp["dc_im"][:, :L])
    nanv = lambda *shape: torch.full(shape, float("nan") if preset is None else preset, device=DEV)
    dmag = torch.full((B, Lr, J), float("nan"), device=DEV, dtype=adt)
    dang = torch.full((B, Lr, J), float("nan"), device=DEV, dtype=adt)
    if concat:      # rows of 2 J elements shared by each activation pair (Sec. 3.5)
        xin = torch.cat([mag, ang], dim=2).contiguous()
        mag, ang = xin[:, :, :J], xin[:, :, J:]
        cc = torch.empty((B, Lr, 2 * J), device=DEV, dtype=adt)
        c_re, c_im = cc[:, :, :J], cc[:, :, J:]
        dcc = torch.cat([dc_re, dc_im], dim=2).contiguous()
        dc_re, dc_im = dcc[:, :, :J], dcc[:, :, J:]
        dxc = torch.full((B, Lr, 2 * J), float("nan"), device=DEV, dtype=adt)
        dmag, dang = dxc[:, :, :J], dxc[:, :, J:]
        d.in_stride_t, d.in_stride_b = 2 * J, Lr * 2 * J
        d.out_stride_t, d.out_stride_b = 2 * J, Lr * 2 * J
    st_in = dev(state_in)
    ckpt = torch.full((max(K.cawn_ckpt_bytes(d) // 4, 1),), float("nan"), device=DEV)
    ws = Workspaces.get(d)
    K.check(K.cawn_phase_accumulate_hconv_fwd(d, mag, ang, vl, rt, rb, gamma, theta, cw, cb, hw, hb, st_in, c_re, c_im,
                                              None, ckpt, None, ws, activations_bf16=1 if bf16 else 0))
    nstate = K.cawn_state_bytes(d) // 4
    dgamma, dtheta = (nanv(J) if ret is None else None), nanv(J)
    dvl = None if valve is None else torch.full((B, Lr, H), float("nan"), device=DEV)
    drt = None if ret is None else torch.full((B, Lr, H), float("nan"), device=DEV)
    dcw = nanv(2, J, conv_k) if conv_k > 0 else None
    dcb = nanv(2, J) if conv_k > 0 else None
    dhw = nanv(2, H, 3) if want_hgrads else None
    dhb = nanv(2, H) if want_hgrads else None
    dst_in = torch.full((nstate,), float("nan"), device=DEV)
    d.lane_consts_cached = 1
    K.check(K.cawn_phase_accumulate_hconv_bwd(d, mag, ang, vl, rt, rb, gamma, theta, cw, cb, hw, hb, st_in, ckpt, dc_re,
                                              dc_im, dev(dstate_out), dmag, dang, dvl, drt, dgamma, dtheta, dcw, dcb, dhw,
                                              dhb, dst_in, ws, activations_bf16=1 if bf16 else 0))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    host = (lambda t: host_bf16(t[:, :L].contiguous())) if bf16 else (lambda t: t[:, :L].cpu().numpy())
    out = dict(c_re=host(c_re), c_im=host(c_im), dmag=host(dmag), dang=host(dang),
               dtheta=dtheta.cpu().numpy(), dstate_in=dst_in.cpu().numpy())
    for k, v in (("dgamma", dgamma), ("dconv_w", dcw), ("dconv_b", dcb), ("dhconv_w", dhw), ("dhconv_b", dhb)):
        if v is not None:
            out[k] = v.cpu().numpy()
    for k, v in (("dvalve", dvl), ("dret", drt)):
        if v is not None:
            out[k] = v[:, :L].cpu().numpy()
    return out


def run_fwd_bwd_bf16(inp, B, L, H, F, conv_k=0, amp_mode=0, gate_tau=0.0, grad_clamp=100.0, state_in=None,
                     dstate_out=None, want_param=True, valve=None, ret=None, ret_bias=None, valve_eps=0.001,
                     concat=False):
    """Forward (for the checkpoints) then backward, bfloat16 activations.  dmag, dang come back as float32
    (widened from what the kernel stored); the other gradients are fp32."""
    J = H * F
    d = K.make_desc(B, L, H, F, conv_k=conv_k, amp_mode=amp_mode, gate_tau=gate_tau, grad_clamp=grad_clamp,
                    gate_mode=0 if valve is None else 1, valve_eps=valve_eps, ret_mode=0 if ret is None else 1)
    mag, ang = dev_bf16(inp["mag"][:, :L]), dev_bf16(inp["ang"][:, :L])
    dz_re, dz_im = dev_bf16(inp["dz_re"][:, :L]), dev_bf16(inp["dz_im"][:, :L])
    gamma, theta = dev(inp.get("gamma")), dev(inp["theta"])
    cw = dev(inp["conv_w"]) if conv_k > 0 else None
    cb = dev(inp["conv_b"]) if conv_k > 0 and inp.get("conv_b") is not None else None
    vl = None if valve is None else dev(np.ascontiguousarray(valve[:, :L]))
    rt = None if ret is None else dev(np.ascontiguousarray(ret[:, :L]))
    rb = dev(ret_bias)
    z_re = torch.empty((B, max(L, 1), J), device=DEV, dtype=torch.bfloat16)
    z_im = torch.empty((B, max(L, 1), J), device=DEV, dtype=torch.bfloat16)
    dmag = torch.full((B, max(L, 1), J), float("nan"), device=DEV, dtype=torch.bfloat16)
    dang = torch.full((B, max(L, 1), J), float("nan"), device=DEV, dtype=torch.bfloat16)
    if concat:      # rows of 2 J elements shared by each activation pair (Sec. 3.5)
        Lr = max(L, 1)
        xin = torch.cat([mag, ang], dim=2).contiguous()
        mag, ang = xin[:, :, :J], xin[:, :, J:]
        zc = torch.empty((B, Lr, 2 * J), device=DEV, dtype=torch.bfloat16)
        z_re, z_im = zc[:, :, :J], zc[:, :, J:]
        dzc = torch.cat([dz_re, dz_im], dim=2).contiguous()
        dz_re, dz_im = dzc[:, :, :J], dzc[:, :, J:]
        dxc = torch.full((B, Lr, 2 * J), float("nan"), device=DEV, dtype=torch.bfloat16)
        dmag, dang = dxc[:, :, :J], dxc[:, :, J:]
        d.in_stride_t, d.in_stride_b = 2 * J, Lr * 2 * J
        d.out_stride_t, d.out_stride_b = 2 * J, Lr * 2 * J
    st_in = dev(state_in)
    ckpt = torch.full((max(K.cawn_ckpt_bytes(d) // 4, 1),), float("nan"), device=DEV)
    ws = Workspaces.get(d)
    K.check(K.cawn_phase_accumulate_bf16_fwd(d, mag, ang, vl, rt, rb, gamma, theta, cw, cb, st_in, z_re, z_im, None, ckpt,
                                             None, ws))
    nstate = K.cawn_state_bytes(d) // 4
    nanv = lambda *shape: torch.full(shape, float("nan"), device=DEV)
    dgamma = nanv(J) if want_param and ret is None else None
    dtheta = nanv(J) if want_param else None
    dcw = nanv(2, J, conv_k) if want_param and conv_k > 0 else None
    dcb = nanv(2, J) if want_param and conv_k > 0 else None
    dvalve = nanv(B, max(L, 1), H) if valve is not None else None
    dret = nanv(B, max(L, 1), H) if ret is not None else None
    dst_in = nanv(nstate)
    d.lane_consts_cached = 1
    K.check(K.cawn_phase_accumulate_bf16_bwd(d, mag, ang, vl, rt, rb, gamma, theta, cw, cb, st_in, ckpt, dz_re, dz_im,
                                             dev(dstate_out), dmag, dang, dvalve, dret, dgamma, dtheta, dcw, dcb,
                                             dst_in, ws))
    torch.cuda.synchronize()
    K.check(K.cawn_workspace_status(ws))
    out = dict(dmag=host_bf16(dmag[:, :L].contiguous()), dang=host_bf16(dang[:, :L].contiguous()),
               dstate_in=dst_in.cpu().numpy())
    for k, v in (("dgamma", dgamma), ("dtheta", dtheta), ("dconv_w", dcw), ("dconv_b", dcb)):
        if v is not None:
            out[k] = v.cpu().numpy()
    if dvalve is not None:
        out["dvalve"] = dvalve[:, :L].cpu().numpy()
    if dret is not None:
        out["dret"] = dret[:, :L].cpu().numpy()
    return out
