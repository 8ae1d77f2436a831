"""Thin ctypes binding of libcawn's C ABI (include/cawn.h): argument marshalling only.

Every step of the hot path runs in the HIP kernels of libcawn.so.  PyTorch tensors are used as
device-memory handles (``data_ptr()``) and for the current stream; nothing here computes.  If the
shared library has not been built the import of a function fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcawn.so")

CAWN_OK, CAWN_EINVAL, CAWN_EUNSUPPORTED, CAWN_EWORKSPACE, CAWN_ELAUNCH, CAWN_ETIMEOUT = 0, -1, -2, -3, -4, -5

EXPORTS = ["cawn_state_bytes", "cawn_workspace_bytes", "cawn_ckpt_bytes", "cawn_tile_len",
           "cawn_status_string", "cawn_workspace_init", "cawn_workspace_status", "cawn_set_spin_limit",
           "cawn_theta_init", "cawn_syntax_conv", "cawn_phase_accumulate_fwd",
           "cawn_phase_accumulate_bwd", "cawn_phase_accumulate_bf16_bwd", "cawn_phase_accumulate_bf16_fwd", "cawn_phase_accumulate_hconv_fwd", "cawn_phase_accumulate_hconv_bwd", "cawn_phase_accumulate_ret_bwd", "cawn_phase_accumulate_ret_fwd",
           "cawn_phase_accumulate_valve_fwd",
           "cawn_phase_accumulate_valve_bwd", "cawn_stream_copy", "cawn_phase_accumulate_fwd_static"]


class cawn_desc(C.Structure):
    _fields_ = [("B", C.c_int32), ("L", C.c_int32), ("H", C.c_int32), ("F", C.c_int32),
                ("conv_k", C.c_int32), ("amp_mode", C.c_int32), ("gate_mode", C.c_int32),
                ("gate_tau", C.c_float), ("conv_clamp", C.c_float), ("out_clamp", C.c_float),
                ("grad_clamp", C.c_float), ("accumulate_param_grads", C.c_int32),
                ("lane_consts_cached", C.c_int32), ("valve_eps", C.c_float),
                ("ret_mode", C.c_int32), ("hconv_k", C.c_int32),
                ("in_stride_b", C.c_int64), ("in_stride_t", C.c_int64),
                ("out_stride_b", C.c_int64), ("out_stride_t", C.c_int64)]

    @property
    def J(self) -> int:
        return self.H * self.F


def make_desc(B, L, H, F, conv_k=0, amp_mode=0, gate_tau=0.0, conv_clamp=50.0, out_clamp=100.0,
              grad_clamp=100.0, accumulate_param_grads=0, lane_consts_cached=0, in_stride_b=0,
              in_stride_t=0, out_stride_b=0, out_stride_t=0, gate_mode=0, valve_eps=0.001,
              ret_mode=0, hconv_k=0) -> cawn_desc:
    return cawn_desc(B, L, H, F, conv_k, amp_mode, gate_mode, gate_tau, conv_clamp, out_clamp, grad_clamp,
                     accumulate_param_grads, lane_consts_cached, valve_eps, ret_mode, hconv_k, in_stride_b, in_stride_t,
                     out_stride_b, out_stride_t)


_lib = None


def lib() -> C.CDLL:
    """Load libcawn.so; raise if it was not built (python -m paper_2604_04250_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(hipcc --offload-arch=gfx950); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        for n in ("cawn_state_bytes", "cawn_workspace_bytes", "cawn_ckpt_bytes"):
            getattr(L, n).restype = C.c_size_t
            getattr(L, n).argtypes = [C.POINTER(cawn_desc)]
        L.cawn_tile_len.restype = C.c_int32
        L.cawn_status_string.restype = C.c_char_p
        L.cawn_status_string.argtypes = [C.c_int]
        L.cawn_workspace_init.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        L.cawn_workspace_status.argtypes = [C.c_void_p, C.c_void_p]
        L.cawn_set_spin_limit.argtypes = [C.c_uint32]
        L.cawn_set_spin_limit.restype = None
        L.cawn_theta_init.argtypes = [C.c_int32, C.c_int32, C.c_void_p]
        L.cawn_syntax_conv.argtypes = [C.POINTER(cawn_desc), C.c_int32] + [C.c_void_p] * 7
        L.cawn_phase_accumulate_fwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 13 +
                                                [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_bwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 19 +
                                                [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_valve_fwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 14 +
                                                      [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_valve_bwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 21 +
                                                      [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_ret_fwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 15 +
                                                    [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_ret_bwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 22 +
                                                    [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_bf16_fwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 16 +
                                                     [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_bf16_bwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 24 +
                                                     [C.c_size_t, C.c_void_p])
        L.cawn_phase_accumulate_hconv_fwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 18 +
                                                      [C.c_size_t, C.c_int32, C.c_void_p])
        L.cawn_phase_accumulate_hconv_bwd.argtypes = ([C.POINTER(cawn_desc)] + [C.c_void_p] * 28 +
                                                      [C.c_size_t, C.c_int32, C.c_void_p])
        L.cawn_stream_copy.argtypes = [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
        L.cawn_phase_accumulate_fwd_static.argtypes = [C.POINTER(cawn_desc)] + [C.c_void_p] * 13
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda, "libcawn takes device pointers"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def check(status: int) -> None:
    if status != CAWN_OK:
        raise RuntimeError(f"libcawn: {cawn_status_string(status)} ({status})")


def cawn_state_bytes(d: cawn_desc) -> int:
    return int(lib().cawn_state_bytes(C.byref(d)))


def cawn_workspace_bytes(d: cawn_desc) -> int:
    return int(lib().cawn_workspace_bytes(C.byref(d)))


def cawn_ckpt_bytes(d: cawn_desc) -> int:
    return int(lib().cawn_ckpt_bytes(C.byref(d)))


def cawn_tile_len() -> int:
    return int(lib().cawn_tile_len())


def cawn_status_string(status: int) -> str:
    return lib().cawn_status_string(int(status)).decode()


def cawn_workspace_init(workspace: torch.Tensor, stream=None) -> int:
    return lib().cawn_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream))


def cawn_workspace_status(workspace: torch.Tensor, stream=None) -> int:
    return lib().cawn_workspace_status(_ptr(workspace), _stream(stream))


def cawn_set_spin_limit(polls: int) -> None:
    lib().cawn_set_spin_limit(int(polls))


def cawn_theta_init(H: int, F: int):
    """Host helper: the paper's rotation-angle initialisation as a float32 numpy array [H*F]."""
    import numpy as np
    out = np.empty(H * F, dtype=np.float32)
    check(lib().cawn_theta_init(H, F, out.ctypes.data_as(C.c_void_p)))
    return out


def cawn_syntax_conv(d, Cch, x, w, bias, conv_state_in, y, conv_state_out, stream=None) -> int:
    return lib().cawn_syntax_conv(C.byref(d), int(Cch), _ptr(x), _ptr(w), _ptr(bias),
                                  _ptr(conv_state_in), _ptr(y), _ptr(conv_state_out), _stream(stream))


def cawn_phase_accumulate_fwd(d, mag, ang, gamma, theta, conv_w, conv_b, state_in, z_re, z_im,
                              state_out, ckpt, gate_mask, workspace, stream=None) -> int:
    return lib().cawn_phase_accumulate_fwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(gamma), _ptr(theta), _ptr(conv_w), _ptr(conv_b),
        _ptr(state_in), _ptr(z_re), _ptr(z_im), _ptr(state_out), _ptr(ckpt), _ptr(gate_mask),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0,
        _stream(stream))


def cawn_phase_accumulate_bwd(d, mag, ang, gamma, theta, conv_w, conv_b, state_in, ckpt, dz_re,
                              dz_im, dstate_out, dmag, dang, dgamma, dtheta, dconv_w, dconv_b,
                              dstate_in, workspace, stream=None) -> int:
    return lib().cawn_phase_accumulate_bwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(gamma), _ptr(theta), _ptr(conv_w), _ptr(conv_b),
        _ptr(state_in), _ptr(ckpt), _ptr(dz_re), _ptr(dz_im), _ptr(dstate_out), _ptr(dmag),
        _ptr(dang), _ptr(dgamma), _ptr(dtheta), _ptr(dconv_w), _ptr(dconv_b), _ptr(dstate_in),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0,
        _stream(stream))


def cawn_phase_accumulate_valve_fwd(d, mag, ang, valve, gamma, theta, conv_w, conv_b, state_in, z_re,
                                    z_im, state_out, ckpt, gate_mask, workspace, stream=None) -> int:
    return lib().cawn_phase_accumulate_valve_fwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(gamma), _ptr(theta), _ptr(conv_w),
        _ptr(conv_b), _ptr(state_in), _ptr(z_re), _ptr(z_im), _ptr(state_out), _ptr(ckpt),
        _ptr(gate_mask), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(stream))


def cawn_phase_accumulate_valve_bwd(d, mag, ang, valve, gamma, theta, conv_w, conv_b, state_in, ckpt,
                                    dz_re, dz_im, dstate_out, dmag, dang, dvalve, dgamma, dtheta,
                                    dconv_w, dconv_b, dstate_in, workspace, stream=None) -> int:
    return lib().cawn_phase_accumulate_valve_bwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(gamma), _ptr(theta), _ptr(conv_w),
        _ptr(conv_b), _ptr(state_in), _ptr(ckpt), _ptr(dz_re), _ptr(dz_im), _ptr(dstate_out),
        _ptr(dmag), _ptr(dang), _ptr(dvalve), _ptr(dgamma), _ptr(dtheta), _ptr(dconv_w),
        _ptr(dconv_b), _ptr(dstate_in), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(stream))


def cawn_phase_accumulate_ret_fwd(d, mag, ang, valve, ret, ret_bias, theta, conv_w, conv_b, state_in, z_re,
                                  z_im, state_out, ckpt, gate_mask, workspace, stream=None) -> int:
    return lib().cawn_phase_accumulate_ret_fwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(ret), _ptr(ret_bias), _ptr(theta), _ptr(conv_w),
        _ptr(conv_b), _ptr(state_in), _ptr(z_re), _ptr(z_im), _ptr(state_out), _ptr(ckpt),
        _ptr(gate_mask), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(stream))


def cawn_phase_accumulate_ret_bwd(d, mag, ang, valve, ret, ret_bias, theta, conv_w, conv_b, state_in, ckpt,
                                  dz_re, dz_im, dstate_out, dmag, dang, dvalve, dret, dtheta, dconv_w,
                                  dconv_b, dstate_in, workspace, stream=None) -> int:
    return lib().cawn_phase_accumulate_ret_bwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(ret), _ptr(ret_bias), _ptr(theta), _ptr(conv_w),
        _ptr(conv_b), _ptr(state_in), _ptr(ckpt), _ptr(dz_re), _ptr(dz_im), _ptr(dstate_out),
        _ptr(dmag), _ptr(dang), _ptr(dvalve), _ptr(dret), _ptr(dtheta), _ptr(dconv_w),
        _ptr(dconv_b), _ptr(dstate_in), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(stream))


def cawn_phase_accumulate_bf16_fwd(d, mag, ang, valve, ret, ret_bias, gamma, theta, conv_w, conv_b, state_in,
                                   z_re, z_im, state_out, ckpt, gate_mask, workspace, stream=None) -> int:
    """mag, ang, z_re, z_im: torch.bfloat16 tensors."""
    return lib().cawn_phase_accumulate_bf16_fwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(ret), _ptr(ret_bias), _ptr(gamma), _ptr(theta),
        _ptr(conv_w), _ptr(conv_b), _ptr(state_in), _ptr(z_re), _ptr(z_im), _ptr(state_out), _ptr(ckpt),
        _ptr(gate_mask), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(stream))


def cawn_phase_accumulate_hconv_fwd(d, mag, ang, valve, ret, ret_bias, gamma, theta, conv_w, conv_b, hconv_w,
                                    hconv_b, state_in, zc_re, zc_im, state_out, ckpt, gate_mask, workspace,
                                    activations_bf16=0, stream=None) -> int:
    """mag, ang, zc_re, zc_im: fp32 tensors, or torch.bfloat16 with activations_bf16=1."""
    return lib().cawn_phase_accumulate_hconv_fwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(ret), _ptr(ret_bias), _ptr(gamma), _ptr(theta),
        _ptr(conv_w), _ptr(conv_b), _ptr(hconv_w), _ptr(hconv_b), _ptr(state_in), _ptr(zc_re), _ptr(zc_im),
        _ptr(state_out), _ptr(ckpt), _ptr(gate_mask), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0,
        C.c_int32(activations_bf16), _stream(stream))


def cawn_phase_accumulate_hconv_bwd(d, mag, ang, valve, ret, ret_bias, gamma, theta, conv_w, conv_b, hconv_w, hconv_b,
                                    state_in, ckpt, dc_re, dc_im, dstate_out, dmag, dang, dvalve, dret, dgamma, dtheta,
                                    dconv_w, dconv_b, dhconv_w, dhconv_b, dstate_in, workspace, activations_bf16=0,
                                    stream=None) -> int:
    """dc_re, dc_im: gradients of the convolved output; dhconv_w [2,H,3], dhconv_b [2,H] beside the usual gradients.
    mag, ang, dc_re, dc_im, dmag, dang: fp32 tensors, or torch.bfloat16 with activations_bf16=1."""
    return lib().cawn_phase_accumulate_hconv_bwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(ret), _ptr(ret_bias), _ptr(gamma), _ptr(theta), _ptr(conv_w),
        _ptr(conv_b), _ptr(hconv_w), _ptr(hconv_b), _ptr(state_in), _ptr(ckpt), _ptr(dc_re), _ptr(dc_im), _ptr(dstate_out),
        _ptr(dmag), _ptr(dang), _ptr(dvalve), _ptr(dret), _ptr(dgamma), _ptr(dtheta), _ptr(dconv_w), _ptr(dconv_b),
        _ptr(dhconv_w), _ptr(dhconv_b), _ptr(dstate_in),
        _ptr(workspace), workspace.numel() * workspace.element_size() if workspace is not None else 0,
        C.c_int32(activations_bf16), _stream(stream))


def cawn_phase_accumulate_bf16_bwd(d, mag, ang, valve, ret, ret_bias, gamma, theta, conv_w, conv_b, state_in, ckpt,
                                   dz_re, dz_im, dstate_out, dmag, dang, dvalve, dret, dgamma, dtheta, dconv_w,
                                   dconv_b, dstate_in, workspace, stream=None) -> int:
    """mag, ang, dz_re, dz_im, dmag, dang: torch.bfloat16 tensors."""
    return lib().cawn_phase_accumulate_bf16_bwd(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(valve), _ptr(ret), _ptr(ret_bias), _ptr(gamma), _ptr(theta),
        _ptr(conv_w), _ptr(conv_b), _ptr(state_in), _ptr(ckpt), _ptr(dz_re), _ptr(dz_im), _ptr(dstate_out),
        _ptr(dmag), _ptr(dang), _ptr(dvalve), _ptr(dret), _ptr(dgamma), _ptr(dtheta), _ptr(dconv_w),
        _ptr(dconv_b), _ptr(dstate_in), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(stream))


def cawn_phase_accumulate_fwd_static(d, mag, ang, gamma, theta, conv_w, conv_b, state_in, z_re, z_im,
                                     state_out, ckpt, gate_mask, stream=None) -> int:
    """cawn_phase_accumulate_fwd on the library's static scratch array: allocates nothing."""
    return lib().cawn_phase_accumulate_fwd_static(
        C.byref(d), _ptr(mag), _ptr(ang), _ptr(gamma), _ptr(theta), _ptr(conv_w), _ptr(conv_b),
        _ptr(state_in), _ptr(z_re), _ptr(z_im), _ptr(state_out), _ptr(ckpt), _ptr(gate_mask), _stream(stream))


def cawn_stream_copy(in0, in1, out0, out1, stream=None) -> int:
    """Plain copy of two fp32 streams (the bandwidth ceiling the scan kernels are read against)."""
    return lib().cawn_stream_copy(_ptr(in0), _ptr(in1), _ptr(out0), _ptr(out1), in0.numel(), _stream(stream))


def alloc_workspace(d: cawn_desc, device="cuda:0") -> torch.Tensor:
    """Allocate (torch caching allocator, 256-byte aligned) and initialise a workspace for `d`."""
    n = cawn_workspace_bytes(d)
    ws = torch.empty((n + 3) // 4, dtype=torch.int32, device=device)
    check(cawn_workspace_init(ws))
    return ws
