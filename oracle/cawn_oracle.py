"""ctypes front for the fp64 CPU oracle (oracle/cawn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing on the GPU product path imports this module, and this module
imports nothing of the GPU package.

Array conventions (numpy, C-contiguous):
  mag, ang          float32 [B, L, J]       J = H*F, lane j = h*F + k fastest
  gamma, theta      float32 [J]             (gamma may be None with ret_mode 1)
  valve, ret        float32 [B, L, H]       per-head logits (gate_mode 1 / ret_mode 1)
  ret_bias          float32 [F]             static per-harmonic retention bias b_k
  conv_w            float32 [2, J, Kc]      stream 0 = magnitude, 1 = angle
  conv_b            float32 [2, J] or None
  scan state        float64 [B, 2, J]       (re, im) of S at the last token, unclamped
  conv tail         float32 [B, Kc-1, 2, J] last Kc-1 pre-conv rows, oldest first
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cawn_oracle.c")
_LIB = os.path.join(_HERE, "libcawn_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent lanes)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("B", C.c_int32), ("L", C.c_int32), ("H", C.c_int32), ("F", C.c_int32),
                ("conv_k", C.c_int32), ("amp_mode", C.c_int32), ("clamp_feedback", C.c_int32),
                ("nthreads", C.c_int32), ("gate_mode", C.c_int32), ("gate_tau", C.c_float),
                ("valve_eps", C.c_float), ("ret_mode", C.c_int32), ("dz_f64", C.c_int32),
                ("conv_clamp", C.c_double), ("out_clamp", C.c_double), ("grad_clamp", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_max_threads.restype = C.c_int
    return _lib


def max_threads() -> int:
    return int(lib().oracle_max_threads())


@dataclass
class Cfg:
    B: int
    L: int
    H: int
    F: int
    conv_k: int = 0
    amp_mode: int = 0
    gate_tau: float = 0.0
    conv_clamp: float = 50.0
    out_clamp: float = 100.0
    grad_clamp: float = 100.0
    clamp_feedback: int = 0
    nthreads: int = 0
    gate_mode: int = 0          # 1: per-head valve (valve logits [B, L, H]), Sec. 3.3
    valve_eps: float = 0.001
    ret_mode: int = 0           # 1: retention sigmoid(ret[B,L,H] + ret_bias[F]), Sec. 3.3 item 4
    dz_f64: int = 0             # phase_bwd: dz_re / dz_im are taken as fp64 (e.g. from harmonic_conv_bwd)

    @property
    def J(self) -> int:
        return self.H * self.F

    def c(self) -> _Cfg:
        return _Cfg(self.B, self.L, self.H, self.F, self.conv_k, self.amp_mode, self.clamp_feedback,
                    self.nthreads, self.gate_mode, np.float32(self.gate_tau),
                    np.float32(self.valve_eps), self.ret_mode, self.dz_f64, self.conv_clamp, self.out_clamp, self.grad_clamp)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a, shape):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _f64(a, shape):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float64)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


def theta_init(H: int, F: int) -> np.ndarray:
    """Rotation angles as the paper initialises them (Sec. 3.4): theta_j = 10000^(-2j/(H*F))
    over the flat lane index j in [0, H*F-1], rounded once to fp32."""
    J = H * F
    j = np.arange(J, dtype=np.float64)
    return np.power(10000.0, -2.0 * j / J).astype(np.float32)


def syntax_conv(x, w, bias=None, hist_in=None, conv_clamp=50.0, want_hist=True):
    """Stand-alone Temporal Syntax Cache (Sec. 3.2).  x [B,L,C] f32, w [C,Kc] -> y f64, hist f32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, L, Cc = x.shape
    w = np.ascontiguousarray(w, dtype=np.float32)
    Kc = w.shape[1]
    assert w.shape == (Cc, Kc)
    bias = _f32(bias, (Cc,))
    hist_in = _f32(hist_in, (B, Kc - 1, Cc))
    y = np.empty((B, L, Cc), dtype=np.float64)
    hist = np.empty((B, Kc - 1, Cc), dtype=np.float32) if want_hist else None
    rc = lib().oracle_syntax_conv(C.c_int(B), C.c_int(L), C.c_int(Cc), C.c_int(Kc),
                                  C.c_double(conv_clamp), _p(x), _p(w), _p(bias), _p(hist_in), _p(y),
                                  _p(hist))
    assert rc == 0, rc
    return y, hist


def harmonic_conv(z_re, z_im, H: int, F: int, w, bias=None):
    """Depth-wise harmonic convolution (Sec. 3.6): z_re, z_im [B,L,H*F] f64, w [2,H,Kh], bias [2,H]
    -> (o_re, o_im) f64.  Channel = (plane, head), positions = the head's harmonics, zero padding
    on both sides, tap i multiplies position k + i - (Kh-1)/2."""
    z_re = np.ascontiguousarray(z_re, dtype=np.float64)
    z_im = np.ascontiguousarray(z_im, dtype=np.float64)
    B, L, J = z_re.shape
    assert J == H * F and z_im.shape == z_re.shape
    w = np.ascontiguousarray(w, dtype=np.float32)
    Kh = w.shape[2]
    assert w.shape == (2, H, Kh)
    bias = _f32(bias, (2, H))
    o_re = np.empty_like(z_re)
    o_im = np.empty_like(z_im)
    rc = lib().oracle_harmonic_conv(C.c_int(B), C.c_int(L), C.c_int(H), C.c_int(F), C.c_int(Kh),
                                    _p(z_re), _p(z_im), _p(w), _p(bias), _p(o_re), _p(o_im))
    assert rc == 0, rc
    return o_re, o_im


def harmonic_conv_bwd(z_re, z_im, H: int, F: int, w, do_re, do_im):
    """Adjoint of harmonic_conv (Sec. 3.6): z_re, z_im [B,L,H*F] (what the forward convolved), w [2,H,Kh],
    do_re, do_im [B,L,H*F] (upstream of the convolution's output) -> dict(dz_re, dz_im [B,L,H*F],
    dw [2,H,Kh], dbias [2,H]) in f64."""
    z_re = np.ascontiguousarray(z_re, dtype=np.float64)
    z_im = np.ascontiguousarray(z_im, dtype=np.float64)
    B, L, J = z_re.shape
    assert J == H * F and z_im.shape == z_re.shape
    w = np.ascontiguousarray(w, dtype=np.float32)
    Kh = w.shape[2]
    assert w.shape == (2, H, Kh)
    do_re = _f64(do_re, (B, L, J))
    do_im = _f64(do_im, (B, L, J))
    out = dict(dz_re=np.empty((B, L, J)), dz_im=np.empty((B, L, J)), dw=np.empty((2, H, Kh)), dbias=np.empty((2, H)))
    rc = lib().oracle_harmonic_conv_bwd(C.c_int(B), C.c_int(L), C.c_int(H), C.c_int(F), C.c_int(Kh), _p(z_re), _p(z_im),
                                        _p(w), _p(do_re), _p(do_im), _p(out["dz_re"]), _p(out["dz_im"]), _p(out["dw"]),
                                        _p(out["dbias"]))
    assert rc == 0, rc
    return out


def _ret_args(cfg: Cfg, ret, ret_bias):
    if cfg.ret_mode != 1:
        return None, None
    return _f32(ret, (cfg.B, cfg.L, cfg.H)), _f32(ret_bias, (cfg.F,))


def phase_fwd(cfg: Cfg, mag, ang, gamma, theta, conv_w=None, conv_b=None, scan_in=None,
              tail_in=None, want_gate=True, valve=None, ret=None, ret_bias=None):
    """Forward.  Returns dict(z_re, z_im [B,L,J] f64, scan_out [B,2,J] f64,
    tail_out [B,Kc-1,2,J] f32 or None, gate [B,L,J] uint8)."""
    B, L, J, Kc = cfg.B, cfg.L, cfg.J, cfg.conv_k
    mag = _f32(mag, (B, L, J))
    ang = _f32(ang, (B, L, J))
    gamma = _f32(gamma, (J,))
    theta = _f32(theta, (J,))
    ret, ret_bias = _ret_args(cfg, ret, ret_bias)
    if Kc > 0:
        conv_w = _f32(conv_w, (2, J, Kc))
        conv_b = _f32(conv_b, (2, J))
        tail_in = _f32(tail_in, (B, Kc - 1, 2, J))
    else:
        conv_w = conv_b = tail_in = None
    scan_in = _f64(scan_in, (B, 2, J))
    z_re = np.empty((B, L, J), dtype=np.float64)
    z_im = np.empty((B, L, J), dtype=np.float64)
    scan_out = np.empty((B, 2, J), dtype=np.float64)
    tail_out = np.empty((B, Kc - 1, 2, J), dtype=np.float32) if Kc > 1 else None
    gate = np.empty((B, L, J), dtype=np.uint8) if want_gate else None
    valve = _f32(valve, (B, L, cfg.H)) if cfg.gate_mode == 1 else None
    cc = cfg.c()
    rc = lib().oracle_phase_fwd(C.byref(cc), _p(mag), _p(ang), _p(valve), _p(ret), _p(ret_bias), _p(gamma), _p(theta), _p(conv_w),
                                _p(conv_b), _p(scan_in), _p(tail_in), _p(z_re), _p(z_im),
                                _p(scan_out), _p(tail_out), _p(gate))
    assert rc == 0, rc
    return dict(z_re=z_re, z_im=z_im, scan_out=scan_out, tail_out=tail_out, gate=gate)


def phase_bwd(cfg: Cfg, mag, ang, gamma, theta, dz_re, dz_im, conv_w=None, conv_b=None,
              scan_in=None, tail_in=None, dscan_out=None, dtail_out=None, valve=None, ret=None,
              ret_bias=None):
    """Backward.  Returns dict(dmag, dang [B,L,J], dgamma, dtheta [J], dconv_w [2,J,Kc],
    dconv_b [2,J], dscan_in [B,2,J], dtail_in [B,Kc-1,2,J]; gate_mode 1: dvalve [B,L,H];
    ret_mode 1: dret [B,L,H] and no dgamma) in f64."""
    B, L, J, Kc = cfg.B, cfg.L, cfg.J, cfg.conv_k
    mag = _f32(mag, (B, L, J))
    ang = _f32(ang, (B, L, J))
    gamma = _f32(gamma, (J,))
    theta = _f32(theta, (J,))
    dz_re = (_f64 if cfg.dz_f64 else _f32)(dz_re, (B, L, J))
    dz_im = (_f64 if cfg.dz_f64 else _f32)(dz_im, (B, L, J))
    if Kc > 0:
        conv_w = _f32(conv_w, (2, J, Kc))
        conv_b = _f32(conv_b, (2, J))
        tail_in = _f32(tail_in, (B, Kc - 1, 2, J))
        dtail_out = _f64(dtail_out, (B, Kc - 1, 2, J))
    else:
        conv_w = conv_b = tail_in = dtail_out = None
    scan_in = _f64(scan_in, (B, 2, J))
    dscan_out = _f64(dscan_out, (B, 2, J))
    out = dict(dmag=np.zeros((B, L, J)), dang=np.zeros((B, L, J)), dgamma=np.zeros(J),
               dtheta=np.zeros(J), dscan_in=np.zeros((B, 2, J)))
    if Kc > 0:
        out.update(dconv_w=np.zeros((2, J, Kc)), dconv_b=np.zeros((2, J)),
                   dtail_in=np.zeros((B, max(Kc - 1, 0), 2, J)))
    term = None
    if cfg.gate_mode == 1:
        valve = _f32(valve, (B, L, cfg.H))
        out["dvalve"] = np.zeros((B, L, cfg.H))
        term = np.zeros((B, L, J))
    else:
        valve = None
    ret, ret_bias = _ret_args(cfg, ret, ret_bias)
    rterm = None
    if cfg.ret_mode == 1:
        out["dret"] = np.zeros((B, L, cfg.H))
        rterm = np.zeros((B, L, J))
        del out["dgamma"]
    cc = cfg.c()
    rc = lib().oracle_phase_bwd(C.byref(cc), _p(mag), _p(ang), _p(valve), _p(ret), _p(ret_bias), _p(gamma), _p(theta), _p(conv_w),
                                _p(conv_b), _p(scan_in), _p(tail_in), _p(dz_re), _p(dz_im),
                                _p(dscan_out), _p(dtail_out), _p(out["dmag"]), _p(out["dang"]),
                                _p(out.get("dgamma")), _p(out["dtheta"]), _p(out.get("dconv_w")),
                                _p(out.get("dconv_b")), _p(out["dscan_in"]), _p(out.get("dtail_in")),
                                _p(out.get("dvalve")), _p(term), _p(out.get("dret")), _p(rterm))
    assert rc == 0, rc
    return out
