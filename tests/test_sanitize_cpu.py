"""Sanitizer builds of the CPU-side code (host compilers only, no GPU): the fp64 oracle and the host part of
the library's gates are compiled with -fsanitize=address,undefined and run on small ragged cases of every
mode.  The oracle's sanitized results are compared with what the ordinary build of the oracle (the one every
pin in test_oracle_pins.py runs against) returns on the same inputs, so a memory error that happens to leave
plausible numbers behind fails here even where the pins pass."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import cawn_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _records(path):
    """Parse the dump written by tests/sanitize/oracle_san.c: a sequence of (header fields, {name: array})."""
    ty = {"f4": np.float32, "f8": np.float64, "u1": np.uint8}
    out = []
    with open(path, "rb") as f:
        while True:
            head = f.readline()
            if not head:
                break
            head = head.decode().split()
            arrs = {}
            while True:
                line = f.readline().decode().split()
                if line[0] == "end":
                    break
                assert line[0] == "arr", line
                dt = np.dtype(ty[line[2]])
                n = int(line[3])
                arrs[line[1]] = np.frombuffer(f.read(n * dt.itemsize), dtype=dt).copy()
                assert f.read(1) == b"\n"
            out.append((head, arrs))
    return out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe, dump = str(tmp_path / "oracle_san"), str(tmp_path / "oracle_san.bin")
    subprocess.check_call(["gcc", *SAN, "-fopenmp", "-ffp-contract=off", os.path.join(HERE, "sanitize", "oracle_san.c"),
                           "-o", exe, "-lm"])
    r = subprocess.run([exe, dump], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    recs = _records(dump)
    assert len(recs) == 11
    n_case = 0
    for head, a in recs:
        if head[0] == "case":
            n_case += 1
            B, L, H, F, Kc, amp, gm, rm, dz64 = (int(v) for v in head[1:10])
            J = H * F
            cfg = O.Cfg(B, L, H, F, conv_k=Kc, amp_mode=amp, gate_tau=float(head[10]), gate_mode=gm, valve_eps=0.3,
                        ret_mode=rm, dz_f64=dz64, conv_clamp=50.0, out_clamp=2.0, grad_clamp=3.0, nthreads=2)
            sh = lambda k, *s: a[k].reshape(s)
            kw = dict(conv_w=sh("conv_w", 2, J, max(Kc, 1)) if Kc else None, conv_b=sh("conv_b", 2, J) if Kc else None,
                      scan_in=sh("scan_in", B, 2, J), tail_in=sh("tail_in", B, Kc - 1, 2, J) if Kc > 1 else None,
                      valve=sh("valve", B, L, H) if gm else None, ret=sh("ret", B, L, H) if rm else None,
                      ret_bias=a["ret_bias"] if rm else None)
            gam = None if rm else a["gamma"]
            f = O.phase_fwd(cfg, sh("mag", B, L, J), sh("ang", B, L, J), gam, a["theta"], **kw)
            for k in ("z_re", "z_im", "scan_out"):
                np.testing.assert_allclose(f[k].ravel(), a[k], rtol=1e-13, atol=1e-13, err_msg=f"{head} {k}")
            if Kc > 1:
                np.testing.assert_array_equal(f["tail_out"].ravel(), a["tail_out"])
            np.testing.assert_array_equal(f["gate"].ravel(), a["gate"])
            g = O.phase_bwd(cfg, sh("mag", B, L, J), sh("ang", B, L, J), gam, a["theta"], sh("dz_re", B, L, J),
                            sh("dz_im", B, L, J), dscan_out=sh("dscan_out", B, 2, J),
                            dtail_out=sh("dtail_out", B, Kc - 1, 2, J) if Kc > 1 else None, **kw)
            for k, v in g.items():
                np.testing.assert_allclose(v.ravel(), a[k], rtol=1e-12, atol=1e-12, err_msg=f"{head} {k}")
        elif head[0] == "conv":
            B, L, Cc, Kc = (int(v) for v in head[1:5])
            y, hist = O.syntax_conv(a["x"].reshape(B, L, Cc), a["w"].reshape(Cc, Kc), a["b"], a["hin"].reshape(B, Kc - 1, Cc))
            np.testing.assert_allclose(y.ravel(), a["y"], rtol=1e-13, atol=1e-13)
            np.testing.assert_array_equal(hist.ravel(), a["hout"])
        else:
            assert head[0] == "hconv"
            B, L, H, F, Kh = (int(v) for v in head[1:6])
            z = [a[k].reshape(B, L, H * F) for k in ("z_re", "z_im", "up_re", "up_im")]
            w, b = a["w"].reshape(2, H, Kh), a["b"].reshape(2, H)
            o = O.harmonic_conv(z[0], z[1], H, F, w, b)
            np.testing.assert_allclose(o[0].ravel(), a["o_re"], rtol=1e-13, atol=1e-13)
            np.testing.assert_allclose(o[1].ravel(), a["o_im"], rtol=1e-13, atol=1e-13)
            g = O.harmonic_conv_bwd(z[0], z[1], H, F, w, z[2], z[3])
            for k in ("dz_re", "dz_im", "dw", "dbias"):
                np.testing.assert_allclose(g[k].ravel(), a[k], rtol=1e-13, atol=1e-13, err_msg=k)
    assert n_case == 9


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_gate_bisection_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "gate_san")
    subprocess.check_call(["g++", "-std=c++17", *SAN, os.path.join(HERE, "sanitize", "gate_san.cpp"), "-o", exe])
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:] + r.stderr[-4000:]
    assert "gate sanitizer run: done" in r.stdout
