"""Writes tests/golden/cfg1_oracle_samples.txt: sampled fp64 oracle outputs for the tiny
configuration (B=1, H=2, F=16, L=256, seed 4250).  Calls only oracle/ and the seeded input module.

The paper prints no worked numeric example for this path (no table or figure gives values of the
phase state), so there is nothing of the paper's to store here; this file is a regression anchor for
the oracle itself: a later change to its arithmetic must either leave these values or say why not.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import cawn_oracle as O                      # noqa: E402
from paper_2604_04250_amd import workloads as WL         # noqa: E402


def samples():
    wl = WL.CONFIGS["cfg1_tiny"]
    d = WL.make_inputs(wl)
    cfg = O.Cfg(wl.B, wl.L, wl.H, wl.F, conv_k=wl.conv_k, gate_tau=wl.gate_tau)
    f = O.phase_fwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], conv_w=d["conv_w"], conv_b=d["conv_b"])
    g = O.phase_bwd(cfg, d["mag"], d["ang"], d["gamma"], d["theta"], d["dz_re"], d["dz_im"],
                    conv_w=d["conv_w"], conv_b=d["conv_b"])
    rows = []
    for t, j in ((0, 0), (1, 5), (17, 31), (63, 16), (64, 16), (128, 7), (255, 0), (255, 31)):
        rows.append(("z_re", t, j, f["z_re"][0, t, j]))
        rows.append(("z_im", t, j, f["z_im"][0, t, j]))
        rows.append(("dmag", t, j, g["dmag"][0, t, j]))
        rows.append(("dang", t, j, g["dang"][0, t, j]))
    for j in (0, 13, 31):
        rows.append(("dgamma", -1, j, g["dgamma"][j]))
        rows.append(("dtheta", -1, j, g["dtheta"][j]))
        rows.append(("scan_re", -1, j, f["scan_out"][0, 0, j]))
    rows.append(("gate_open_count", -1, -1, float(f["gate"].sum())))
    return rows


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle_samples.txt")
    with open(out, "w") as fh:
        fh.write("# name t j value   (fp64 oracle, cfg1_tiny, seed 4250; written by make_golden.py)\n")
        for name, t, j, v in samples():
            fh.write(f"{name} {t} {j} {float(v)!r}\n")
    print(out)
