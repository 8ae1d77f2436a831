#!/usr/bin/env python3
"""Benchmark of the fused conv + phase-accumulation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--paper]

One "step" is one pass of the whole hot path over one batch of seeded synthetic input that is
already resident in HBM: forward (writing the checkpoints) followed by backward with every
gradient requested, on the training-step configuration (B=8, H=12, F=64, L=8192, fp32, conv
kernel 4, threshold 0.1).  Other workloads: cfg2_layer_fwd (forward only), cfg4_stream (2,000,000
tokens in 4096-token chunks with the state carried in place; --chunk 32768 for the paper's own chunk
length), cfg5_wide (forward + backward), cfg6_paper_heads, decode (one token per call, state in place:
eager launches and a replayed HIP graph).  --paper runs the layer as the paper states it (4 heads of
64 harmonics, conv kernel 3, softplus amplitude, per-head valve, data-dependent retention).

Prints ONE JSON line: tokens/s of the whole step, plus
  roofline      - algorithmic HBM bytes of the dominant kernel / its measured duration vs 8 TB/s;
  copy_ceiling  - what a plain 8 B in / 8 B out streaming copy (cawn_stream_copy) reaches in this
                  run, at the dominant kernel's byte count and at 50 / 100 MB;
  cpu_baseline  - the fp64 oracle timed on the host cores on a bounded sample of the same inputs;
  other_workloads (default run only) - the same measurements for cfg2_layer_fwd, cfg4_stream and
                  cfg5_wide, each with its roofline fraction and a sampled parity figure.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
FWD_BYTES_PER_TOKEN_LANE = 16   # read mag, ang; write z_re, z_im
BWD_BYTES_PER_TOKEN_LANE = 24   # read mag, ang, dz_re, dz_im; write dmag, dang


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 100; 3 for cfg4_stream)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps (default 20; 1 for cfg4_stream)")
    ap.add_argument("--preheat", type=float, default=0.3,
                    help="seconds of untimed steps in front of the warm-up (reported as preheat_s): the clocks "
                         "ramp up over tens of milliseconds of load, and a timed region of a few milliseconds "
                         "would otherwise depend on the number of warm-up steps")
    ap.add_argument("--valve", action="store_true",
                    help="gate_mode 1: the per-head input valve of Sec. 3.3 instead of the per-lane threshold "
                         "(extra line, not the headline; no CPU baseline)")
    ap.add_argument("--ret", action="store_true",
                    help="ret_mode 1: the data-dependent retention of Sec. 3.3 item 4 instead of the constant gamma "
                         "(extra line, not the headline; no CPU baseline)")
    ap.add_argument("--paper", action="store_true",
                    help="the layer as the paper states it: 4 heads of 64 harmonics (Sec. 4.3), conv kernel 3 "
                         "(Sec. 3.2), amplitude min(softplus, 10) (Sec. 3.3 item 1), per-head valve with eps = 0.001 "
                         "and data-dependent retention (Sec. 3.3), on the training-step batch B=8, L=8192 "
                         "(extra line, not the headline; no CPU baseline)")
    ap.add_argument("--bf16", action="store_true",
                    help="activations (inputs, outputs, upstream and returned gradients) are bfloat16 in memory, "
                         "arithmetic and state fp32 (extra line, not the headline; no CPU baseline)")
    ap.add_argument("--hconv", action="store_true",
                    help="the depth-wise harmonic convolution of Sec. 3.6 fused behind the output clamp: the forward "
                         "stores the convolved output, the backward takes its gradients and returns the taps' and "
                         "biases' gradients as well (same bytes per token-lane; fp32 or --bf16, alone or with --valve, --ret "
                         "or --paper; extra line, not the headline; no CPU baseline)")
    ap.add_argument("--unfused", action="store_true",
                    help="cfg2_layer_fwd only: the Temporal Syntax Cache as separate calls (cawn_syntax_conv on each "
                         "stream, then the scan without conv front-end): 32 instead of 16 bytes per token-lane; "
                         "a comparison line, not the headline")
    ap.add_argument("--workload", default="cfg3_train",
                    choices=["cfg2_layer_fwd", "cfg3_train", "cfg4_stream", "cfg5_wide", "cfg6_paper_heads", "decode"])
    ap.add_argument("--chunk", type=int, default=None, help="cfg4_stream: tokens per call (default 4096)")
    ap.add_argument("--decode-batch", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default run only: skip the cfg2 / cfg4 / cfg5 measurements that ride on the headline line")
    return ap.parse_args()


def read_traffic(workload):
    """HBM bytes per launch of the dominant kernel from a committed rocprofv3 --pmc summary (profiles/*_pmc.txt
    holds a line 'TRAFFIC_BYTES_PER_LAUNCH <workload> <bytes>'): (bytes, file) or (None, None).  This is a
    figure of an earlier profiling run of the same command, not a measurement of this run."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None, None
    for fn in sorted(os.listdir(pdir)):
        if not fn.endswith("_pmc.txt"):
            continue
        for line in open(os.path.join(pdir, fn)):
            p = line.split()
            if len(p) == 3 and p[0] == "TRAFFIC_BYTES_PER_LAUNCH" and p[1] == workload:
                return float(p[2]), "profiles/" + fn
    return None, None


def decode_bench(args, np, torch, K, WL, dev):
    """Autoregressive steps of the 150M-shaped layer: one token per call, state carried in place.
    Measured twice: plain launches, and 64 steps captured in a HIP graph and replayed."""
    wl = WL.CONFIGS["cfg2_layer_fwd"].with_(B=args.decode_batch, L=64)
    B, H, F, J, Kc = wl.B, wl.H, wl.F, wl.J, wl.conv_k
    theta = K.cawn_theta_init(H, F)
    inp = WL.make_inputs(wl, theta=theta, with_grads=False)
    t = lambda a: torch.from_numpy(a).to(dev)
    gamma, th, cw, cb = t(inp["gamma"]), t(inp["theta"]), t(inp["conv_w"]), t(inp["conv_b"])
    # one [B,1,J] slice per step at a fixed address (a graph replays fixed pointers)
    mag = [t(np.ascontiguousarray(inp["mag"][:, i:i + 1])) for i in range(wl.L)]
    ang = [t(np.ascontiguousarray(inp["ang"][:, i:i + 1])) for i in range(wl.L)]
    zr = [torch.empty((B, 1, J), device=dev) for _ in range(wl.L)]
    zi = [torch.empty((B, 1, J), device=dev) for _ in range(wl.L)]
    d = K.make_desc(B, 1, H, F, conv_k=Kc, gate_tau=wl.gate_tau)
    ws = K.alloc_workspace(d, dev)
    state = torch.zeros(K.cawn_state_bytes(d) // 4, device=dev)

    def steps():
        for i in range(wl.L):
            st = K.cawn_phase_accumulate_fwd(d, mag[i], ang[i], gamma, th, cw, cb, state, zr[i], zi[i], state,
                                             None, None, ws)
            assert st == 0, st

    steps()                      # builds the lane table
    d.lane_consts_cached = 1
    torch.cuda.synchronize()
    # eager
    state.zero_()
    for _ in range(args.warmup):
        steps()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        steps()
    torch.cuda.synchronize()
    eager_us = (time.perf_counter() - t0) * 1e6 / (args.steps * wl.L)
    # graph: capture on a side stream (default priority), replay
    state.zero_()
    steps()
    torch.cuda.synchronize()
    ref_state = state.clone()
    ref_z = zr[-1].clone()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    state.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        steps()
    state.zero_()
    g.replay()
    torch.cuda.synchronize()
    graph_ok = bool(torch.equal(state, ref_state) and torch.equal(zr[-1], ref_z))
    for _ in range(args.warmup):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.replay()
    torch.cuda.synchronize()
    graph_us = (time.perf_counter() - t0) * 1e6 / (args.steps * wl.L)
    K.check(K.cawn_workspace_status(ws))
    out = {"metric": "decode tokens/s (one token per call, state in place)", "value": B / (graph_us * 1e-6),
           "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": graph_us * wl.L * 1e-3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"decode: B={B} H={H} F={F} conv_k={Kc} tau={wl.gate_tau}, {wl.L} single-token "
                                  f"calls per step, state carried in place"},
           "us_per_token_eager": eager_us, "us_per_token_graph": graph_us, "graph_matches_eager": graph_ok,
           "state_bytes": int(state.numel() * 4)}
    print(json.dumps(out), flush=True)


class CopyCeiling:
    """cawn_stream_copy timed with HIP events on the launch stream, on buffer sets rotated so that the
    last-level cache cannot serve them.  Results are cached per byte count."""

    def __init__(self, np, torch, K, dev):
        self.np, self.torch, self.K, self.dev, self.cache = np, torch, K, dev, {}

    def gbps(self, nbytes, reps=30, heat_s=0.1):
        """nbytes = bytes read + bytes written by one launch (8 + 8 per element of each stream pair)."""
        torch, K = self.torch, self.K
        n = int(nbytes) // 16
        n -= n % 4
        if n <= 0:
            return None
        if n in self.cache:
            return self.cache[n]
        nset = max(2, int((600 << 20) // (16 * n)) + 1)
        bufs = [[torch.empty(n, device=self.dev).normal_() for _ in range(2)] +
                [torch.empty(n, device=self.dev) for _ in range(2)] for _ in range(nset)]
        call = lambda i: K.check(K.cawn_stream_copy(*bufs[i % nset]))
        t0 = time.perf_counter()
        i = 0
        while time.perf_counter() - t0 < heat_s:
            for _ in range(10):
                call(i)
                i += 1
            torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for r, (e0, e1) in enumerate(evs):
            e0.record()
            call(r)
            e1.record()
        torch.cuda.synchronize()
        ms = float(self.np.mean([a.elapsed_time(b) for a, b in evs]))
        assert bool(torch.equal(bufs[0][0], bufs[0][2])), "copy kernel"
        del bufs
        self.cache[n] = 16.0 * n / (ms * 1e-3) / 1e9
        return self.cache[n]


def lane_sample_parity(np, G, O, wl, inp, got, mode, Kc, amp_mode=0, valve=None, valve_eps=0.001, ret=None, ret_bias=None,
                       max_tokens=None, hconv=None):
    """Parity of the timed configuration itself on sampled lanes: the harmonics of head 0, every batch row,
    every token (lanes are independent, so the oracle runs on those lanes alone).  `got` holds the timed
    run's outputs (torch tensors).  Returns the worst relative error (rms-floored, as in the tests)."""
    B, L, H, F = wl.B, (wl.chunk or wl.L) if mode == "stream" else wl.L, wl.H, wl.F
    if max_tokens is not None:
        L = min(L, max_tokens)
    sl = slice(0, F)
    sub = lambda a: np.ascontiguousarray(a[:, :L, sl])
    cfg = O.Cfg(B, L, 1, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=wl.gate_tau, gate_mode=0 if valve is None else 1,
                valve_eps=valve_eps, ret_mode=0 if ret is None else 1, nthreads=O.max_threads())
    kw = dict(conv_w=np.ascontiguousarray(inp["conv_w"][:, sl]), conv_b=np.ascontiguousarray(inp["conv_b"][:, sl]))
    if valve is not None:
        kw["valve"] = np.ascontiguousarray(valve[:, :L, :1])
    if ret is not None:
        kw["ret"] = np.ascontiguousarray(ret[:, :L, :1])
        kw["ret_bias"] = ret_bias
    gam = None if ret is not None else inp["gamma"][sl]
    of = O.phase_fwd(cfg, sub(inp["mag"]), sub(inp["ang"]), gam, inp["theta"][sl], want_gate=False, **kw)
    host = lambda t: t[:, :L, sl].float().cpu().numpy()
    zo = (of["z_re"], of["z_im"])
    if hconv is not None:       # (hw [2,H,3], hb [2,H]): the stored planes are the convolved ones; head 0 stands alone
        hw0, hb0 = np.ascontiguousarray(hconv[0][:, :1]), np.ascontiguousarray(hconv[1][:, :1])
        zo = O.harmonic_conv(of["z_re"], of["z_im"], 1, F, hw0, hb0)
    err = {"z": max(G.rel_err(host(got["z_re"]), zo[0]), G.rel_err(host(got["z_im"]), zo[1]))}
    if "dmag" in got and L == wl.L:
        up_re, up_im = sub(inp["dz_re"]), sub(inp["dz_im"])
        bcfg = cfg
        if hconv is not None:   # the upstream gradients are those of the convolved planes
            gh = O.harmonic_conv_bwd(of["z_re"], of["z_im"], 1, F, hw0, up_re, up_im)
            up_re, up_im = gh["dz_re"], gh["dz_im"]
            bcfg = O.Cfg(B, L, 1, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=wl.gate_tau, gate_mode=0 if valve is None else 1,
                         valve_eps=valve_eps, ret_mode=0 if ret is None else 1, dz_f64=1, nthreads=O.max_threads())
            err["dhconv_w"] = G.rel_err(got["dhconv_w"][:, :1].cpu().numpy(), gh["dw"])
            err["dhconv_b"] = G.rel_err(got["dhconv_b"][:, :1].cpu().numpy(), gh["dbias"])
        ob = O.phase_bwd(bcfg, sub(inp["mag"]), sub(inp["ang"]), gam, inp["theta"][sl], up_re, up_im, **kw)
        err["dmag"] = G.rel_err(host(got["dmag"]), ob["dmag"])
        err["dang"] = G.rel_err(host(got["dang"]), ob["dang"])
        for k in ("dgamma", "dtheta"):
            if got.get(k) is not None and k in ob:
                err[k] = G.rel_err(got[k][sl].cpu().numpy(), ob[k])
        if got.get("dconv_w") is not None:
            err["dconv_w"] = G.rel_err(got["dconv_w"][:, sl].cpu().numpy(), ob["dconv_w"])
            err["dconv_b"] = G.rel_err(got["dconv_b"][:, sl].cpu().numpy(), ob["dconv_b"])
        if got.get("dvalve") is not None:
            err["dvalve"] = G.rel_err(got["dvalve"][:, :L, :1].cpu().numpy(), ob["dvalve"])
        if got.get("dret") is not None:
            err["dret"] = G.rel_err(got["dret"][:, :L, :1].cpu().numpy(), ob["dret"])
    return err


def run_workload(args, name, np, torch, K, WL, dev, ceiling, steps, warmup, headline):
    """Measure one workload; returns the result dictionary (the JSON line of a headline run, or the
    sub-result of another configuration riding on it)."""
    wl = WL.CONFIGS[name]
    paper = args.paper and headline
    valve_on, ret_on = (args.valve or paper) and headline, (args.ret or paper) and headline
    bf16, hconv, unfused = args.bf16 and headline, args.hconv and headline, args.unfused and headline
    amp_mode = 1 if paper else 0
    if paper:
        wl = WL.CONFIGS["cfg6_paper_heads"].with_(name="paper_layer", conv_k=3)
    if name == "cfg4_stream" and args.chunk:
        wl = wl.with_(chunk=args.chunk)
    B, H, F, J, Kc = wl.B, wl.H, wl.F, wl.J, wl.conv_k
    theta = K.cawn_theta_init(H, F)
    # (the training workloads run forward + backward in every mode; the others time the forward)
    do_bwd = name in ("cfg3_train", "cfg5_wide", "cfg6_paper_heads")
    stream_mode = name == "cfg4_stream"
    L = wl.chunk if stream_mode else wl.L
    valve_eps = 0.001

    # ---- inputs: the seeded host recipe for one batch (one chunk pool entry when streaming)
    inp = WL.make_inputs(wl, theta=theta, with_grads=do_bwd, L=L)
    gamma, th = torch.from_numpy(inp["gamma"]).to(dev), torch.from_numpy(inp["theta"]).to(dev)
    cw, cb = torch.from_numpy(inp["conv_w"]).to(dev), torch.from_numpy(inp["conv_b"]).to(dev)
    esize = 2 if bf16 else 4
    adt = torch.bfloat16 if bf16 else torch.float32
    per_set = (8 if do_bwd else 4) * B * L * J * esize
    # >= 4 disjoint sets, > 512 MiB in total: the LLC cannot serve them (one set of the wide configuration is 8.6 GB)
    nsets = 2 if per_set > (4 << 30) else max(4, min(16 if not bf16 else 32, -(-(600 << 20) // per_set)))
    names = ["mag", "ang"] + (["dz_re", "dz_im"] if do_bwd else [])
    sets = []
    base = {k: torch.from_numpy(inp[k]).to(dev).to(adt) for k in names}
    for s in range(nsets):
        cur = {k: (base[k] if s == 0 else torch.roll(base[k], shifts=7 * s, dims=1).contiguous()) for k in names}
        cur["z_re"] = torch.empty((B, L, J), device=dev, dtype=adt)
        cur["z_im"] = torch.empty((B, L, J), device=dev, dtype=adt)
        if do_bwd:
            cur["dmag"] = torch.empty((B, L, J), device=dev, dtype=adt)
            cur["dang"] = torch.empty((B, L, J), device=dev, dtype=adt)
        sets.append(cur)

    d = K.make_desc(B, L, H, F, conv_k=Kc, amp_mode=amp_mode, gate_tau=wl.gate_tau, gate_mode=1 if valve_on else 0,
                    ret_mode=1 if ret_on else 0, hconv_k=3 if hconv else 0, valve_eps=valve_eps)
    no_cpu = args.no_cpu_baseline or not headline
    hw = hb = None
    if hconv:
        assert not unfused, "--hconv: not with --unfused"
        no_cpu = True
        rh = np.random.Generator(np.random.PCG64(4250 + 97))
        hw = torch.from_numpy((rh.standard_normal((2, H, 3)) / np.sqrt(3.0)).astype(np.float32)).to(dev)
        hb = torch.from_numpy((0.1 * rh.standard_normal((2, H))).astype(np.float32)).to(dev)
        dhw, dhb = torch.empty((2, H, 3), device=dev), torch.empty((2, H), device=dev)
    if bf16:
        no_cpu = True
    ret = ret_bias = dret = ret_h = ret_bias_h = None
    if ret_on:
        assert not stream_mode, "--ret: cfg2_layer_fwd, cfg3_train, cfg5_wide or --paper"
        no_cpu = True
        # logits around the paper's initial projection bias -2, b_k falling from +3 to 0 over the harmonics
        rr = np.random.Generator(np.random.PCG64(4250 + 98))
        ret_h = (-2.0 + 1.5 * rr.standard_normal((B, L, H))).astype(np.float32)
        ret_bias_h = np.linspace(3.0, 0.0, F).astype(np.float32)
        ret, ret_bias = torch.from_numpy(ret_h).to(dev), torch.from_numpy(ret_bias_h).to(dev)
        dret = torch.empty((B, L, H), device=dev)
    valve = dvalve = valve_h = None
    if valve_on:
        assert not stream_mode, "--valve: cfg2_layer_fwd, cfg3_train, cfg5_wide or --paper"
        no_cpu = True
        # logits around the closing point 3 + ln(0.001/0.999) = -3.9: about half the valves are shut
        rv = np.random.Generator(np.random.PCG64(4250 + 99))
        valve_h = (-3.9 + 3.0 * rv.standard_normal((B, L, H))).astype(np.float32)
        valve = torch.from_numpy(valve_h).to(dev)
        dvalve = torch.empty((B, L, H), device=dev)
    ws = K.alloc_workspace(d, dev)
    ckpt = torch.empty(K.cawn_ckpt_bytes(d) // 4, device=dev) if do_bwd else None
    dgamma, dtheta = torch.empty(J, device=dev), torch.empty(J, device=dev)
    dcw, dcb = torch.empty((2, J, max(Kc, 1)), device=dev), torch.empty((2, J), device=dev)
    nstate = K.cawn_state_bytes(d) // 4
    state = torch.zeros(nstate, device=dev)

    # first call builds the lane table; later calls reuse it (parameters do not change in the bench)
    if unfused:
        assert name == "cfg2_layer_fwd" and not (bf16 or valve_on or ret_on), "--unfused: plain cfg2_layer_fwd"
        no_cpu = True
        d_plain = K.make_desc(B, L, H, F, conv_k=0, gate_tau=wl.gate_tau)
        xm, xa = torch.empty((B, L, J), device=dev), torch.empty((B, L, J), device=dev)
        cwm, cwa = cw[0].contiguous(), cw[1].contiguous()
        cbm, cba = cb[0].contiguous(), cb[1].contiguous()

    def fwd_call(dd, p, st_in, st_out, ck, mask=None):
        if unfused:
            st = K.cawn_syntax_conv(d, J, p["mag"], cwm, cbm, None, xm, None)
            st |= K.cawn_syntax_conv(d, J, p["ang"], cwa, cba, None, xa, None)
            return st | K.cawn_phase_accumulate_fwd(d_plain, xm, xa, gamma, th, None, None, st_in, p["z_re"], p["z_im"],
                                                    st_out, ck, mask, ws)
        if hconv:
            return K.cawn_phase_accumulate_hconv_fwd(dd, p["mag"], p["ang"], valve, ret, ret_bias, gamma, th, cw, cb,
                                                     hw, hb, st_in, p["z_re"], p["z_im"], st_out, ck, mask, ws,
                                                     activations_bf16=1 if bf16 else 0)
        if bf16:
            return K.cawn_phase_accumulate_bf16_fwd(dd, p["mag"], p["ang"], valve, ret, ret_bias, gamma, th, cw, cb,
                                                    st_in, p["z_re"], p["z_im"], st_out, ck, mask, ws)
        if ret is not None:
            return K.cawn_phase_accumulate_ret_fwd(dd, p["mag"], p["ang"], valve, ret, ret_bias, th, cw, cb, st_in,
                                                   p["z_re"], p["z_im"], st_out, ck, mask, ws)
        if valve is not None:
            return K.cawn_phase_accumulate_valve_fwd(dd, p["mag"], p["ang"], valve, gamma, th, cw, cb, st_in,
                                                     p["z_re"], p["z_im"], st_out, ck, mask, ws)
        return K.cawn_phase_accumulate_fwd(dd, p["mag"], p["ang"], gamma, th, cw, cb, st_in, p["z_re"], p["z_im"],
                                           st_out, ck, mask, ws)

    K.check(fwd_call(d, sets[0], None, None, ckpt))
    # A training step follows an optimizer update: its forward rebuilds the lane constants from the parameters, its
    # backward reuses them.  Inference calls (forward-only workloads, streaming chunks) keep them: parameters fixed.
    d_train = type(d).from_buffer_copy(d)
    d_train.lane_consts_cached = 0
    d.lane_consts_cached = 1
    if unfused:
        d_plain.lane_consts_cached = 1
    d_tail = None
    if stream_mode:
        nfull, rem = divmod(wl.L, wl.chunk)
        d_tail = K.make_desc(B, rem, H, F, conv_k=Kc, gate_tau=wl.gate_tau, lane_consts_cached=1,
                             hconv_k=3 if hconv else 0) if rem else None

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(i, rec=None):
        s = sets[i % nsets]
        if stream_mode:
            state.zero_()
            for c in range(nfull):
                p = sets[c % nsets]
                fwd_call(d, p, state, state, None)
            if d_tail is not None:
                p = sets[nfull % nsets]
                fwd_call(d_tail, p, state, state, None)
            return
        if rec is not None:
            rec[0].record()
        st = fwd_call(d_train if do_bwd and not unfused else d, s, None, None, ckpt)
        if rec is not None:
            rec[1].record()
        if do_bwd:
            if hconv:
                st |= K.cawn_phase_accumulate_hconv_bwd(d, s["mag"], s["ang"], valve, ret, ret_bias, gamma, th, cw, cb, hw,
                                                        hb, None, ckpt, s["dz_re"], s["dz_im"], None, s["dmag"], s["dang"],
                                                        dvalve, dret, None if ret is not None else dgamma, dtheta, dcw, dcb,
                                                        dhw, dhb, None, ws, activations_bf16=1 if bf16 else 0)
            elif bf16:
                st |= K.cawn_phase_accumulate_bf16_bwd(d, s["mag"], s["ang"], valve, ret, ret_bias, gamma, th, cw, cb,
                                                       None, ckpt, s["dz_re"], s["dz_im"], None, s["dmag"], s["dang"],
                                                       dvalve, dret, None if ret is not None else dgamma, dtheta,
                                                       dcw, dcb, None, ws)
            elif ret is not None:
                st |= K.cawn_phase_accumulate_ret_bwd(d, s["mag"], s["ang"], valve, ret, ret_bias, th, cw, cb, None,
                                                      ckpt, s["dz_re"], s["dz_im"], None, s["dmag"], s["dang"],
                                                      dvalve, dret, dtheta, dcw, dcb, None, ws)
            elif valve is not None:
                st |= K.cawn_phase_accumulate_valve_bwd(d, s["mag"], s["ang"], valve, gamma, th, cw, cb, None, ckpt,
                                                        s["dz_re"], s["dz_im"], None, s["dmag"], s["dang"], dvalve,
                                                        dgamma, dtheta, dcw, dcb, None, ws)
            else:
                st |= K.cawn_phase_accumulate_bwd(d, s["mag"], s["ang"], gamma, th, cw, cb, None, ckpt, s["dz_re"],
                                                  s["dz_im"], None, s["dmag"], s["dang"], dgamma, dtheta, dcw, dcb,
                                                  None, ws)
            if rec is not None:
                rec[2].record()
        assert st == 0, st

    # ---- pre-heat (fixed duration), warm-up (W steps), then exactly K timed steps
    t_heat = time.perf_counter()
    i = 0
    while args.preheat > 0 and time.perf_counter() - t_heat < args.preheat:
        for _ in range(1 if stream_mode else 10):
            step(i)
            i += 1
        torch.cuda.synchronize()
    preheat_s = time.perf_counter() - t_heat if args.preheat > 0 else 0.0
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    mem0 = torch.cuda.memory_allocated()
    recs = [(ev(), ev(), ev()) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, recs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    mem1 = torch.cuda.memory_allocated()
    K.check(K.cawn_workspace_status(ws))
    ms_per_step = wall * 1e3 / steps
    tokens = wl.B * wl.L
    value = tokens / (ms_per_step * 1e-3)

    dtype = "bf16 activations, f32 arithmetic and state" if bf16 else "f32"
    out = {"metric": "phase-accumulation tokens/s (fwd+bwd)" if do_bwd else "phase-accumulation tokens/s (fwd)",
           "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "preheat_s": round(preheat_s, 3), "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": dtype, "data": "synthetic",
           "config": {"workload": f"{wl.name}: B={wl.B} H={H} F={F} L={wl.L} conv_k={Kc} tau={wl.gate_tau} "
                                  f"gamma~U[{wl.gamma_lo},{wl.gamma_hi}] theta_j=10000^(-2j/J)"
                                  + (f" chunk={wl.chunk} state carried in place" if stream_mode else ""),
                      "pass": "fwd+bwd (all gradients)" if do_bwd else "fwd",
                      "gate": f"per-head valve (gate_mode 1, eps {valve_eps}), about half shut" if valve_on else "per-lane threshold",
                      "retention": "sigmoid(logit[t][h] + b_k) (ret_mode 1), logits ~ N(-2, 1.5^2), b_k from +3 to 0"
                                   if ret_on else "constant per lane",
                      "amplitude": "min(softplus(x), 10) (amp_mode 1)" if amp_mode else "the magnitude stream itself (amp_mode 0)",
                      "lane_constants": "rebuilt from the parameters in every step's forward" if do_bwd and not unfused
                                        else "built once (inference: parameters fixed)",
                      "buffer_sets_rotated": nsets}}
    bflag = lambda x: "true" if x else "false"
    fwd_label = f"fwd_kernel<1,{Kc},{bflag(valve_on)},{bflag(ret_on)},{bflag(bf16)},{bflag(hconv)}>"
    bwd_label = f"bwd_kernel<1,{Kc},true,{bflag(valve_on)},{bflag(ret_on)},{bflag(bf16)},{bflag(hconv)}>"
    extra = valve_on or ret_on or bf16 or unfused or hconv
    if paper:
        out["config"]["layer"] = ("the paper's statement of the layer: H=4, K=64 (Sec. 4.3), conv kernel 3 (Sec. 3.2), "
                                  "softplus amplitude, per-head valve, data-dependent retention (Sec. 3.3)")
    if unfused:
        fwd_label = "2 x syntax_conv_kernel<4> + fwd_kernel<1,0,false,false,false,false> (one event span; the path's own 16 B per token-lane)"
    out["config"]["activations"] = "bfloat16 in memory, fp32 arithmetic and state" if bf16 else "fp32"
    if hconv:
        out["config"]["epilogue"] = "depth-wise harmonic convolution (3 taps per (plane, head) channel) fused behind the clamp"
    if unfused:
        out["config"]["front_end"] = "conv as separate calls (2 x cawn_syntax_conv + scan): 32 B per token-lane"
    fwd_bpl = FWD_BYTES_PER_TOKEN_LANE // (2 if bf16 else 1)
    bwd_bpl = BWD_BYTES_PER_TOKEN_LANE // (2 if bf16 else 1)
    traffic, traffic_src = (None, None) if extra or (stream_mode and args.chunk) else read_traffic(name)

    # ---- roofline of the dominant kernel, from HIP events on the launch stream
    if stream_mode:
        ncalls = nfull + (1 if d_tail is not None else 0)
        per_call_ms = ms_per_step / ncalls
        alg = fwd_bpl * tokens * J / ncalls
        achieved = alg / (per_call_ms * 1e-3) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": fwd_label + f" (per {wl.chunk}-token chunk call, launch gaps included)",
                           "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "traffic": traffic, "traffic_source": traffic_src, "avg_ms": per_call_ms}
        out["stream"] = {"calls": ncalls, "chunk_tokens": wl.chunk, "state_bytes": nstate * 4,
                         "device_mem_delta_bytes": int(mem1 - mem0)}
    else:
        fwd_all = [r[0].elapsed_time(r[1]) for r in recs]
        fwd_ms = float(np.mean(fwd_all))
        out["fwd_ms"] = fwd_ms
        out["fwd_ms_median_min"] = [float(np.median(fwd_all)), float(np.min(fwd_all))]
        out["fwd_tokens_per_s"] = tokens / (fwd_ms * 1e-3)
        out["fwd_GBps"] = fwd_bpl * tokens * J / (fwd_ms * 1e-3) / 1e9
        out["fwd_frac_of_hbm_peak"] = out["fwd_GBps"] / HBM_PEAK_GBS
        if do_bwd:
            bwd_all = [r[1].elapsed_time(r[2]) for r in recs]
            bwd_ms = float(np.mean(bwd_all))
            out["bwd_ms"] = bwd_ms
            out["bwd_ms_median_min"] = [float(np.median(bwd_all)), float(np.min(bwd_all))]
            alg = bwd_bpl * tokens * J
            achieved = alg / (bwd_ms * 1e-3) / 1e9
            out["roofline"] = {"bound": "hbm", "kernel": bwd_label + " (+ its partial-sum reduction)",
                               "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                               "avg_ms": bwd_ms}
        else:
            alg = fwd_bpl * tokens * J
            out["roofline"] = {"bound": "hbm", "kernel": fwd_label, "achieved": out["fwd_GBps"],
                               "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": out["fwd_GBps"] / HBM_PEAK_GBS,
                               "traffic": traffic, "traffic_source": traffic_src, "avg_ms": fwd_ms}
    # the plain-copy ceiling of this run at the dominant kernel's byte count (and at the forward's, for a step
    # with a backward): a copy moves fp32, so a bf16 line is set against the copy of its own byte count too
    cc = {"at_dominant_kernel_bytes": ceiling.gbps(alg)}
    if do_bwd:
        cc["at_forward_bytes"] = ceiling.gbps(fwd_bpl * tokens * J)
    if headline:
        cc["at_50MB"], cc["at_100MB"] = ceiling.gbps(50.3e6), ceiling.gbps(100.7e6)
    out["copy_ceiling_GBps"] = cc
    if cc["at_dominant_kernel_bytes"]:
        out["roofline"]["frac_of_copy_ceiling"] = out["roofline"]["achieved"] / cc["at_dominant_kernel_bytes"]

    # ---- the measured gate: closed fraction over the first batch row of set 0 (one forward with the mask)
    if not unfused:
        W = (J + 31) // 32
        mask = torch.zeros((B, L, W), dtype=torch.int32, device=dev)
        K.check(fwd_call(d, sets[0], None, None, ckpt, mask))
        torch.cuda.synchronize()
        bits = np.unpackbits(mask[0].cpu().numpy().view(np.uint8), bitorder="little").reshape(L, W * 32)[:, :J]
        out["gate_closed_fraction"] = float(1.0 - bits.mean())

    # ---- parity of the timed configuration itself on sampled lanes (head 0: lanes are independent)
    if not (bf16 or unfused):
        from oracle import cawn_oracle as O
        import gpu_util as G
        if stream_mode:                  # the first chunk of a stream: zero state in, state carried out in place
            state.zero_()
            K.check(fwd_call(d, sets[0], state, state, None))
        else:
            step(0)                      # set 0 once more, by the timed calls themselves
        torch.cuda.synchronize()
        got = dict(sets[0])
        if do_bwd:
            got.update(dgamma=None if ret_on else dgamma, dtheta=dtheta, dconv_w=dcw if Kc else None, dconv_b=dcb if Kc else None,
                       dvalve=dvalve, dret=dret)
            if hconv:
                got.update(dhconv_w=dhw, dhconv_b=dhb)
        t_par = time.perf_counter()
        errs = lane_sample_parity(np, G, O, wl, inp, got, "stream" if stream_mode else "batch", Kc, amp_mode=amp_mode,
                                  valve=valve_h, valve_eps=valve_eps, ret=ret_h, ret_bias=ret_bias_h,
                                  hconv=(hw.cpu().numpy(), hb.cpu().numpy()) if hconv else None)
        out["parity_sample"] = {"lanes": f"head 0 ({F} lanes), all {B} batch rows, all tokens of one call",
                                "max_rel_err": max(errs.values()), "per_tensor": errs,
                                "oracle_seconds": round(time.perf_counter() - t_par, 2)}

    # ---- the fp64 oracle on the host cores, on a bounded sample of the same inputs (baseline only)
    if not no_cpu:
        from oracle import cawn_oracle as O
        Ls = min(L, 8192)
        Bs = max(1, min(B, (48 << 20) // (Ls * J)))       # about 10-30 s of CPU work over the host cores
        sub = {k: np.ascontiguousarray(inp[k][:Bs, :Ls]) for k in names}
        cores = O.max_threads()
        cfg = O.Cfg(Bs, Ls, H, F, conv_k=Kc, gate_tau=wl.gate_tau, nthreads=cores)
        t1 = time.perf_counter()
        O.phase_fwd(cfg, sub["mag"], sub["ang"], inp["gamma"], inp["theta"], conv_w=inp["conv_w"],
                    conv_b=inp["conv_b"], want_gate=False)
        if do_bwd:
            O.phase_bwd(cfg, sub["mag"], sub["ang"], inp["gamma"], inp["theta"], sub["dz_re"], sub["dz_im"],
                        conv_w=inp["conv_w"], conv_b=inp["conv_b"])
        cpu_s = time.perf_counter() - t1
        # the same on one thread, on 1/8 of the lanes' worth of tokens
        Ls1 = max(64, Ls // 8)
        cfg1 = O.Cfg(1, Ls1, H, F, conv_k=Kc, gate_tau=wl.gate_tau, nthreads=1)
        sub1 = {k: np.ascontiguousarray(inp[k][:1, :Ls1]) for k in names}
        t2 = time.perf_counter()
        O.phase_fwd(cfg1, sub1["mag"], sub1["ang"], inp["gamma"], inp["theta"], conv_w=inp["conv_w"],
                    conv_b=inp["conv_b"], want_gate=False)
        if do_bwd:
            O.phase_bwd(cfg1, sub1["mag"], sub1["ang"], inp["gamma"], inp["theta"], sub1["dz_re"], sub1["dz_im"],
                        conv_w=inp["conv_w"], conv_b=inp["conv_b"])
        cpu1_s = time.perf_counter() - t2
        out["cpu_baseline"] = {"value": Bs * Ls / cpu_s, "unit": "tokens/s", "cores": cores,
                               "kind": "oracle", "seconds": cpu_s, "single_thread_value": Ls1 / cpu1_s,
                               "sample": f"first {Bs} batch rows x {Ls} tokens x {J} lanes of the same inputs, "
                                         f"{'fwd+bwd' if do_bwd else 'fwd'}, fp64, OpenMP over lanes"}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (lanes and batch rows are independent and would shard "
              f"with no traffic between GPUs); --gpus {args.gpus} is not available", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2604_04250_amd import binding as K
    from paper_2604_04250_amd import workloads as WL

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    K.lib()   # fails loudly when libcawn.so was not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream_like = args.workload == "cfg4_stream"
    if args.steps is None:
        args.steps = 3 if stream_like else 100
    if args.warmup is None:
        args.warmup = 1 if stream_like else 20
    if args.workload == "decode":
        return decode_bench(args, np, torch, K, WL, dev)
    if args.paper:
        assert args.workload == "cfg3_train" and not (args.bf16 or args.unfused), "--paper: alone or with --hconv"
    ceiling = CopyCeiling(np, torch, K, dev)
    out = run_workload(args, args.workload, np, torch, K, WL, dev, ceiling, args.steps, args.warmup, True)
    plain_default = args.workload == "cfg3_train" and not (args.valve or args.ret or args.bf16 or args.hconv or
                                                           args.unfused or args.paper)
    if plain_default and not args.no_other_workloads:
        # the other benchmark configurations ride on the default line (kernel event times, tokens/s, roofline
        # fraction, sampled parity), each with step counts that keep the whole run to a few minutes
        others = {}
        for name, k, w in (("cfg2_layer_fwd", 100, 20), ("cfg4_stream", 2, 1), ("cfg5_wide", 10, 3)):
            torch.cuda.empty_cache()
            r = run_workload(args, name, np, torch, K, WL, dev, ceiling, k, w, False)
            keep = ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "fwd_ms", "bwd_ms", "fwd_GBps",
                    "fwd_frac_of_hbm_peak", "roofline", "copy_ceiling_GBps", "gate_closed_fraction", "parity_sample",
                    "stream")
            others[name] = {"workload": r["config"]["workload"], **{kk: r[kk] for kk in keep if kk in r}}
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
