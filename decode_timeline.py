#!/usr/bin/env python3
"""In-kernel timeline of the decode FFN kernels, from the 100 MHz time stamps of a development build.

    CI_EXTRA_FLAGS=-DCI_FUSED_STAMPS python3 -m paper_2410_18311_amd.build
    python3 decode_timeline.py --workload llama2_13b_swiglu_bf16 --beta 0.2
    python3 -m paper_2410_18311_amd.build          # back to the normal library

With that flag the kernels write s_memrealtime stamps into the tail of the decode workspace (nothing else
changes; a normal build ignores this script's request and it says so).  For one layer shape the script
runs a few dependent layer calls, eagerly for the stamps and from a HIP graph for the launch-to-launch
period, through both compact layouts:
  neuron-major: ffn_decode_kernel (+ decode_reduce_kernel): start and end of every workgroup;
  output-major: ffn_decode_fused_kernel: start, ring primed, end of every phase (compute wave 0 and the
                service wave), arrival of each chunk of hidden values in LDS, end.
Printed per event: min / median / max over the workgroups, in microseconds after the first workgroup's
start.  period - (last end - first start) is what the launch itself costs (dispatch of a dependent kernel,
ramp-up of the first waves, drain)."""

from __future__ import annotations

import argparse

import numpy as np
import torch

from paper_2410_18311_amd import coreinfer as ci
from paper_2410_18311_amd import workloads as wl

DEV = "cuda:0"
WS_BYTES = 24 << 20


def graph_period_us(fn, layers, reps=20):
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    g.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        g.replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps / layers * 1e3


def stat(col, t0):
    col = (col - t0) / 100.0
    return f"{col.min():7.2f} {np.median(col):7.2f} {col.max():7.2f}"


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--workload", default="llama2_13b_swiglu_bf16")
    p.add_argument("--beta", type=float, default=None)
    p.add_argument("--layers", type=int, default=6)
    p.add_argument("--skew", action="store_true",
                   help="instead of the timelines: end times of the workgroups of ffn_decode_kernel over 48 launches, "
                        "by compute die (workgroup number modulo 8)")
    args = p.parse_args()
    cfg = wl.WORKLOADS[args.workload]
    beta = cfg.betas[0] if args.beta is None else args.beta
    d, N, L = cfg.d, cfg.N, args.layers
    K = ci.keep_count(beta, N)
    e = 2 if cfg.dtype != "f32" else 4
    nbytes = cfg.n_mat * K * d * e + (K * e if cfg.b_up is not None else 0) + 2 * d * e
    print(f"workload {cfg.name} beta {beta}: K = {K}, d = {d}, {nbytes} algorithmic bytes per layer-token "
          f"({nbytes / 8e6:.2f} us at 8 TB/s)")
    xs = wl.decode_hidden(cfg, 1, DEV, tokens=L)
    ys = torch.empty((L, d), dtype=cfg.torch_dtype, device=DEV)
    descs = {"neuron_major": [], "out_major": []}
    keep = []
    for l in range(L):
        w = wl.layer_weights(cfg, l, DEV)
        g = torch.Generator(device="cpu")
        g.manual_seed(l)
        S = torch.randperm(N, generator=g)[:K].sort().values.to(torch.int32).to(DEV)
        for layout in descs:
            c = ci.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], cfg.down_layout, cfg.act, S,
                           down_c_layout=layout)
            descs[layout].append(ci.make_compact_weights(c, w["b_down"]))
            keep.append(c)
        keep.append(w)

    if args.skew:
        ws = torch.zeros(WS_BYTES, dtype=torch.uint8, device=DEV)
        ends = []
        for rep in range(48 // L + 1):
            for l in range(L):
                ci.ffn_decode(xs[l], descs["neuron_major"][l], cfg.act, y=ys[l], ws=ws)
                torch.cuda.synchronize()
                raw = ws[(8 << 20):(8 << 20) + 256 * 8 * 8].view(torch.int64).cpu().numpy().reshape(256, 8).astype(np.float64)
                if raw.max() <= 0:
                    print("no stamps: this is not a -DCI_FUSED_STAMPS build")
                    return
                ends.append((raw[:, 5] - raw[:, 0].min()) / 100.0)
        E = np.array(ends[:48])
        m = E.mean(0)
        print(f"-- ffn_decode_kernel, 256 workgroups, {E.shape[0]} launches: time from the first workgroup's start to each "
              f"workgroup's end, us")
        print(f"   mean over workgroups and launches {E.mean():.2f}; first to end (mean over launches) {E.min(1).mean():.2f}; "
              f"last to end {E.max(1).mean():.2f}")
        print(f"   per-workgroup mean: min {m.min():.2f}, max {m.max():.2f}, standard deviation {m.std():.3f}; "
              f"launch-to-launch standard deviation within a workgroup {E.std(0).mean():.3f}")
        print("   mean end by compute die (workgroup number modulo 8): " + " ".join(f"{m[x::8].mean():.2f}" for x in range(8)))
        half = E.shape[0] // 2
        cc = np.corrcoef(E[:half].mean(0), E[half:].mean(0))[0, 1]
        print(f"   correlation of the per-workgroup mean end between the first and the second half of the launches: {cc:.3f}")
        return

    for layout in ("neuron_major", "out_major"):
        ws = torch.zeros(WS_BYTES, dtype=torch.uint8, device=DEV)

        def layers():
            for l in range(L):
                ci.ffn_decode(xs[l], descs[layout][l], cfg.act, y=ys[l], ws=ws)
        for _ in range(3):
            layers()
        torch.cuda.synchronize()
        if layout == "neuron_major":
            raw = ws[(8 << 20):(8 << 20) + 256 * 8 * 8].view(torch.int64).cpu().numpy().reshape(256, 8).astype(np.float64)
            if raw.max() <= 0:
                print("no stamps: this is not a -DCI_FUSED_STAMPS build")
                return
            t0 = raw[:, 0].min()
            print(f"-- neuron-major compact buffers: ffn_decode_kernel, 256 workgroups (last layer call; the "
                  f"stamps inside the loop are those of the last group of 64 neurons)")
            for i, nm in enumerate(["start", "last up rows dotted", "after the barrier", "hidden values ready",
                                    "last down rows added", "partial sums stored"]):
                print(f"   {nm:26s} {stat(raw[:, i], t0)}")
            span = (raw[:, 5].max() - t0) / 100.0
        else:
            plan = ci.dev_fused_plan(K, d, cfg.torch_dtype, cfg.act)
            C = plan["chunks"]
            ep = int(ws[:4].view(torch.int32).item())
            nst = 8 * 256 * 64
            raw = ws[(1 << 20):(1 << 20) + nst * 8].view(torch.int64).cpu().numpy().reshape(8, 256, 2, 32)
            raw = raw.astype(np.float64)[(ep - 1) & 7]
            cw, sw = raw[:, 0, :], raw[:, 1, :]
            t0 = cw[:, 0].min()
            gs = ws[(1 << 20) + nst * 8:(1 << 20) + nst * 8 + 256 * 96 * 8].view(torch.int64).cpu().numpy()
            gs = gs.reshape(256, 96).astype(np.float64)
            print(f"-- output-major compact buffers: ffn_decode_fused_kernel, {plan} (status {ci.ffn_decode_status(ws)})")
            print(f"   {'compute wave 0: start':40s} {stat(cw[:, 0], t0)}")
            print(f"   {'compute wave 0: ring primed':40s} {stat(cw[:, 1], t0)}")
            for ph in range(2 * C):
                nm = f"A({ph})" if ph < C else f"B({ph - C})"
                print(f"   {'barrier at the end of ' + nm + ' passed':40s} {stat(cw[:, 2 + ph], t0)}")
            for j in range(min(C, 4)):
                if sw[:, 16 + j].max() > 0:
                    print(f"   {'service waves: chunk ' + str(j) + ' in LDS':40s} {stat(sw[:, 16 + j], t0)}")
            print(f"   {'service wave: y written':40s} {stat(sw[:, 31], t0)}")
            row = gs[100]
            n = int((row > 0).sum())
            ends = (row[:n] - t0) / 100.0
            print(f"   workgroup 100, end of each ring group ({n} groups of 4 rows): " + " ".join(f"{v:.2f}" for v in ends))
            if n > 2:
                print(f"   median group period {np.median(np.diff(ends)):.2f} us")
            span = (sw[:, 31].max() - t0) / 100.0
        period = graph_period_us(layers, L)
        print(f"   first start -> last end {span:.2f} us; launch-to-launch period in a HIP graph {period:.2f} us "
              f"({nbytes / period / 1e3:.0f} GB/s, {nbytes / period / 1e3 / 8000:.3f} of 8 TB/s); "
              f"outside that span: {period - span:.2f} us"
              + (" (dispatch of two dependent kernels and decode_reduce_kernel)" if layout == "neuron_major"
                 else " (dispatch of one dependent kernel)"))


if __name__ == "__main__":
    main()
