"""Small driver for hardware-counter runs of the decode kernel.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT -- \
        python3 pmc_probe.py --workload opt6.7b_relu_f16

It launches (a) a plain device-to-device copy of a known size (the calibration
against which the FETCH_SIZE / WRITE_SIZE readings are scaled) and (b) the
sparse decode FFN of every layer of the workload, on random compacted buffers
of the workload's shapes, a few times.  `--what prefill` runs the prefill side
instead: the dense FFN of one layer on the workload's prompt, the selection on
its activations and the deployment of the selected neurons, a few times (for
instruction-issue and LDS counters of those kernels); `--what union` runs the
union-batched decode of the workload's sentences over resident weights after
the calibration copy.  Nothing is timed here.
"""

from __future__ import annotations

import argparse

import torch

from paper_2410_18311_amd import coreinfer as ci
from paper_2410_18311_amd import workloads as wl

COPY_BYTES = 256 << 20


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--workload", default="opt6.7b_relu_f16")
    p.add_argument("--layers", type=int, default=8)
    p.add_argument("--reps", type=int, default=3)
    p.add_argument("--what", choices=["decode", "prefill", "union"], default="decode")
    p.add_argument("--beta", type=float, default=None, help="sentence keep fraction (default: the workload's first)")
    p.add_argument("--down-layout", choices=["auto", "out_major", "neuron_major"], default="auto",
                   help="compact down matrix of the decode run (auto: the library's preference for the shape)")
    args = p.parse_args()
    cfg = wl.WORKLOADS[args.workload]
    dev = "cuda:0"
    d, N, B = cfg.d, cfg.N, cfg.sentences
    beta = cfg.betas[0] if args.beta is None else args.beta
    K = ci.keep_count(beta, N)
    dt = cfg.torch_dtype

    if args.what == "prefill":
        w = wl.layer_weights(cfg, 0, dev)
        X = wl.prefill_hidden(cfg, 0, dev)
        M = X.shape[0]
        A = torch.empty(M, N, dtype=torch.float32, device=dev)
        Y = torch.empty(M, d, dtype=dt, device=dev)
        dws = torch.empty(ci.ffn_dense_workspace_size(M, d, N, dt), dtype=torch.uint8, device=dev)
        sws = torch.empty(ci.select_workspace_size(M, N), dtype=torch.uint8, device=dev)
        core = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.empty(N, dtype=torch.int32, device=dev)
        bufs = None
        for _ in range(args.reps):
            ci.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], cfg.down_layout, cfg.act,
                         want_y=True, want_a=True, Y=Y, A=A, ws=dws)
            ci.select(A, cfg.alpha, beta, core_idx=core, counts=cnt, ws=sws)
            if B == 1:
                bufs = ci.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], cfg.down_layout, cfg.act, core,
                                  out=bufs)
        torch.cuda.synchronize()
        print(f"workload {cfg.name}: prefill of one layer, M={M} d={d} N={N} K={K}, {args.reps} times")
        return

    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)                       # calibration: reads and writes COPY_BYTES each
    torch.cuda.synchronize()

    g = torch.Generator(device=dev)
    g.manual_seed(0)
    mk = lambda *s: (torch.randn(*s, generator=g, device=dev) * 0.02).to(dt)
    gathered = B > 1
    rows = N if gathered else K
    layers = []
    layout = "neuron_major"
    if not gathered and args.what == "decode":
        layout = ci.compact_preferred_layout(K, d, dt, cfg.act) if args.down_layout == "auto" else args.down_layout
    ld = ci.compact_down_ld(K, dt)
    for _ in range(args.layers):
        up = mk(rows, d)
        down = mk(d, ld) if layout == "out_major" else mk(rows, d)
        gate = mk(rows, d) if cfg.act == "swiglu" else None
        bias = mk(ld if layout == "out_major" else rows) if cfg.b_up is not None else None
        idx = None
        if gathered:
            idx = torch.stack([torch.sort(torch.randperm(N, generator=g, device=dev)[:K]).values
                               for _ in range(B)]).to(torch.int32).contiguous()
        layers.append((ci.make_weights(up, gate, bias, down, None, core_idx=idx, down_layout=layout),
                       (up, gate, bias, down, idx)))
    x = mk(B, d) * 50
    y = torch.empty_like(x)
    ws = ci.decode_workspace(B, K, d, dev)
    if args.what == "union":
        rows_total = 0
        for _ in range(args.reps):
            for desc, (up, gate, bias, down, idx) in layers:
                sets = idx if idx is not None else torch.sort(torch.randperm(N, generator=g, device=dev)[:K]).values.to(torch.int32).unsqueeze(0)
                uidx, umask, ucount = ci.union_build(sets.contiguous(), up.shape[0])
                resident = ci.make_weights(up, gate, bias, down, None)
                ci.ffn_decode_union(x[:sets.shape[0]], resident, uidx, umask, ucount, cfg.act)
                rows_total = int(ucount.item())
        torch.cuda.synchronize()
        e = 2 if cfg.dtype != "f32" else 4
        print(f"workload {cfg.name}: union of {B} core sets of {K} = {rows_total} of {N} rows (last layer); "
              f"algorithmic bytes per union-batched decode = {cfg.n_mat * rows_total * d * e} "
              f"(each row of up / gate / down once); calibration copy = {COPY_BYTES} bytes read + {COPY_BYTES} bytes written")
        return
    for _ in range(args.reps):
        for desc, _keep in layers:
            ci.ffn_decode(x, desc, cfg.act, y=y, ws=ws)
    torch.cuda.synchronize()
    n_mat = cfg.n_mat
    e = 2 if cfg.dtype != "f32" else 4
    print(f"workload {cfg.name}: K={K} d={d} B={B} beta={beta} compact down matrix {layout}; algorithmic bytes per decode launch = "
          f"{B * (n_mat * K * d * e + (K * e if cfg.b_up is not None else 0) + 2 * d * e)}; "
          f"calibration copy = {COPY_BYTES} bytes read + {COPY_BYTES} bytes written")


if __name__ == "__main__":
    main()
