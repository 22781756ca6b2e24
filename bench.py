#!/usr/bin/env python3
"""Benchmark of the CoreInfer hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input
(the OPT-6.7B-shaped stack by default): for every FFN layer the dense prefill
FFN, the core-neuron selection and the weight compaction, then every decode
token through every layer's sparse FFN.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line (see README / DESIGN for the fields).

    python bench.py --gpus 1 --steps 3 --warmup 1 [--workload NAME]
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0, "f32": 157.3}
ROOT = os.path.dirname(os.path.abspath(__file__))


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=3)
    p.add_argument("--warmup", type=int, default=1)
    p.add_argument("--workload", default="opt6.7b_relu_f16")
    p.add_argument("--beta", type=float, default=None, help="sentence keep fraction (default: the workload's first)")
    p.add_argument("--decode-tokens", type=int, default=None, help="override (shorter runs while profiling)")
    p.add_argument("--layers", type=int, default=None, help="override the stack depth (profiling only)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-graph", action="store_true", help="launch decode kernels directly instead of a HIP graph")
    p.add_argument("--kernel-reps", type=int, default=20, help="replays of the kernel-only timing graph")
    return p.parse_args()


def read_traffic_note(workload: str, algorithmic_bytes: int):
    """HBM bytes per launch of the dominant kernel measured with rocprofv3
    --pmc (FETCH_SIZE / WRITE_SIZE), if a summary has been committed for this
    workload at the same launch size (same keep fraction)."""
    path = os.path.join(ROOT, "profiles", f"pmc_ffn_decode_{workload}.txt")
    traffic, alg = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":", 1)[1])
            if line.startswith("algorithmic_bytes_per_launch:"):
                alg = int(line.split(":", 1)[1])
    except OSError:
        return None
    if alg is None or abs(alg - algorithmic_bytes) > 0.001 * algorithmic_bytes:
        return None
    return traffic


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2410_18311_amd import build as _build
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library()
    from paper_2410_18311_amd import coreinfer as ci
    from paper_2410_18311_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = wl.WORKLOADS[args.workload]
    if args.layers:
        cfg = cfg.scaled(L=args.layers)
    if args.decode_tokens:
        cfg = cfg.scaled(decode_tokens=args.decode_tokens)
    beta = args.beta if args.beta is not None else cfg.betas[0]
    L, M, d, N, T, B = cfg.L, cfg.M, cfg.d, cfg.N, cfg.decode_tokens, cfg.sentences
    e = 4 if cfg.dtype == "f32" else 2
    K = ci.keep_count(beta, N)
    gathered = B > 1                      # several sentences: rows gathered from the resident weights
    dtype = cfg.torch_dtype

    # ------------------------------------------------------------------ inputs (untimed)
    weights = [wl.layer_weights(cfg, l, dev) for l in range(L)]
    # the sentences of a batch share the layer's weights: their prompts go through the dense prefill
    # FFN as one [B * M, d] matrix (one pass over the weights), selection then runs per sentence
    X = [torch.cat([wl.prefill_hidden(cfg, l, dev, sentence=s) for s in range(B)], dim=0).contiguous()
         for l in range(L)]
    # decode inputs: x_all[t] is [L, B, d], one fresh hidden state per layer, sentence and step
    x_all = torch.stack([torch.stack([wl.decode_hidden(cfg, l, dev, sentence=s) for s in range(B)], dim=1)
                         for l in range(L)], dim=1).contiguous()          # [T, L, B, d]
    x_cur = torch.empty((L, B, d), dtype=dtype, device=dev)
    y_out = torch.empty((L, B, d), dtype=dtype, device=dev)
    A_buf = torch.empty((B * M, N), dtype=torch.float32, device=dev)
    Y_buf = torch.empty((B * M, d), dtype=dtype, device=dev)
    dense_ws = torch.empty(ci.ffn_dense_workspace_size(B * M, d, N, dtype), dtype=torch.uint8, device=dev)
    sel_ws = torch.empty(ci.select_workspace_size(M, N), dtype=torch.uint8, device=dev)
    counts = torch.empty(N, dtype=torch.int32, device=dev)
    counts_all = torch.empty((L, N), dtype=torch.int32, device=dev) if (B == 1 and len(cfg.betas) > 1) else None
    core_idx = torch.empty((L, B, K), dtype=torch.int32, device=dev)
    dec_ws = torch.empty(ci.ffn_decode_workspace_size(B, K, d), dtype=torch.uint8, device=dev)
    if gathered:
        cbuf = None
        descs = [ci.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], core_idx=core_idx[l])
                 for l, w in enumerate(weights)]
    else:
        cbuf = [{"w_up_c": torch.empty((K, d), dtype=dtype, device=dev),
                 "w_gate_c": torch.empty((K, d), dtype=dtype, device=dev) if cfg.act == "swiglu" else None,
                 "b_up_c": torch.empty((K,), dtype=dtype, device=dev) if cfg.b_up is not None else None,
                 "w_down_c": torch.empty((K, d), dtype=dtype, device=dev)} for _ in range(L)]
        descs = [ci.make_weights(c["w_up_c"], c["w_gate_c"], c["b_up_c"], c["w_down_c"], w["b_down"])
                 for c, w in zip(cbuf, weights)]
    torch.cuda.synchronize()

    def prefill_layer(l):
        w = weights[l]
        ci.ffn_dense(X[l], w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], cfg.down_layout,
                     cfg.act, want_y=True, want_a=True, Y=Y_buf, A=A_buf, ws=dense_ws)
        for s in range(B):
            ci.select(A_buf[s * M:(s + 1) * M], cfg.alpha, beta, core_idx=core_idx[l, s],
                      counts=counts if counts_all is None else counts_all[l], ws=sel_ws)
        if not gathered:
            ci.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], cfg.down_layout, cfg.act,
                       core_idx[l, 0], out=cbuf[l])

    def decode_token_layers():
        for l in range(L):
            ci.ffn_decode(x_cur[l], descs[l], cfg.act, y=y_out[l], ws=dec_ws)

    # first pass outside any capture: fills core_idx / compact buffers, sets kernel attributes
    for l in range(L):
        prefill_layer(l)
    x_cur.copy_(x_all[0])
    decode_token_layers()
    torch.cuda.synchronize()

    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            decode_token_layers()
        torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(marks=None):
        if marks is not None:
            marks[0].record()
        for l in range(L):
            prefill_layer(l)
        if marks is not None:
            marks[1].record()
        for t in range(T):
            x_cur.copy_(x_all[t])
            if graph is not None:
                graph.replay()
            else:
                decode_token_layers()
        if marks is not None:
            marks[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [[ev(), ev(), ev()] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(marks[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    prefill_ms = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps
    decode_ms = sum(m[1].elapsed_time(m[2]) for m in marks) / args.steps
    decode_tokens_per_step = T * B
    tokens_per_s = decode_tokens_per_step / (decode_ms * 1e-3)

    # ---------------------------------------------- per-stage latencies (untimed extra pass)
    def timed(fn, reps=1):
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def timed_graph(fn, reps=3):
        """GPU time of fn's launches replayed from a HIP graph: for stages of a few tens of
        microseconds, where launching from Python would otherwise be what is measured."""
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        return timed(g.replay, reps)

    w0 = weights[0]
    dense_ms = timed(lambda: [ci.ffn_dense(X[l], weights[l]["w_up"], weights[l]["w_gate"], weights[l]["b_up"],
                                           weights[l]["w_down"], weights[l]["b_down"], cfg.down_layout, cfg.act,
                                           want_y=True, want_a=True, Y=Y_buf, A=A_buf, ws=dense_ws)
                              for l in range(L)]) / L   # per layer, all B sentences together
    scratch_idx = torch.empty(K, dtype=torch.int32, device=dev)   # keeps the real core sets intact
    select_ms = timed_graph(lambda: [ci.select(A_buf[:M], cfg.alpha, beta, core_idx=scratch_idx, counts=counts,
                                               ws=sel_ws) for l in range(L)]) / L
    # the same prefill without an fp32 score matrix: the dense FFN hands out the hidden matrix in the
    # element type and the selection ranks it (reported beside the default path, never part of `value`)
    hidden_prefill = None
    if cfg.dtype != "f32":
        H_buf = torch.empty((B * M, N), dtype=dtype, device=dev)
        hws = dense_ws   # large enough: it also holds the split partial products of Y
        run_h = lambda: [ci.ffn_dense_hidden(X[l], weights[l]["w_up"], weights[l]["w_gate"], weights[l]["b_up"],
                                             weights[l]["w_down"], weights[l]["b_down"], cfg.down_layout, cfg.act,
                                             Y=Y_buf, H=H_buf, ws=hws) for l in range(L)]
        run_h()
        dense_h_ms = timed(run_h) / L
        idx_h = torch.empty(K, dtype=torch.int32, device=dev)
        cnt_h = torch.empty(N, dtype=torch.int32, device=dev)
        sel_h = lambda: [ci.select_hidden(H_buf[:M], cfg.act, cfg.alpha, beta, core_idx=idx_h, counts=cnt_h, ws=sel_ws)
                         for l in range(L)]
        select_h_ms = timed_graph(sel_h) / L
        hidden_prefill = {"dense_ms_per_layer": dense_h_ms, "select_us_per_layer": select_h_ms * 1e3,
                          "fp32_score_bytes_not_written_per_layer": B * M * N * 4,
                          "note": "coreinfer_ffn_dense_hidden + coreinfer_select_hidden: the selection ranks the "
                                  "16-bit hidden matrix the down projection reads; a different reading of which "
                                  "activation Def. 1 ranks, so its core sets can differ from the default path's"}
        del H_buf
    compact_ms = None
    if not gathered:
        compact_ms = timed(lambda: [ci.compact(weights[l]["w_up"], weights[l]["w_gate"], weights[l]["b_up"],
                                               weights[l]["w_down"], cfg.down_layout, cfg.act, core_idx[l, 0],
                                               out=cbuf[l]) for l in range(L)]) / L
    # dense decode baseline (all N neurons), one token through every layer
    Yd = torch.empty((B, d), dtype=dtype, device=dev)
    dws = torch.empty(ci.ffn_dense_workspace_size(1, d, N, dtype), dtype=torch.uint8, device=dev)
    def dense_decode():
        for l in range(L):
            w = weights[l]
            for s in range(B):
                ci.ffn_dense(x_cur[l, s:s + 1], w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"],
                             cfg.down_layout, cfg.act, want_y=True, want_a=False, Y=Yd[s:s + 1], ws=dws)
    dense_decode()
    dense_decode_ms = timed(dense_decode, reps=3)

    # ------------- keep-fraction sweep: one prefill and one count set, Def. 2 + deployment + decode per beta
    sweep = None
    if counts_all is not None and args.beta is None:
        sweep = []
        cs_ws = torch.empty(256, dtype=torch.uint8, device=dev)
        n_tok = max(1, min(T, 64))
        for b2 in cfg.betas[1:]:
            K2 = ci.keep_count(b2, N)
            idx2 = torch.empty((L, K2), dtype=torch.int32, device=dev)
            bufs2 = [{"w_up_c": torch.empty((K2, d), dtype=dtype, device=dev),
                      "w_gate_c": torch.empty((K2, d), dtype=dtype, device=dev) if cfg.act == "swiglu" else None,
                      "b_up_c": torch.empty((K2,), dtype=dtype, device=dev) if cfg.b_up is not None else None,
                      "w_down_c": torch.empty((K2, d), dtype=dtype, device=dev)} for _ in range(L)]

            def redeploy():
                for l in range(L):
                    w = weights[l]
                    ci.count_select(counts_all[l], M, b2, core_idx=idx2[l], ws=cs_ws)
                    ci.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], cfg.down_layout, cfg.act, idx2[l],
                               out=bufs2[l])
            redeploy()
            redeploy_ms = timed(redeploy) / L
            descs2 = [ci.make_weights(c["w_up_c"], c["w_gate_c"], c["b_up_c"], c["w_down_c"], w["b_down"])
                      for c, w in zip(bufs2, weights)]
            ws2 = torch.empty(ci.ffn_decode_workspace_size(1, K2, d), dtype=torch.uint8, device=dev)

            def layers2():
                for l in range(L):
                    ci.ffn_decode(x_cur[l], descs2[l], cfg.act, y=y_out[l], ws=ws2)
            layers2()
            torch.cuda.synchronize()
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                layers2()
            torch.cuda.synchronize()

            def tokens2():
                for t in range(n_tok):
                    x_cur.copy_(x_all[t])
                    g2.replay()
            tokens2()
            tok_ms = timed(tokens2) / n_tok
            bytes2 = cfg.n_mat * K2 * d * e + (K2 * e if cfg.b_up is not None else 0) + 2 * d * e
            sweep.append({"beta": b2, "core_neurons": K2, "tokens_per_s": 1.0 / (tok_ms * 1e-3),
                          "decode_hbm_gbps_whole_phase": bytes2 * L / (tok_ms * 1e-3) / 1e9,
                          "count_select_plus_compact_us_per_layer": redeploy_ms * 1e3, "decode_tokens_timed": n_tok})
            del g2, bufs2, descs2, idx2, ws2

    # --------------------- several sentences: the same decode through the union of their core sets
    # (a different algorithm from the gathered decode that `value` reports: every union row is read
    # once for all its owners; reported beside it, never as `value`)
    union = None
    if gathered and B <= 8:
        resident = [ci.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"]) for w in weights]
        ubuild_ms = timed(lambda: [ci.union_build(core_idx[l], N) for l in range(L)]) / L
        unions = [ci.union_build(core_idx[l], N) for l in range(L)]
        u_ws = torch.empty(ci.ffn_decode_union_workspace_size(B, min(N, B * K), d, dtype, cfg.act),
                           dtype=torch.uint8, device=dev)
        y_union = torch.empty((L, B, d), dtype=dtype, device=dev)

        def union_token_layers():
            for l in range(L):
                ci.ffn_decode_union(x_cur[l], resident[l], *unions[l], cfg.act, y=y_union[l], ws=u_ws)

        x_cur.copy_(x_all[0])
        union_token_layers()
        decode_token_layers()
        torch.cuda.synchronize()
        rms = float(y_out.float().pow(2).mean().sqrt())
        union_vs_gathered = float((y_union.float() - y_out.float()).abs().max()) / rms
        ugraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(ugraph):
            union_token_layers()
        torch.cuda.synchronize()
        ugraph.replay()
        n_rep = max(1, min(T, 8))
        union_ms = timed(ugraph.replay, reps=n_rep)
        del ugraph
        rows0 = int(unions[0][2].item())
        union_bytes = rows0 * d * e * cfg.n_mat
        union = {"tokens_per_s": B / (union_ms * 1e-3), "us_per_layer_step": union_ms * 1e3 / L,
                 "union_rows_layer0": rows0, "algorithmic_bytes_per_layer_step": union_bytes,
                 "gbps": union_bytes * L / (union_ms * 1e-3) / 1e9,
                 "union_build_us_per_layer": ubuild_ms * 1e3,
                 "max_abs_diff_vs_gathered_over_rms": union_vs_gathered,
                 "note": "each row of the union of the sentences' core sets is read once; a different "
                         "algorithm from the gathered decode, same result per sentence"}

    # ------------------------------- dominant kernel alone: HIP events around a graph of its launches
    ci.set_param("decode_skip_reduce", 1)
    try:
        decode_token_layers()
        torch.cuda.synchronize()
        kgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(kgraph):
            decode_token_layers()
        torch.cuda.synchronize()
        kgraph.replay()
        kernel_ms = timed(kgraph.replay, reps=args.kernel_reps) / L
        del kgraph
    finally:
        ci.set_param("decode_skip_reduce", 0)
    n_mat = cfg.n_mat
    bytes_per_launch = B * (n_mat * K * d * e + (K * e if cfg.b_up is not None else 0) + 2 * d * e)
    if gathered:
        bytes_per_launch += B * K * 4
    achieved_gbps = bytes_per_launch / (kernel_ms * 1e-3) / 1e9
    e2e_gbps = bytes_per_launch * L * T / (decode_ms * 1e-3) / 1e9
    traffic = read_traffic_note(cfg.name, bytes_per_launch)

    # ------------------------------------------------------------- CPU oracle baseline + parity
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import coreinfer_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
        f64 = lambda t: None if t is None else t.detach().cpu().to(torch.float64).numpy()
        # fresh prefill of layer 0, sentence 0 on the GPU, its activations handed to the oracle
        ci.ffn_dense(X[0], w0["w_up"], w0["w_gate"], w0["b_up"], w0["w_down"], w0["b_down"], cfg.down_layout,
                     cfg.act, want_y=True, want_a=True, Y=Y_buf, A=A_buf, ws=dense_ws)
        torch.cuda.synchronize()
        A_host = A_buf[:M].cpu().numpy()
        ts = time.perf_counter()
        S_ref, _ = orc.select(A_host, cfg.alpha, beta)
        select_cpu_ms = (time.perf_counter() - ts) * 1e3
        sets_equal = bool(np.array_equal(S_ref, core_idx[0, 0].cpu().numpy().astype(np.int64)))
        Wu, Wg = f64(w0["w_up"]), f64(w0["w_gate"])
        Wd = f64(w0["w_down"])
        if cfg.down_layout == "neuron_major":
            Wd = Wd.T
        bu, bd = f64(w0["b_up"]), f64(w0["b_down"])
        # a bounded sample: decode tokens of layer 0 until about ten seconds of oracle time have gone
        max_tok = min(64, T)
        xs = x_all[:max_tok, 0, 0]
        ts = time.perf_counter()
        refs = []
        while len(refs) < max_tok and (len(refs) < 6 or time.perf_counter() - ts < 10.0):
            xi = f64(xs[len(refs)])
            if cfg.act == "relu":
                refs.append(orc.ffn_relu(xi, S_ref, Wu, bu, Wd, bd))
            else:
                refs.append(orc.ffn_swiglu(xi, S_ref, Wg, Wu, Wd, bd))
        n_tok = len(refs)
        per_layer_token = (time.perf_counter() - ts) / n_tok
        cpu = {"value": 1.0 / (per_layer_token * L), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"float64 numpy oracle, layer 0 only, {n_tok} decode tokens, scaled by L={L}; "
                         f"oracle select of one layer took {select_cpu_ms:.0f} ms",
               "select_ms_per_layer": select_cpu_ms}
        worst = 0.0
        for i in range(n_tok):
            x1 = xs[i].reshape(1, d).contiguous()
            if gathered:
                dsc = ci.make_weights(w0["w_up"], w0["w_gate"], w0["b_up"], w0["w_down"], w0["b_down"],
                                      core_idx=core_idx[0, :1])
            else:
                dsc = descs[0]
            y = ci.ffn_decode(x1, dsc, cfg.act)
            torch.cuda.synchronize()
            ref = refs[i]
            worst = max(worst, float(np.max(np.abs(f64(y[0]) - ref)) / np.sqrt(np.mean(ref ** 2))))
        parity = {"core_set_bit_exact": sets_equal, "decode_max_abs_err_over_rms": worst,
                  "tolerance": 1e-5 if cfg.dtype == "f32" else 2e-2}

    out = {
        "metric": "decode_sparse_ffn_tokens_per_s",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "act": cfg.act, "d_model": d, "d_ff": N, "layers": L,
                   "prefill_tokens": M, "decode_tokens": T, "sentences": B, "alpha": cfg.alpha, "beta": beta,
                   "core_neurons": K, "decode_mode": "gathered" if gathered else "compacted",
                   "decode_launch": "direct" if args.no_graph else "hip_graph_per_token",
                   "value_definition": "decode tokens of a step / GPU time of the step's decode phase (HIP events)"},
        "step_breakdown_ms": {"prefill_select_compact": prefill_ms, "decode": decode_ms,
                              "tokens_per_s_whole_step": decode_tokens_per_step / (ms_per_step * 1e-3)},
        "decode_hbm_gbps_whole_phase": e2e_gbps,
        "decode_hbm_frac_whole_phase": e2e_gbps / HBM_PEAK_GBPS,
        "select_us_per_layer": select_ms * 1e3,
        "compact_us_per_layer": None if compact_ms is None else compact_ms * 1e3,
        "dense_prefill_ms_per_layer": dense_ms,
        "dense_prefill_tflops": 2.0 * B * M * d * N * n_mat / (dense_ms * 1e-3) / 1e12,
        "dense_prefill_mfma_frac": 2.0 * B * M * d * N * n_mat / (dense_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[cfg.dtype],
        "dense_decode_tokens_per_s": B / (dense_decode_ms * 1e-3),
        "roofline": {"kernel": "ffn_decode_kernel", "bound": "hbm", "achieved": achieved_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved_gbps / HBM_PEAK_GBPS,
                     "traffic": traffic, "bytes_per_launch": bytes_per_launch,
                     "us_per_launch": kernel_ms * 1e3},
        "hidden_ranked_prefill": hidden_prefill,
        "beta_sweep": sweep,
        "union_batched_decode": union,
        "cpu_baseline": cpu,
        "parity": parity,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
