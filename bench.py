#!/usr/bin/env python3
"""Benchmark of the CoreInfer hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
for every FFN layer the dense prefill FFN, the core-neuron selection and the
weight compaction, then every decode token through every layer's sparse FFN.
Inputs are resident in HBM before the timed region.

A run with no --workload times every workload of the build -- the Llama-2-13B
shape at each of its four keep fractions, the OPT-6.7B and Llama-2-7B shapes
and the OPT-66B shape with eight sentences -- and prints ONE JSON line: its
top-level fields are the Llama-2-13B shape at its first keep fraction (timed
with --steps / --warmup), `workloads` carries the same fields for the others
(at fewer steps, stated in each record).

    python bench.py --gpus 1 --steps 20 --warmup 5
    python bench.py --workload opt6.7b_relu_f16 [--beta 0.4] [--layers 8] ...
"""

from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0, "f32": 157.3}
ROOT = os.path.dirname(os.path.abspath(__file__))
TOP_WORKLOAD = "llama2_13b_swiglu_bf16"
# the other workloads of a default run, with the (steps, warmup) each is timed at
OTHER_WORKLOADS = (("opt6.7b_relu_f16", None, 3, 1), ("llama2_7b_swiglu_bf16", None, 3, 1),
                   (TOP_WORKLOAD, 0.3, 2, 1), (TOP_WORKLOAD, 0.4, 2, 1), (TOP_WORKLOAD, 0.6, 2, 1),
                   ("opt66b_relu_f16_8sent", None, 2, 1))


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=3)
    p.add_argument("--warmup", type=int, default=1)
    p.add_argument("--workload", default=None, help="time this workload only (default: all of them)")
    p.add_argument("--beta", type=float, default=None, help="sentence keep fraction (default: the workload's first)")
    p.add_argument("--decode-tokens", type=int, default=None, help="override (shorter runs while profiling)")
    p.add_argument("--layers", type=int, default=None, help="override the stack depth (profiling only)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--down-layout", choices=["auto", "out_major", "neuron_major"], default="auto",
                   help="layout of the compact down matrix (auto: the library's preference for the shape)")
    p.add_argument("--no-graph", action="store_true", help="launch decode kernels directly instead of a HIP graph")
    p.add_argument("--kernel-reps", type=int, default=20, help="replays of the kernel-only timing graph")
    p.add_argument("--cpu-seconds", type=float, default=12.0, help="oracle time of the top-level cpu_baseline sample")
    return p.parse_args()


def read_traffic_note(workload: str, beta: float, algorithmic_bytes: int):
    """HBM-side bytes per decode launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE),
    if a summary has been committed for this workload at the same launch size."""
    for name in (f"pmc_ffn_decode_{workload}_beta{beta:g}.txt", f"pmc_ffn_decode_{workload}.txt"):
        traffic, alg = None, None
        try:
            for line in open(os.path.join(ROOT, "profiles", name)):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = float(line.split(":", 1)[1])
                if line.startswith("algorithmic_bytes_per_launch:"):
                    alg = int(line.split(":", 1)[1])
        except OSError:
            continue
        if alg is not None and abs(alg - algorithmic_bytes) <= 0.001 * algorithmic_bytes:
            return traffic
    return None


class Inputs:
    """Weights and hidden states of one workload, resident on the GPU (shared by its keep fractions)."""

    def __init__(self, cfg, dev):
        import torch
        from paper_2410_18311_amd import workloads as wl
        L, B = cfg.L, cfg.sentences
        self.cfg = cfg
        self.weights = [wl.layer_weights(cfg, l, dev) for l in range(L)]
        # the sentences of a batch share the layer's weights: their prompts go through the dense prefill
        # FFN as one [B * M, d] matrix (one pass over the weights), selection then runs per sentence
        self.X = [torch.cat([wl.prefill_hidden(cfg, l, dev, sentence=s) for s in range(B)], dim=0).contiguous()
                  for l in range(L)]
        # decode inputs: x_all[t] is [L, B, d], one fresh hidden state per layer, sentence and step
        self.x_all = torch.stack([torch.stack([wl.decode_hidden(cfg, l, dev, sentence=s) for s in range(B)], dim=1)
                                  for l in range(L)], dim=1).contiguous()          # [T, L, B, d]
        torch.cuda.synchronize()


def run_workload(inp: Inputs, beta: float, steps: int, warmup: int, args, cpu_seconds: float) -> dict:
    import numpy as np
    import torch
    from paper_2410_18311_amd import coreinfer as ci

    cfg = inp.cfg
    dev = inp.x_all.device
    weights, X, x_all = inp.weights, inp.X, inp.x_all
    L, M, d, N, T, B = cfg.L, cfg.M, cfg.d, cfg.N, cfg.decode_tokens, cfg.sentences
    e = 4 if cfg.dtype == "f32" else 2
    K = ci.keep_count(beta, N)
    gathered = B > 1                      # several sentences: rows gathered from the resident weights
    dtype = cfg.torch_dtype
    n_mat = cfg.n_mat

    # ------------------------------------------------------------------ buffers (untimed)
    x_cur = torch.empty((L, B, d), dtype=dtype, device=dev)
    y_out = torch.empty((L, B, d), dtype=dtype, device=dev)
    A_buf = torch.empty((B * M, N), dtype=torch.float32, device=dev)
    Y_buf = torch.empty((B * M, d), dtype=dtype, device=dev)
    dense_ws = torch.empty(ci.ffn_dense_workspace_size(B * M, d, N, dtype), dtype=torch.uint8, device=dev)
    sel_ws = torch.empty(ci.select_batch_workspace_size(B, M, N), dtype=torch.uint8, device=dev)
    counts = torch.empty((B, N), dtype=torch.int32, device=dev)
    core_idx = torch.empty((L, B, K), dtype=torch.int32, device=dev)
    # zeroed once: the single-launch decode exchanges hidden values through tagged words in it
    dec_ws = ci.decode_workspace(B, K, d, dev)
    if gathered:
        cbuf = None
        descs = [ci.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], core_idx=core_idx[l])
                 for l, w in enumerate(weights)]
    else:
        # compact buffers in the layout the library prefers for this shape: output-major down matrix
        # (single-launch decode) for large layers, neuron-major (two launches) for small ones
        down_c_layout = (ci.compact_preferred_layout(K, d, dtype, cfg.act) if args.down_layout == "auto"
                         else args.down_layout)
        cbuf = [ci.compact_buffers(K, d, dtype, dev, cfg.act == "swiglu", cfg.b_up is not None, down_c_layout)
                for _ in range(L)]
        descs = [ci.make_compact_weights(c, w["b_down"]) for c, w in zip(cbuf, weights)]
    torch.cuda.synchronize()

    def dense_layer(l):
        w = weights[l]
        ci.ffn_dense(X[l], w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], cfg.down_layout,
                     cfg.act, want_y=True, want_a=True, Y=Y_buf, A=A_buf, ws=dense_ws)

    def prefill_layer(l):
        w = weights[l]
        dense_layer(l)
        # all sentences of the batch in one set of launches
        ci.select_batch(A_buf, B, cfg.alpha, beta, core_idx=core_idx[l], counts=counts, ws=sel_ws)
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

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    marks = [[ev(), ev(), ev()] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(marks[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    prefill_ms = sum(m[0].elapsed_time(m[1]) for m in marks) / steps
    decode_ms = sum(m[1].elapsed_time(m[2]) for m in marks) / steps
    decode_tokens_per_step = T * B
    tokens_per_s = decode_tokens_per_step / (decode_ms * 1e-3)
    decode_status = ci.ffn_decode_status(dec_ws) if (not gathered and down_c_layout == "out_major") else 0

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

    dense_ms = timed(lambda: [dense_layer(l) for l in range(L)]) / L   # per layer, all B sentences together
    scratch_idx = torch.empty(K, dtype=torch.int32, device=dev)   # keeps the real core sets intact
    select_ms = timed_graph(lambda: [ci.select(A_buf[:M], cfg.alpha, beta, core_idx=scratch_idx, counts=counts[0],
                                               ws=sel_ws) for l in range(L)]) / L
    select_batch_ms = None
    if B > 1:
        scratch_idx_b = torch.empty((B, K), dtype=torch.int32, device=dev)
        select_batch_ms = timed_graph(lambda: [ci.select_batch(A_buf, B, cfg.alpha, beta, core_idx=scratch_idx_b,
                                                               counts=counts, ws=sel_ws) for l in range(L)]) / L
    # the same prefill without an fp32 score matrix: the dense FFN hands out the hidden matrix in the
    # element type and the selection ranks it (reported beside the default path, never part of `value`)
    hidden_prefill = None
    if cfg.dtype != "f32":
        H_buf = torch.empty((B * M, N), dtype=dtype, device=dev)
        run_h = lambda: [ci.ffn_dense_hidden(X[l], weights[l]["w_up"], weights[l]["w_gate"], weights[l]["b_up"],
                                             weights[l]["w_down"], weights[l]["b_down"], cfg.down_layout, cfg.act,
                                             Y=Y_buf, H=H_buf, ws=dense_ws) for l in range(L)]
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

    # what a launch of the decode's size reaches on this chip when it only streams: a plain GEMV over
    # rows of w_up of (about) the same byte count per layer, no dependency between workgroups, one
    # dependent launch per layer from a HIP graph like the decode
    stream_ref = None
    if not gathered:
        rows = min(N, n_mat * K) // 64 * 64
        a_ref = torch.empty((1, rows), dtype=torch.float32, device=dev)

        def stream_layers():
            for l in range(L):
                ci.ffn_dense(x_cur[l, :1], weights[l]["w_up"][:rows], None, None, None, None, cfg.down_layout, "relu",
                             want_y=False, want_a=True, A=a_ref, ws=dws)
        s_ms = timed_graph(stream_layers, reps=5) / L
        s_bytes = rows * d * e
        stream_ref = {"kernel": "up_rows_kernel (one GEMV over rows of w_up, no dependency between workgroups)",
                      "bytes_per_launch": s_bytes, "us_per_launch": s_ms * 1e3,
                      "gbps": s_bytes / (s_ms * 1e-3) / 1e9, "frac_of_hbm_peak": s_bytes / (s_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    # --------------------- several sentences: the same decode through the union of their core sets
    # (a different algorithm from the gathered decode that `value` reports: every union row is read
    # once for all its owners; reported beside it, never as `value`)
    union = None
    if gathered and B <= 8:
        resident = [ci.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"]) for w in weights]
        # GPU time of the build's launches (replayed from a HIP graph: launched one by one from Python the
        # host's output allocations and four launches per call would be what is measured)
        ubuild_ms = timed_graph(lambda: [ci.union_build(core_idx[l], N) for l in range(L)]) / L
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
        union_bytes = rows0 * d * e * n_mat
        union = {"tokens_per_s": B / (union_ms * 1e-3), "us_per_layer_step": union_ms * 1e3 / L,
                 "union_rows_layer0": rows0, "algorithmic_bytes_per_layer_step": union_bytes,
                 "gbps": union_bytes * L / (union_ms * 1e-3) / 1e9,
                 "frac_of_hbm_peak": union_bytes * L / (union_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                 "union_build_us_per_layer": ubuild_ms * 1e3,
                 "max_abs_diff_vs_gathered_over_rms": union_vs_gathered,
                 "note": "each row of the union of the sentences' core sets is read once; a different "
                         "algorithm from the gathered decode, same result per sentence"}
        del unions, resident, u_ws

    # ------------- everything coreinfer_ffn_decode launches, alone: HIP events on the launch stream
    # around a graph of the L dependent calls of one token (no input copies in between)
    decode_token_layers()
    torch.cuda.synchronize()
    kgraph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(kgraph):
        decode_token_layers()
    torch.cuda.synchronize()
    kgraph.replay()
    kernel_ms = timed(kgraph.replay, reps=args.kernel_reps) / L
    del kgraph

    # the least a launch of that size can take (measured last: it leaves the roofline figure above alone): a kernel that only reads the same number of bytes
    # (16-byte loads, 64 KB in flight per compute unit, no arithmetic, nothing passed from one half to
    # the other, nothing written), again one dependent launch per layer from a HIP graph
    read_ref = None
    if not gathered:
        per_iter = 512 * 8 * 16
        want = n_mat * K * d * e
        iters = max(1, want // (256 * per_iter))
        r_bytes = iters * per_iter * 256
        regions = max(4, min(L, -(-(600 << 20) // r_bytes)))   # more than the memory-side cache holds
        probe_buf = torch.ones(regions * r_bytes, dtype=torch.uint8, device=dev)
        probe_out = torch.zeros(256, dtype=torch.int32, device=dev)

        def read_layers():
            for r in range(regions):
                ci.dev_stream_probe(probe_buf[r * r_bytes:(r + 1) * r_bytes], iters * per_iter, True, 256, 512, 8, iters,
                                    probe_out)
        r_ms = timed_graph(read_layers, reps=5) / regions
        read_ref = {"kernel": "stream_probe_kernel (reads only: no dots, no dependency, no output)",
                    "bytes_per_launch": r_bytes, "us_per_launch": r_ms * 1e3,
                    "gbps": r_bytes / (r_ms * 1e-3) / 1e9, "frac_of_hbm_peak": r_bytes / (r_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        del probe_buf

    bytes_per_launch = B * (n_mat * K * d * e + (K * e if cfg.b_up is not None else 0) + 2 * d * e)
    if gathered:
        bytes_per_launch += B * K * 4
    traffic = read_traffic_note(cfg.name, beta, bytes_per_launch)
    e2e_gbps = bytes_per_launch * L * T / (decode_ms * 1e-3) / 1e9
    if gathered:
        # the sentences' core sets overlap and the rows shared between them are served by the caches:
        # algorithmic bytes over time would exceed what memory delivered, so the counter bytes are used
        basis = traffic if traffic is not None else bytes_per_launch
        achieved_gbps = basis / (kernel_ms * 1e-3) / 1e9
        roof_note = ("achieved = bytes that missed the L2 (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy of "
                     "known size: requests the L2 passed on, served by the memory-side cache or HBM) / time; "
                     "not a bandwidth claim for HBM alone" if traffic is not None else
                     "no committed counter summary for this launch size: algorithmic bytes / time, which counts "
                     "rows shared between sentences once per sentence; not a bandwidth claim")
        kernels = "ffn_decode_kernel + decode_reduce_kernel (gathered rows of resident weights)"
    else:
        achieved_gbps = bytes_per_launch / (kernel_ms * 1e-3) / 1e9
        roof_note = "achieved = algorithmic bytes of one layer-token / time of everything coreinfer_ffn_decode launches"
        kernels = ("ffn_decode_fused_kernel (one launch per layer-token)" if down_c_layout == "out_major" else
                   "ffn_decode_kernel + decode_reduce_kernel (two launches per layer-token)")
    roofline = {"kernel": kernels, "bound": "hbm", "achieved": achieved_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved_gbps / HBM_PEAK_GBPS, "traffic": traffic, "bytes_per_launch": bytes_per_launch,
                "us_per_launch": kernel_ms * 1e3, "note": roof_note}

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
        sample_layers = sorted({0, L // 2, L - 1})
        sample_sentences = sorted({0, B - 1})
        per_layer_budget = cpu_seconds / len(sample_layers)
        max_tok = min(64, T)
        sets_equal = True
        worst = 0.0
        oracle_s, oracle_tokens, select_cpu_ms = 0.0, 0, []
        for l in sample_layers:
            w = weights[l]
            dense_layer(l)          # fresh prefill of this layer on the GPU, its activations handed to the oracle
            torch.cuda.synchronize()
            S_refs = {}
            for s in sample_sentences:
                A_host = A_buf[s * M:(s + 1) * M].cpu().numpy()
                ts = time.perf_counter()
                S_refs[s], _ = orc.select(A_host, cfg.alpha, beta)
                select_cpu_ms.append((time.perf_counter() - ts) * 1e3)
                sets_equal &= bool(np.array_equal(S_refs[s], core_idx[l, s].cpu().numpy().astype(np.int64)))
            Wu, Wg = f64(w["w_up"]), f64(w["w_gate"])
            Wd = f64(w["w_down"])
            if cfg.down_layout == "neuron_major":
                Wd = Wd.T
            bu, bd = f64(w["b_up"]), f64(w["b_down"])
            # a bounded sample: decode tokens of this layer until its share of the oracle time has gone
            spent, n_l = 0.0, 0
            while n_l < max_tok and (n_l < 2 or spent < per_layer_budget):
                s = sample_sentences[n_l % len(sample_sentences)]
                xt = x_all[n_l, l, s]
                xi = f64(xt)
                ts = time.perf_counter()
                if cfg.act == "relu":
                    ref = orc.ffn_relu(xi, S_refs[s], Wu, bu, Wd, bd)
                else:
                    ref = orc.ffn_swiglu(xi, S_refs[s], Wg, Wu, Wd, bd)
                spent += time.perf_counter() - ts
                if gathered:
                    dsc = ci.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"],
                                          core_idx=core_idx[l, s:s + 1])
                    y = ci.ffn_decode(xt.reshape(1, d).contiguous(), dsc, cfg.act)
                else:
                    y = ci.ffn_decode(xt.reshape(1, d).contiguous(), descs[l], cfg.act, ws=dec_ws)
                torch.cuda.synchronize()
                worst = max(worst, float(np.max(np.abs(f64(y[0]) - ref)) / np.sqrt(np.mean(ref ** 2))))
                n_l += 1
            oracle_s += spent
            oracle_tokens += n_l
            del Wu, Wg, Wd
        per_layer_token = oracle_s / oracle_tokens
        cpu = {"value": 1.0 / (per_layer_token * L), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"float64 numpy oracle, layers {sample_layers}, {oracle_tokens} layer-tokens in "
                         f"{oracle_s:.1f} s, scaled by L={L}; oracle select of one layer and sentence took "
                         f"{np.mean(select_cpu_ms):.0f} ms",
               "select_ms_per_layer": float(np.mean(select_cpu_ms))}
        parity = {"core_set_bit_exact": sets_equal, "decode_max_abs_err_over_rms": worst,
                  "tolerance": 1e-5 if cfg.dtype == "f32" else 2e-2, "layers": sample_layers,
                  "sentences": sample_sentences, "layer_tokens_checked": oracle_tokens}

    dense_flops = 2.0 * B * M * d * N * n_mat
    return {
        "metric": "decode_sparse_ffn_tokens_per_s",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "dtype": cfg.dtype,
        "config": {"workload": cfg.name, "act": cfg.act, "d_model": d, "d_ff": N, "layers": L,
                   "prefill_tokens": M, "decode_tokens": T, "sentences": B, "alpha": cfg.alpha, "beta": beta,
                   "core_neurons": K, "decode_mode": "gathered" if gathered else f"compacted, w_down_c {down_c_layout}",
                   "decode_launch": "direct" if args.no_graph else "hip_graph_per_token",
                   "value_definition": "decode tokens of a step / GPU time of the step's decode phase (HIP events)"},
        "step_breakdown_ms": {"prefill_select_compact": prefill_ms, "decode": decode_ms,
                              "tokens_per_s_whole_step": decode_tokens_per_step / (ms_per_step * 1e-3)},
        "decode_hbm_gbps_whole_phase": e2e_gbps,
        "decode_hbm_frac_whole_phase": e2e_gbps / HBM_PEAK_GBPS,
        "decode_status_word": decode_status,
        "select_us_per_layer": select_ms * 1e3,
        "select_batch_us_per_layer": None if select_batch_ms is None else select_batch_ms * 1e3,
        "compact_us_per_layer": None if compact_ms is None else compact_ms * 1e3,
        "dense_prefill_ms_per_layer": dense_ms,
        "dense_prefill_tflops": dense_flops / (dense_ms * 1e-3) / 1e12,
        "dense_prefill_mfma_frac": dense_flops / (dense_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[cfg.dtype],
        "dense_decode_tokens_per_s": B / (dense_decode_ms * 1e-3),
        "roofline": roofline,
        "streaming_reference": stream_ref,
        "read_only_reference": read_ref,
        "hidden_ranked_prefill": hidden_prefill,
        "union_batched_decode": union,
        "cpu_baseline": cpu,
        "parity": parity,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2410_18311_amd import build as _build
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library()
    from paper_2410_18311_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def config_of(name):
        cfg = wl.WORKLOADS[name]
        if args.layers:
            cfg = cfg.scaled(L=args.layers)
        if args.decode_tokens:
            cfg = cfg.scaled(decode_tokens=args.decode_tokens)
        return cfg

    def note(msg):
        print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)

    if args.workload is not None:
        cfg = config_of(args.workload)
        beta = args.beta if args.beta is not None else cfg.betas[0]
        top = run_workload(Inputs(cfg, dev), beta, args.steps, args.warmup, args, args.cpu_seconds)
        others = None
    else:
        t_start = time.perf_counter()
        cfg = config_of(TOP_WORKLOAD)
        inputs = Inputs(cfg, dev)
        note(f"{cfg.name} beta {cfg.betas[0]}: {args.steps} steps")
        top = run_workload(inputs, cfg.betas[0], args.steps, args.warmup, args, args.cpu_seconds)
        others = []
        for name, beta, steps, warmup in OTHER_WORKLOADS:
            cfg = config_of(name)
            if inputs.cfg.name != cfg.name:
                del inputs
                gc.collect()
                torch.cuda.empty_cache()
                inputs = Inputs(cfg, dev)
            beta = cfg.betas[0] if beta is None else beta
            note(f"{cfg.name} beta {beta}: {steps} steps ({time.perf_counter() - t_start:.0f} s so far)")
            others.append(run_workload(inputs, beta, steps, warmup, args, min(args.cpu_seconds, 4.0)))
            gc.collect()
            torch.cuda.empty_cache()
        note(f"done in {time.perf_counter() - t_start:.0f} s")

    out = dict(top)
    out.update({"n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"})
    if others is not None:
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
