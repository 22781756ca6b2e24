"""GPU parity of the single-launch decode (compact buffers with an output-major
down matrix, coreinfer_ffn_decode with down_layout = CI_DOWN_OUT_MAJOR) and of
the deployment that writes those buffers, against the CPU oracle."""

import numpy as np
import pytest
import torch

from oracle import coreinfer_oracle as orc
from tests._util import assert_close_rms, down_out_major64, f64, rand_weights

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _say(*a):
    print(*a, flush=True)


def _oracle_ffn(act, x, S, w, layout):
    Wd = down_out_major64(w, layout)
    if act == "relu":
        return orc.ffn_relu(f64(x), S, f64(w["w_up"]), f64(w["b_up"]), Wd, f64(w["b_down"]))
    return orc.ffn_swiglu(f64(x), S, f64(w["w_gate"]), f64(w["w_up"]), Wd, f64(w["b_down"]))


def _check_out_major_buffers(lib, out, ref, K, dtype, bias):
    """w_down_c [d, ld]: the oracle's columns (it returns them transposed) and zero padding."""
    ld = lib.compact_down_ld(K, dtype)
    got = f64(out["w_down_c"])
    assert got.shape[1] == ld and ld >= K and ld % (16 // out["w_down_c"].element_size()) == 0
    assert np.array_equal(got[:, :K], ref["w_down_c"].T)
    assert not got[:, K:].any(), "padding columns must be zero"
    assert np.array_equal(f64(out["w_up_c"]), ref["w_up_c"])
    if "w_gate_c" in ref:
        assert np.array_equal(f64(out["w_gate_c"]), ref["w_gate_c"])
    if bias:
        assert np.array_equal(f64(out["b_up_c"])[:K], ref["b_up_c"])


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("act,layout", [("relu", "out_major"), ("swiglu", "out_major"), ("relu", "neuron_major"),
                                        ("swiglu", "neuron_major")])
@pytest.mark.parametrize("d,N,K", [(64, 200, 77), (1024, 3000, 1201), (256, 1024, 1024), (8, 5, 1),
                                   (104, 520, 300), (72, 4096, 100), (192, 2056, 2056), (136, 1544, 97)])
def test_compact_out_major_matches_oracle(lib, dt, act, layout, d, N, K):
    _say("compact (output-major) case", dt, act, layout, d, N, K)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, layout, seed=d + N + K, device=DEV)
    S = np.sort(np.random.default_rng(K).choice(N, size=K, replace=False))
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act, idx, status=status,
                      down_c_layout="out_major")
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    ref = orc.compact(S, f64(w["w_up"]), down_out_major64(w, layout), f64(w["w_gate"]), f64(w["b_up"]))
    _check_out_major_buffers(lib, out, ref, K, dtype, w["b_up"] is not None)


def test_compact_out_major_flags_bad_indices_without_faulting(lib):
    d, N = 64, 100
    for layout in ("out_major", "neuron_major"):
        w = rand_weights(d, N, torch.float16, "relu", layout, seed=1, device=DEV)
        idx = torch.tensor([3, 5, 5, 250, -1, 40, 41], dtype=torch.int32, device=DEV)  # repeat, out of range, descending
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        out = lib.compact(w["w_up"], None, w["b_up"], w["w_down"], layout, "relu", idx, status=status,
                          down_c_layout="out_major")
        torch.cuda.synchronize()
        assert int(status.item()) == 1
        Wd = down_out_major64(w, layout)
        got = f64(out["w_down_c"])
        for k, n in enumerate([3, 5, None, None, None, 40, 41]):
            want = np.zeros(d) if n is None else Wd[:, n]
            assert np.array_equal(got[:, k], want), (layout, k)
        assert not got[:, 7:].any()


@pytest.mark.parametrize("dt,act,layout", [("f16", "relu", "out_major"), ("bf16", "swiglu", "out_major"),
                                           ("f32", "relu", "neuron_major"), ("f16", "swiglu", "neuron_major")])
@pytest.mark.parametrize("d,N,K,turnover", [(64, 200, 77, 0.3), (1024, 3000, 1201, 0.1), (256, 500, 500, 0.0),
                                            (512, 4000, 1500, 1.0), (8, 5, 1, 1.0)])
def test_compact_update_out_major_matches_oracle(lib, dt, act, layout, d, N, K, turnover):
    """Two updates in a row on buffers with an output-major down matrix: slot map and buffers
    bit-exact against the oracle's rule, the single-launch decode over the updated buffers against
    the oracle FFN of the new set."""
    _say("compact update (output-major) case", dt, act, layout, d, N, K, turnover)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, layout, seed=d + N + K, device=DEV)
    rng = np.random.default_rng(K * 3 + d)
    S = np.sort(rng.choice(N, size=K, replace=False))
    slot = torch.from_numpy(S.astype(np.int32)).to(DEV)
    bufs = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act, slot, down_c_layout="out_major")
    slot_ref = S.copy()
    x = torch.randn(1, d, generator=torch.Generator().manual_seed(K)).to(dtype).to(DEV)
    ws = lib.decode_workspace(1, K, d, DEV)
    for step in range(2):
        n_new = min(int(round(turnover * K)), N - K)
        stay = rng.choice(slot_ref, size=K - n_new, replace=False)
        fresh = rng.choice(np.setdiff1d(np.arange(N), slot_ref), size=n_new, replace=False)
        S_new = np.sort(np.concatenate([stay, fresh]))
        changed = lib.compact_update(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act,
                                     torch.from_numpy(S_new.astype(np.int32)).to(DEV), slot, bufs)
        torch.cuda.synchronize()
        slot_ref, changed_ref = orc.compact_update_slots(slot_ref, S_new)
        assert int(changed.item()) == changed_ref == n_new
        assert slot.cpu().numpy().astype(np.int64).tolist() == slot_ref.tolist()
        ref = orc.compact(slot_ref, f64(w["w_up"]), down_out_major64(w, layout), f64(w["w_gate"]), f64(w["b_up"]))
        _check_out_major_buffers(lib, bufs, ref, K, dtype, w["b_up"] is not None)
        y = lib.ffn_decode(x, lib.make_compact_weights(bufs, w["b_down"]), act, ws=ws)
        torch.cuda.synchronize()
        assert lib.ffn_decode_status(ws) == 0
        assert_close_rms(y[0], _oracle_ffn(act, x[0], np.sort(slot_ref), w, layout), dtype, f"decode after update {step}")


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("act", ["relu", "swiglu"])
@pytest.mark.parametrize("d,N,K,B", [
    (256, 1024, 410, 1), (64, 300, 1, 2), (1000, 2500, 999, 1), (4096, 3000, 1201, 1), (5120, 1500, 577, 3),
    (9216, 700, 333, 2), (2048, 4000, 2765, 1), (4096, 7000, 6554, 1), (512, 9000, 9000, 1), (8, 40, 17, 1),
    (24576, 300, 130, 1),
])
def test_decode_single_launch_matches_oracle(lib, dt, act, d, N, K, B):
    _say("single-launch decode case", dt, act, d, N, K, B)
    dtype = DTYPES[dt]
    if dt == "f32" and d > 16384:
        pytest.skip("more than four 16-byte loads per thread and row")
    w = rand_weights(d, N, dtype, act, "out_major", seed=d * 7 + K, device=DEV)
    S = np.sort(np.random.default_rng(K + 1).choice(N, size=K, replace=False))
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], "out_major", act, idx, down_c_layout="out_major")
    x = torch.randn(B, d, generator=torch.Generator().manual_seed(d + B)).to(dtype).to(DEV)
    desc = lib.make_compact_weights(c, w["b_down"])
    ws = lib.decode_workspace(B, K, d, DEV)
    y = lib.ffn_decode(x, desc, act, ws=ws)
    y2 = lib.ffn_decode(x, desc, act, ws=ws)      # the same workspace again: every call leaves it ready
    torch.cuda.synchronize()
    assert lib.ffn_decode_status(ws) == 0
    assert torch.equal(y, y2), "decode must be deterministic"
    assert_close_rms(y, _oracle_ffn(act, x, S, w, "out_major"), dtype, "single-launch decode")
    # and the two-launch path over neuron-major buffers of the same set agrees within the same bar
    c2 = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], "out_major", act, idx)
    y3 = lib.ffn_decode(x, lib.make_compact_weights(c2, w["b_down"]), act)
    torch.cuda.synchronize()
    assert_close_rms(y3, _oracle_ffn(act, x, S, w, "out_major"), dtype, "two-launch decode")


def test_decode_single_launch_random_shapes(lib):
    """Seeded sweep: widths that are no multiple of any tile, core sets from one neuron to all of
    them, one to four rows of x, with and without biases, both layouts of the resident down matrix."""
    rng = np.random.default_rng(11)
    for case in range(40):
        dt = ["f16", "bf16", "f32"][case % 3]
        act = ["relu", "swiglu"][(case // 3) % 2]
        dtype = DTYPES[dt]
        d = 8 * int(rng.integers(1, 900))
        N = int(rng.integers(1, 9000))
        K = int(rng.choice([1, N, max(1, N // 2), int(rng.integers(1, N + 1))]))
        B = int(rng.integers(1, 5))
        layout = ["out_major", "neuron_major"][case % 2]
        bias = case % 4 != 3
        _say("single-launch random case", case, dt, act, d, N, K, B, layout, "bias" if bias else "no bias")
        w = rand_weights(d, N, dtype, act, layout, seed=1900 + case, device=DEV, bias=bias)
        x = torch.randn(B, d, generator=torch.Generator().manual_seed(case)).to(dtype).to(DEV)
        S = np.sort(rng.choice(N, size=K, replace=False))
        c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act,
                        torch.from_numpy(S.astype(np.int32)).to(DEV), down_c_layout="out_major")
        ws = lib.decode_workspace(B, K, d, DEV)
        y = lib.ffn_decode(x, lib.make_compact_weights(c, w["b_down"]), act, ws=ws)
        torch.cuda.synchronize()
        assert lib.ffn_decode_status(ws) == 0
        for b in range(B):
            assert_close_rms(y[b], _oracle_ffn(act, x[b], S, w, layout), dtype, f"random case {case} row {b}")


def test_decode_single_launch_one_workspace_for_many_layers(lib):
    """One zeroed workspace serves a stack of layers of the same shape, call after call (the way a
    decoder uses it): no call needs it cleared again."""
    d, N, K, L = 1024, 3000, 1201, 6
    ws = lib.decode_workspace(1, K, d, DEV)
    layers = []
    for l in range(L):
        w = rand_weights(d, N, torch.bfloat16, "swiglu", "out_major", seed=300 + l, device=DEV)
        S = np.sort(np.random.default_rng(l).choice(N, size=K, replace=False))
        c = lib.compact(w["w_up"], w["w_gate"], None, w["w_down"], "out_major", "swiglu",
                        torch.from_numpy(S.astype(np.int32)).to(DEV), down_c_layout="out_major")
        layers.append((w, S, lib.make_compact_weights(c, w["b_down"]), c))
    for t in range(3):
        x = torch.randn(L, d, generator=torch.Generator().manual_seed(40 + t)).to(torch.bfloat16).to(DEV)
        ys = [lib.ffn_decode(x[l], layers[l][2], "swiglu", ws=ws) for l in range(L)]
        torch.cuda.synchronize()
        assert lib.ffn_decode_status(ws) == 0
        for l in range(L):
            w, S = layers[l][0], layers[l][1]
            assert_close_rms(ys[l], _oracle_ffn("swiglu", x[l], S, w, "out_major"), torch.bfloat16, f"token {t} layer {l}")


def test_decode_single_launch_graph_replays_match_eager(lib):
    """The single launch captured in a HIP graph gives the eager result on every replay, with other
    work and synchronisations in between: the call's tag advances on the device."""
    d, N, K = 1024, 3000, 1201
    w = rand_weights(d, N, torch.float16, "relu", "out_major", seed=5, device=DEV)
    S = np.sort(np.random.default_rng(1).choice(N, size=K, replace=False))
    c = lib.compact(w["w_up"], None, w["b_up"], w["w_down"], "out_major", "relu",
                    torch.from_numpy(S.astype(np.int32)).to(DEV), down_c_layout="out_major")
    desc = lib.make_compact_weights(c, w["b_down"])
    x = torch.randn(1, d, generator=torch.Generator().manual_seed(2)).half().to(DEV)
    y = torch.empty_like(x)
    ws = lib.decode_workspace(1, K, d, DEV)
    lib.ffn_decode(x, desc, "relu", y=y, ws=ws)
    torch.cuda.synchronize()
    eager = y.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        lib.ffn_decode(x, desc, "relu", y=y, ws=ws)
        lib.ffn_decode(x, desc, "relu", y=y, ws=ws)   # two dependent launches on one workspace
    for i in range(5):
        y.zero_()
        (torch.randn(256, 256, device=DEV) @ torch.randn(256, 256, device=DEV)).sum().item()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager), f"replay {i}"
        assert lib.ffn_decode_status(ws) == 0
    # new input through the same graph
    x.copy_(torch.randn(1, d, generator=torch.Generator().manual_seed(3)).half())
    g.replay()
    torch.cuda.synchronize()
    assert_close_rms(y[0], _oracle_ffn("relu", x[0], S, w, "out_major"), torch.float16, "graph, new input")
