"""GPU parity: every entry point of the C ABI against the CPU oracle on the
same seeded inputs.  Index sets and counts bit-exact; FFN outputs within
TOL * rms(oracle output) (tests/_util.py)."""

import numpy as np
import pytest
import torch

from oracle import coreinfer_oracle as orc
from paper_2410_18311_amd import workloads as wl
from tests._util import TOL, assert_close_rms, down_out_major64, f64, rand_weights, score_bound

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _say(*a):
    print(*a, flush=True)


# --------------------------------------------------------------------- select

def _select_case(lib, A_np, alpha, beta, what):
    _say("select case", what, A_np.shape, alpha, beta)
    A = torch.from_numpy(np.ascontiguousarray(A_np, dtype=np.float32)).to(DEV)
    S_gpu, c_gpu = lib.select(A, alpha, beta)
    torch.cuda.synchronize()
    S_ref, c_ref = orc.select(A_np.astype(np.float32), alpha, beta)
    assert c_gpu.cpu().numpy().astype(np.int64).tolist() == c_ref.tolist(), what + ": counts"
    assert S_gpu.cpu().numpy().astype(np.int64).tolist() == S_ref.tolist(), what + ": core set"


@pytest.mark.parametrize("M,N,kind,levels,alpha,beta", [
    (1, 1, "abs", 0, 0.2, 0.4),
    (1, 64, "relu", 0, 0.5, 0.5),
    (3, 100, "raw", 0, 0.2, 0.4),
    (32, 1024, "relu", 0, 0.2, 0.4),
    (7, 4097, "relu", 0, 0.2, 0.4),
    (17, 4100, "abs", 5, 0.3, 0.25),          # heavy ties in the activations
    (64, 11008, "abs", 0, 0.2, 0.4),
    (33, 16384, "relu", 0, 0.2, 0.4),
    (300, 2048, "relu", 0, 0.2, 0.4),          # more tokens than workgroups: LDS-private counters
    (700, 1500, "abs", 3, 0.1, 0.6),
    (300, 11008, "abs", 0, 0.2, 0.4),          # more tokens than compute units: two workgroups per unit
    (515, 16384, "relu", 9, 0.2, 0.4),
    (5, 36864, "relu", 0, 0.2, 0.4),
    (6, 22016, "abs", 0, 0.2, 0.4),            # 22, 28, 36, 40 keys per thread: the register-cached variants
    (4, 28672, "relu", 4, 0.2, 0.4),
    (3, 36000, "abs", 6, 0.3, 0.3),
    (3, 40960, "relu", 0, 0.2, 0.4),
    (3, 50000, "abs", 0, 0.05, 0.1),           # beyond the register-cached sizes
    (2, 70001, "relu", 0, 0.2, 0.4),           # more than 65536 neurons: Def. 2 in one workgroup, streaming
    (40, 66000, "abs", 4, 0.1, 0.3),
    (9, 13824, "abs", 0, 1.0, 1.0),
    (9, 1000, "relu", 2, 1.0, 0.001),
])
def test_select_matches_oracle(lib, M, N, kind, levels, alpha, beta):
    A = wl.activation_like(M, N, seed=M * 131 + N, kind=kind, levels=levels)
    _select_case(lib, A, alpha, beta, f"{kind}/{levels}")


def test_select_random_shapes_and_tie_patterns(lib):
    """Seeded sweep over shapes and value patterns the fixed cases do not list: every
    keys-per-thread variant of the kernels, few and many distinct values, keep fractions
    from 0.1 % to 100 %, rows of different sparsity, special values."""
    rng = np.random.default_rng(20241018)
    widths = [1, 2, 63, 64, 65, 255, 257, 1000, 4095, 4096, 4097, 8200, 12288, 16385, 20000, 24577, 30000,
              33000, 36865, 40961, 45000]
    for case in range(48):
        N = int(widths[case % len(widths)]) if case < 2 * len(widths) else int(rng.integers(1, 45000))
        M = int(rng.integers(1, 24)) if N > 8192 else int(rng.integers(1, 400))
        kind = ["relu", "abs", "raw"][case % 3]
        levels = int(rng.choice([0, 0, 1, 2, 3, 7, 50]))
        alpha = float(rng.choice([0.001, 0.05, 0.2, 0.33, 0.5, 0.999, 1.0]))
        beta = float(rng.choice([0.001, 0.1, 0.25, 0.4, 0.75, 1.0]))
        A = wl.activation_like(M, N, seed=1000 + case, kind=kind, levels=levels)
        if case % 5 == 0:      # rows with very different numbers of positives
            keep = rng.random((M, 1)) ** 3
            A = np.where(rng.random((M, N)) < keep, A, np.float32(0.0)).astype(np.float32)
        if case % 7 == 0:      # special values: +inf ranks first, NaN and -0.0 are never positive
            flat = A.reshape(-1)
            idx = rng.integers(0, flat.size, size=min(6, flat.size))
            flat[idx] = np.array([np.inf, np.nan, -0.0, np.float32(1e-45), -np.inf, np.float32(3.4e38)],
                                 dtype=np.float32)[:idx.size]
        _select_case(lib, A, alpha, beta, f"random case {case}: {kind}/{levels}")


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("act", ["relu", "swiglu"])
@pytest.mark.parametrize("M,N,ld_pad", [(1, 1, 0), (7, 100, 3), (40, 4097, 0), (300, 2048, 4), (9, 16384, 0),
                                        (270, 11008, 0), (5, 36864, 8), (3, 50000, 1)])
def test_select_hidden_matches_oracle(lib, dt, act, M, N, ld_pad):
    """Selection on the hidden matrix in the layer's element type: the oracle ranks the very same
    values (their fp64 images; magnitudes for the gated FFN).  16-bit values tie all the time."""
    dtype = DTYPES[dt]
    _say("select hidden case", dt, act, M, N, ld_pad)
    g = torch.Generator().manual_seed(M * 7 + N)
    h = torch.randn(M, N, generator=g) * 1.5
    if act == "relu":
        h = h.clamp_min(0)
    buf = torch.zeros(M, N + ld_pad, dtype=dtype, device=DEV)
    buf[:, :N] = h.to(dtype).to(DEV)
    H = buf[:, :N]
    S, counts = lib.select_hidden(H, act, 0.2, 0.4)
    torch.cuda.synchronize()
    ranked = f64(H) if act == "relu" else np.abs(f64(H))
    S_ref, c_ref = orc.select(ranked, 0.2, 0.4)
    assert counts.cpu().numpy().tolist() == c_ref.tolist()
    assert S.cpu().numpy().tolist() == S_ref.tolist()


def test_select_hidden_special_values_and_fp32_equivalence(lib):
    h = torch.tensor([[float("inf"), -float("inf"), float("nan"), -0.0, 0.0, 1.0, -2.0, 6e-8, -6e-8, 65504.0]] * 3,
                     dtype=torch.float16, device=DEV)
    for act in ("relu", "swiglu"):
        S, counts = lib.select_hidden(h, act, 0.5, 0.5)
        torch.cuda.synchronize()
        ranked = f64(h) if act == "relu" else np.abs(f64(h))
        S_ref, c_ref = orc.select(ranked, 0.5, 0.5)
        assert counts.cpu().numpy().tolist() == c_ref.tolist() and S.cpu().numpy().tolist() == S_ref.tolist()
    # an fp32 hidden matrix of a ReLU layer: the same call as coreinfer_select
    A = torch.from_numpy(wl.activation_like(33, 3000, seed=5, kind="relu", levels=6)).to(DEV)
    S1, c1 = lib.select(A, 0.2, 0.4)
    S2, c2 = lib.select_hidden(A, "relu", 0.2, 0.4)
    torch.cuda.synchronize()
    assert torch.equal(S1, S2) and torch.equal(c1, c2)


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("act,layout", [("relu", "out_major"), ("swiglu", "neuron_major")])
@pytest.mark.parametrize("M,d,N", [(3, 256, 512), (130, 320, 520), (256, 512, 768), (512, 256, 1024)])
def test_dense_hidden_then_select_hidden(lib, dt, act, layout, M, d, N):
    """The prefill pass without an fp32 score matrix: H against the oracle's hidden state within the
    rounding of the element type, Y against the oracle FFN, and the selection on H bit-exact
    against the oracle ranking those very values."""
    _say("dense hidden case", dt, act, layout, M, d, N)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, layout, seed=M + d + N + 3, device=DEV)
    X = torch.randn(M, d, generator=torch.Generator().manual_seed(M + 2)).to(dtype).to(DEV)
    Y, H = lib.ffn_dense_hidden(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], layout, act)
    S, counts = lib.select_hidden(H, act, 0.2, 0.4)
    torch.cuda.synchronize()
    if act == "relu":
        H_ref = orc.score_relu(f64(X), f64(w["w_up"]), f64(w["b_up"]))
    else:
        H_ref = orc.hidden_swiglu(f64(X), f64(w["w_gate"]), f64(w["w_up"]))
    # one rounding of an fp32 accumulator: half an ulp of the element type, plus fp32 summation noise
    ulp = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8, "f32": 2.0 ** -20}[dt]
    err = np.abs(f64(H) - H_ref)
    assert np.all(err <= ulp * np.abs(H_ref) * 1.01 + 2e-5 * np.sqrt(np.mean(H_ref ** 2)) + 1e-7)
    assert_close_rms(Y, _oracle_ffn(act, X, None, w, layout), dtype, "dense hidden Y")
    ranked = f64(H) if act == "relu" else np.abs(f64(H))
    S_ref, c_ref = orc.select(ranked, 0.2, 0.4)
    assert counts.cpu().numpy().tolist() == c_ref.tolist() and S.cpu().numpy().tolist() == S_ref.tolist()
    # the same H as the dense call that also writes fp32 scores keeps in its workspace -> same Y
    Y2, _ = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], layout, act,
                          want_y=True, want_a=True)
    torch.cuda.synchronize()
    if M > 4:
        assert torch.equal(Y, Y2)


def test_select_ties_at_infinity_and_rows_without_positives(lib):
    """Several +inf in a row with fewer places than infinities (the threshold is +inf and the cut
    falls among them), rows with no positive value at all, and a cut inside a lane's four neurons."""
    N = 300
    A = np.zeros((6, N), dtype=np.float32)
    A[0, [3, 17, 18, 19, 250]] = np.inf          # 5 infinities + 5 ones, alpha keeps 2 of 10
    A[0, [5, 6, 7, 8, 9]] = 1.0
    A[1] = -1.0                                   # nothing positive
    A[2] = np.nan
    A[3, 40:48] = 2.0                             # eight equal values, three kept: the cut is 42
    A[4, 41:44] = 7.0                             # all kept
    A[5, [0, 299]] = np.inf
    for alpha, beta in ((0.2, 0.1), (0.375, 0.05), (1.0, 0.02)):
        _select_case(lib, A, alpha, beta, "ties at infinity")
        H = torch.from_numpy(A).to(torch.float16).to(DEV)
        S, counts = lib.select_hidden(H, "relu", alpha, beta)
        torch.cuda.synchronize()
        S_ref, c_ref = orc.select(f64(H), alpha, beta)
        assert counts.cpu().numpy().tolist() == c_ref.tolist() and S.cpu().numpy().tolist() == S_ref.tolist()


def test_select_degenerate_rows(lib):
    rng = np.random.default_rng(5)
    N = 3000
    A = np.abs(rng.standard_normal((12, N))).astype(np.float32)
    A[0] = 0.0                      # no positive activation at all
    A[1] = 1.25                     # every neuron tied
    A[2] = -np.abs(A[2])            # all negative
    A[3, ::2] = np.nan              # NaN is never positive
    A[4, 7] = np.inf                # +inf ranks first
    A[5, :] = 0.0
    A[5, 2999] = 1e-45              # a single denormal positive
    A[6] = np.float32(1e-38) * np.arange(1, N + 1, dtype=np.float32) / N   # tiny values, low exponents
    A[7, 100:] = 0.0
    A[8] = np.repeat(np.arange(N // 4, dtype=np.float32), 4)[:N]           # runs of four equal values
    _select_case(lib, A, 0.2, 0.4, "degenerate")
    _select_case(lib, A, 0.5, 0.05, "degenerate2")
    _select_case(lib, np.zeros((4, 257), dtype=np.float32), 0.2, 0.4, "all-zero sentence")


def test_select_strided_rows_and_null_counts(lib):
    M, N, ld = 10, 1000, 1024
    A_np = wl.activation_like(M, ld, seed=3, kind="relu")
    A = torch.from_numpy(A_np).to(DEV)
    view = A[:, :N]
    K = lib.keep_count(0.4, N)
    core = torch.empty(K, dtype=torch.int32, device=DEV)
    ws = torch.empty(lib.select_workspace_size(M, N), dtype=torch.uint8, device=DEV)
    rc = lib.raw.coreinfer_select(view.data_ptr(), M, N, ld, 0.2, 0.4, core.data_ptr(), None,
                                  ws.data_ptr(), ws.numel(), None)
    assert rc == 0
    torch.cuda.synchronize()
    S_ref, _ = orc.select(A_np[:, :N], 0.2, 0.4)
    assert core.cpu().numpy().tolist() == S_ref.tolist()


def test_select_is_deterministic_and_permutation_invariant(lib):
    A_np = wl.activation_like(200, 4096, seed=9, kind="relu", levels=8)
    A = torch.from_numpy(A_np).to(DEV)
    S1, c1 = lib.select(A, 0.2, 0.4)
    S2, c2 = lib.select(A, 0.2, 0.4)
    perm = torch.randperm(200, generator=torch.Generator().manual_seed(1)).to(DEV)
    S3, c3 = lib.select(A[perm].contiguous(), 0.2, 0.4)
    torch.cuda.synchronize()
    assert torch.equal(S1, S2) and torch.equal(c1, c2)
    assert torch.equal(S1, S3) and torch.equal(c1, c3)


# -------------------------------------------------------------------- compact

@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("act,layout", [("relu", "out_major"), ("swiglu", "out_major"), ("relu", "neuron_major")])
@pytest.mark.parametrize("d,N,K", [(64, 200, 77), (1024, 3000, 1201), (256, 1024, 1024), (8, 5, 1),
                                   (104, 520, 300), (72, 4096, 100), (192, 2056, 2056), (136, 1544, 97)])
def test_compact_matches_oracle(lib, dt, act, layout, d, N, K):
    _say("compact case", dt, act, layout, d, N, K)
    dtype = DTYPES[dt]
    if dt == "f32" and d % 4:
        pytest.skip("d must be a multiple of 4")
    w = rand_weights(d, N, dtype, act, layout, seed=d + N + K, device=DEV)
    S = np.sort(np.random.default_rng(K).choice(N, size=K, replace=False))
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act, idx, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    ref = orc.compact(S, f64(w["w_up"]), down_out_major64(w, layout), f64(w["w_gate"]), f64(w["b_up"]))
    assert np.array_equal(f64(out["w_up_c"]), ref["w_up_c"])
    assert np.array_equal(f64(out["w_down_c"]), ref["w_down_c"])
    if act == "swiglu":
        assert np.array_equal(f64(out["w_gate_c"]), ref["w_gate_c"])
    if w["b_up"] is not None:
        assert np.array_equal(f64(out["b_up_c"]), ref["b_up_c"])


@pytest.mark.parametrize("B,M,N,alpha,beta,kind", [(8, 64, 5000, 0.2, 0.4, "relu"), (2, 300, 1000, 0.3, 0.25, "abs"),
                                                   (3, 2100, 520, 0.2, 0.4, "relu"), (5, 1, 4097, 0.5, 0.1, "relu"),
                                                   (4, 37, 70000, 0.1, 0.3, "relu"), (1, 40, 300, 0.2, 0.4, "relu")])
def test_select_batch_matches_oracle(lib, B, M, N, alpha, beta, kind):
    """Several sentences selected by one call: each sentence's core set and counts bit-exact against
    the oracle on its own rows (one set of launches where Def. 2 runs in parallel; M >= 2048 or
    N > 65536 take the sentences one after the other), also with a padded row stride."""
    _say("select batch case", B, M, N, alpha, beta, kind)
    A = wl.activation_like(B * M, N, seed=B * 1000 + M + N, kind=kind, levels=16 if M < 100 else 0)
    buf = torch.zeros(B * M, N + 4, dtype=torch.float32, device=DEV)
    buf[:, :N] = torch.from_numpy(A).to(DEV)
    S, counts = lib.select_batch(buf[:, :N], B, alpha, beta)
    torch.cuda.synchronize()
    assert S.shape == (B, orc.keep_count(beta, N)) and counts.shape == (B, N)
    for b in range(B):
        S_ref, c_ref = orc.select(A[b * M:(b + 1) * M], alpha, beta)
        assert counts[b].cpu().numpy().tolist() == c_ref.tolist(), f"sentence {b}: counts"
        assert S[b].cpu().numpy().tolist() == S_ref.tolist(), f"sentence {b}: core set"


@pytest.mark.parametrize("dt,act,layout", [("f16", "relu", "out_major"), ("bf16", "swiglu", "out_major"),
                                           ("f32", "relu", "neuron_major"), ("f16", "swiglu", "neuron_major")])
@pytest.mark.parametrize("d,N,K,turnover", [(64, 200, 77, 0.3), (1024, 3000, 1201, 0.1), (256, 500, 500, 0.0),
                                            (512, 4000, 1500, 1.0), (8, 5, 1, 1.0)])
def test_compact_update_matches_oracle(lib, dt, act, layout, d, N, K, turnover):
    """Two updates in a row: slot map and buffers bit-exact against the oracle's rule, decode over
    the updated buffers against the oracle FFN of the new set."""
    _say("compact update case", dt, act, layout, d, N, K, turnover)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, layout, seed=d + N + K, device=DEV)
    rng = np.random.default_rng(K * 3 + d)
    S = np.sort(rng.choice(N, size=K, replace=False))
    slot = torch.from_numpy(S.astype(np.int32)).to(DEV)
    bufs = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act, slot)
    slot_ref = S.copy()
    x = torch.randn(1, d, generator=torch.Generator().manual_seed(K)).to(dtype).to(DEV)
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
        for key, t in bufs.items():
            if torch.is_tensor(t):
                assert np.array_equal(f64(t), ref[key]), f"{key} after update {step}"
        desc = lib.make_weights(bufs["w_up_c"], bufs["w_gate_c"], bufs["b_up_c"], bufs["w_down_c"], w["b_down"])
        y = lib.ffn_decode(x, desc, act)
        torch.cuda.synchronize()
        assert_close_rms(y[0], _oracle_ffn(act, x[0], np.sort(slot_ref), w, layout), dtype, f"decode after update {step}")


def test_compact_flags_bad_indices_without_faulting(lib):
    d, N = 64, 100
    w = rand_weights(d, N, torch.float16, "relu", "out_major", seed=1, device=DEV)
    idx = torch.tensor([3, 5, 5, 250, -1, 40, 41], dtype=torch.int32, device=DEV)  # repeat, out of range, descending
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = lib.compact(w["w_up"], None, w["b_up"], w["w_down"], "out_major", "relu", idx, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 1
    up_c, down_c = f64(out["w_up_c"]), f64(out["w_down_c"])
    W_up, W_down = f64(w["w_up"]), f64(w["w_down"])
    for k, n in enumerate([3, 5, None, None, None, 40, 41]):
        if n is None:
            assert not up_c[k].any() and not down_c[k].any()
        else:
            assert np.array_equal(up_c[k], W_up[n]) and np.array_equal(down_c[k], W_down[:, n])


# --------------------------------------------------------------------- decode

def _oracle_ffn(act, x, S, w, layout):
    Wd = down_out_major64(w, layout)
    if act == "relu":
        return orc.ffn_relu(f64(x), S, f64(w["w_up"]), f64(w["b_up"]), Wd, f64(w["b_down"]))
    return orc.ffn_swiglu(f64(x), S, f64(w["w_gate"]), f64(w["w_up"]), Wd, f64(w["b_down"]))


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("act", ["relu", "swiglu"])
@pytest.mark.parametrize("d,N,K,B", [
    (256, 1024, 410, 1), (64, 300, 1, 2), (1000, 2500, 999, 1), (4096, 3000, 1201, 1),
    (5120, 1500, 577, 3), (9216, 700, 333, 2), (2048, 4000, 2765, 1),
])
def test_decode_compacted_matches_oracle(lib, dt, act, d, N, K, B):
    _say("decode compact case", dt, act, d, N, K, B)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, "out_major", seed=d * 7 + K, device=DEV)
    S = np.sort(np.random.default_rng(K + 1).choice(N, size=K, replace=False))
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], "out_major", act, idx)
    x = torch.randn(B, d, generator=torch.Generator().manual_seed(d + B)).to(dtype).to(DEV)
    desc = lib.make_weights(c["w_up_c"], c["w_gate_c"], c["b_up_c"], c["w_down_c"], w["b_down"])
    y = lib.ffn_decode(x, desc, act)
    y2 = lib.ffn_decode(x, desc, act)
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "decode must be deterministic"
    assert_close_rms(y, _oracle_ffn(act, x, S, w, "out_major"), dtype, "decode compacted")


@pytest.mark.parametrize("dt,act", [("f16", "relu"), ("bf16", "swiglu"), ("f32", "relu")])
@pytest.mark.parametrize("d,N,K,B", [(512, 2000, 801, 4), (9216, 1200, 480, 8), (64, 64, 64, 1)])
def test_decode_gathered_matches_oracle(lib, dt, act, d, N, K, B):
    _say("decode gathered case", dt, act, d, N, K, B)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, "neuron_major", seed=d + N, device=DEV)
    rng = np.random.default_rng(B * 100 + K)
    S = np.stack([np.sort(rng.choice(N, size=K, replace=False)) for _ in range(B)])
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    x = torch.randn(B, d, generator=torch.Generator().manual_seed(K)).to(dtype).to(DEV)
    desc = lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], core_idx=idx)
    y = lib.ffn_decode(x, desc, act)
    torch.cuda.synchronize()
    for b in range(B):
        assert_close_rms(y[b], _oracle_ffn(act, x[b], S[b], w, "neuron_major"), dtype, f"gathered b={b}")


def test_decode_random_shapes(lib):
    """Seeded sweep: widths that are no multiple of any tile, core sets from one neuron to all of
    them, one to eight rows of x, both ways of handing over the core neurons."""
    rng = np.random.default_rng(7)
    for case in range(36):
        dt = ["f16", "bf16", "f32"][case % 3]
        act = ["relu", "swiglu"][(case // 3) % 2]
        dtype = DTYPES[dt]
        d = 8 * int(rng.integers(1, 700))
        N = int(rng.integers(1, 3000))
        K = int(rng.choice([1, N, max(1, N // 2), int(rng.integers(1, N + 1))]))
        B = int(rng.integers(1, 9))
        gathered = case % 2 == 1
        _say("decode random case", case, dt, act, d, N, K, B, "gathered" if gathered else "compacted")
        layout = "neuron_major" if gathered else "out_major"
        w = rand_weights(d, N, dtype, act, layout, seed=900 + case, device=DEV)
        x = torch.randn(B, d, generator=torch.Generator().manual_seed(case)).to(dtype).to(DEV)
        if gathered:
            S = np.stack([np.sort(rng.choice(N, size=K, replace=False)) for _ in range(B)])
            desc = lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"],
                                    core_idx=torch.from_numpy(S.astype(np.int32)).to(DEV))
        else:
            S1 = np.sort(rng.choice(N, size=K, replace=False))
            S = np.stack([S1] * B)
            c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], layout, act,
                            torch.from_numpy(S1.astype(np.int32)).to(DEV))
            desc = lib.make_weights(c["w_up_c"], c["w_gate_c"], c["b_up_c"], c["w_down_c"], w["b_down"])
        y = lib.ffn_decode(x, desc, act)
        torch.cuda.synchronize()
        for b in range(B):
            assert_close_rms(y[b], _oracle_ffn(act, x[b], S[b], w, layout), dtype, f"random case {case} row {b}")


def test_decode_gathered_ignores_out_of_range_entries(lib):
    d, N, K = 256, 500, 40
    w = rand_weights(d, N, torch.float16, "relu", "neuron_major", seed=2, device=DEV)
    S = np.sort(np.random.default_rng(0).choice(N, size=K, replace=False))
    bad = S.copy().astype(np.int64)
    bad[[3, 17]] = [-5, N + 9]
    idx = torch.from_numpy(bad.astype(np.int32)).to(DEV).unsqueeze(0)
    x = torch.randn(1, d, generator=torch.Generator().manual_seed(1)).half().to(DEV)
    y = lib.ffn_decode(x, lib.make_weights(w["w_up"], None, w["b_up"], w["w_down"], w["b_down"], core_idx=idx), "relu")
    torch.cuda.synchronize()
    keep = np.delete(S, [3, 17])
    assert_close_rms(y[0], _oracle_ffn("relu", x[0], keep, w, "neuron_major"), torch.float16, "skip invalid")


def test_decode_empty_core_set_gives_the_output_bias(lib):
    d = 128
    b_down = (torch.randn(d) * 0.1).half().to(DEV)
    dummy = torch.zeros(1, d, dtype=torch.float16, device=DEV)
    x = torch.randn(2, d).half().to(DEV)
    desc = lib.make_weights(dummy, None, None, dummy, b_down, K=0)
    y = lib.ffn_decode(x, desc, "relu")
    torch.cuda.synchronize()
    assert torch.equal(y[0], b_down) and torch.equal(y[1], b_down)


# ---------------------------------------------------------------------- dense

@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("act,layout", [("relu", "out_major"), ("swiglu", "out_major"),
                                        ("relu", "neuron_major"), ("swiglu", "neuron_major")])
@pytest.mark.parametrize("M,d,N", [(1, 256, 1024), (3, 512, 1000), (32, 256, 1024), (130, 320, 520), (256, 1024, 768)])
def test_dense_matches_oracle(lib, dt, act, layout, M, d, N):
    _say("dense case", dt, act, layout, M, d, N)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, layout, seed=M + d + N, device=DEV)
    X = torch.randn(M, d, generator=torch.Generator().manual_seed(M)).to(dtype).to(DEV)
    Y, A = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], layout, act,
                         want_y=True, want_a=True)
    torch.cuda.synchronize()
    if act == "relu":
        A_ref = orc.score_relu(f64(X), f64(w["w_up"]), f64(w["b_up"]))
    else:
        A_ref = orc.score_swiglu(f64(X), f64(w["w_gate"]), f64(w["w_up"]))
    # the scores are fp32 whatever the element type: fp32 layers are held to the fp32 bar
    assert np.max(np.abs(f64(A) - A_ref)) <= score_bound(dtype, act, A_ref, X, w)
    assert_close_rms(Y, _oracle_ffn(act, X, None, w, layout), dtype, "dense Y")
    # A only (no Y) must give the same scores
    _, A2 = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], None, None, layout, act,
                          want_y=False, want_a=True)
    torch.cuda.synchronize()
    assert torch.equal(A, A2)


@pytest.mark.parametrize("direct", [1, 0])
def test_dense_random_shapes(lib, direct):
    """Seeded sweep over prompt lengths and widths around the tile edges of every GEMM variant
    (ragged and even, reduction lengths that are and are not multiples of the k tile), with the
    128 x 128 tiles loaded straight into LDS (the default) and through the register ring."""
    lib.dev_set_param("gemm_direct", direct)
    try:
        _dense_random_shapes(lib)
    finally:
        lib.dev_set_param("gemm_direct", 1)


def _dense_random_shapes(lib):
    rng = np.random.default_rng(11)
    for case in range(30):
        dt = ["f16", "bf16", "f32"][case % 3]
        act = ["relu", "swiglu"][(case // 3) % 2]
        layout = ["out_major", "neuron_major"][(case // 6) % 2]
        dtype = DTYPES[dt]
        vec = 4 if dt == "f32" else 8
        M = int(rng.choice([5, 64, 127, 128, 129, 255, 256, 300, 512]))
        d = vec * int(rng.integers(1, 1200 // vec))
        N = vec * int(rng.integers(1, 1600 // vec))
        if case % 5 == 0:          # shapes every kernel divides
            M, d, N = 256 * int(rng.integers(1, 3)), 64 * int(rng.integers(1, 12)), 256 * int(rng.integers(1, 6))
        _say("dense random case", case, dt, act, layout, M, d, N)
        w = rand_weights(d, N, dtype, act, layout, seed=500 + case, device=DEV)
        X = torch.randn(M, d, generator=torch.Generator().manual_seed(case)).to(dtype).to(DEV)
        Y, A = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], layout, act,
                             want_y=True, want_a=True)
        torch.cuda.synchronize()
        A_ref = (orc.score_relu(f64(X), f64(w["w_up"]), f64(w["b_up"])) if act == "relu"
                 else orc.score_swiglu(f64(X), f64(w["w_gate"]), f64(w["w_up"])))
        rms = np.sqrt(np.mean(A_ref ** 2))
        assert np.max(np.abs(f64(A) - A_ref)) <= score_bound(dtype, act, A_ref, X, w), f"random case {case}: scores"
        assert_close_rms(Y, _oracle_ffn(act, X, None, w, layout), dtype, f"random case {case}: Y")


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("act", ["relu", "swiglu"])
@pytest.mark.parametrize("layout", ["out_major", "neuron_major"])
@pytest.mark.parametrize("M,d,N", [(256, 128, 256), (512, 1024, 768), (256, 576, 1280), (768, 256, 512)])
def test_dense_large_tile_kernel_matches_oracle(lib, dt, act, layout, M, d, N):
    """The 256 x 256 tile kernel, forced for shapes it divides (normally chosen only for large
    grids): up projection with both epilogues and the down projection, split over k or not."""
    _say("dense large-tile case", dt, act, layout, M, d, N)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, layout, seed=M + d + N + 9, device=DEV)
    X = torch.randn(M, d, generator=torch.Generator().manual_seed(M + 1)).to(dtype).to(DEV)
    lib.dev_set_param("gemm_big", 2)
    try:
        Y, A = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], layout, act,
                             want_y=True, want_a=True)
        torch.cuda.synchronize()
    finally:
        lib.dev_set_param("gemm_big", 1)
    if act == "relu":
        A_ref = orc.score_relu(f64(X), f64(w["w_up"]), f64(w["b_up"]))
    else:
        A_ref = orc.score_swiglu(f64(X), f64(w["w_gate"]), f64(w["w_up"]))
    rms = np.sqrt(np.mean(A_ref ** 2))
    assert np.max(np.abs(f64(A) - A_ref)) <= 1e-4 * rms
    assert_close_rms(Y, _oracle_ffn(act, X, None, w, layout), dtype, "dense Y, large tiles")


# ------------------------------------------------------------- whole small path

@pytest.mark.parametrize("layout", ["out_major", "neuron_major"])
def test_dense_many_tiles_with_split_down_projection(lib, layout):
    """288 large tiles (two rounds of workgroups, the second nearly empty): the down projection is
    split over k although the grid is full.  Sampled rows against the oracle."""
    M, d, N = 4096, 4608, 6400
    _say("dense many-tile case", layout, M, d, N)
    w = rand_weights(d, N, torch.float16, "relu", layout, seed=77, device=DEV)
    X = torch.randn(M, d, generator=torch.Generator().manual_seed(3)).to(torch.float16).to(DEV)
    Y, A = lib.ffn_dense(X, w["w_up"], None, w["b_up"], w["w_down"], w["b_down"], layout, "relu",
                         want_y=True, want_a=True)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, M - 1], np.random.default_rng(1).integers(0, M, size=44)]))
    Xs = f64(X)[rows]
    A_ref = orc.score_relu(Xs, f64(w["w_up"]), f64(w["b_up"]))
    assert np.max(np.abs(f64(A)[rows] - A_ref)) <= 1e-4 * np.sqrt(np.mean(A_ref ** 2))
    Y_ref = orc.ffn_relu(Xs, None, f64(w["w_up"]), f64(w["b_up"]), down_out_major64(w, layout), f64(w["b_down"]))
    assert_close_rms(Y[torch.from_numpy(rows).to(DEV)], Y_ref, torch.float16, "split down projection")


@pytest.mark.parametrize("knob,value,default", [("gemm_ring", 0, 1), ("gemm_direct", 0, 1), ("gemm_big", 0, 1), ("select_wgs_per_cu", 1, 2),
                                                ("select_def2_single", 1, 0), ("decode_depth", 8, 4), ("decode_depth", 16, 4),
                                                ("decode_wgs_per_cu", 2, 1), ("decode_nt_store", 0, 1),
                                                ("reduce_cq", 4, 8), ("reduce_cq", 16, 8), ("reduce_threads", 64, 256), ("reduce_threads", 1024, 256),
                                                ("union_depth", 16, 8),
                                                ("union_down_threads", 128, 384), ("decode_threads", 512, 0), ("decode_threads", 64, 0),
                                                ("decode_wgs", 7, 0), ("decode_wgs", 1024, 0), ("union_up_wgs_per_cu", 3, 1),
                                                ("union_down_wgs_per_cu", 1, 2)])
def test_alternative_launch_shapes_give_the_same_results(lib, knob, value, default):
    """Every tuning knob selects among kernels / launch shapes that must all be correct: one prefill
    (dense FFN, selection, deployment) and decode (compacted, gathered, union-batched) pass per
    setting, against the oracle."""
    _say("knob case", knob, value)
    M, d, N, B = 300, 512, 2304, 3
    dt = torch.bfloat16
    w = rand_weights(d, N, dt, "swiglu", "neuron_major", seed=21, device=DEV)
    X = torch.randn(M, d, generator=torch.Generator().manual_seed(8)).to(dt).to(DEV)
    lib.dev_set_param(knob, value)
    try:
        Y, A = lib.ffn_dense(X, w["w_up"], w["w_gate"], None, w["w_down"], w["b_down"], "neuron_major", "swiglu",
                             want_y=True, want_a=True)
        S, counts = lib.select(A, 0.2, 0.3)
        c = lib.compact(w["w_up"], w["w_gate"], None, w["w_down"], "neuron_major", "swiglu", S)
        x = torch.randn(B, d, generator=torch.Generator().manual_seed(9)).to(dt).to(DEV)
        y_c = lib.ffn_decode(x, lib.make_weights(c["w_up_c"], c["w_gate_c"], None, c["w_down_c"], w["b_down"]), "swiglu")
        sets = torch.stack([S, S.flip(0).sort().values, S]).contiguous()
        resident = lib.make_weights(w["w_up"], w["w_gate"], None, w["w_down"], w["b_down"])
        y_g = lib.ffn_decode(x, lib.make_weights(w["w_up"], w["w_gate"], None, w["w_down"], w["b_down"], core_idx=sets),
                             "swiglu")
        uidx, umask, ucount = lib.union_build(sets, N)
        y_u = lib.ffn_decode_union(x, resident, uidx, umask, ucount, "swiglu")
        torch.cuda.synchronize()
    finally:
        lib.dev_set_param(knob, default)
    A_ref = orc.score_swiglu(f64(X), f64(w["w_gate"]), f64(w["w_up"]))
    assert np.max(np.abs(f64(A) - A_ref)) <= 1e-4 * np.sqrt(np.mean(A_ref ** 2))
    assert_close_rms(Y, _oracle_ffn("swiglu", X, None, w, "neuron_major"), dt, f"{knob}: dense Y")
    S_ref, c_ref = orc.select(A.cpu().numpy(), 0.2, 0.3)
    assert S.cpu().numpy().tolist() == S_ref.tolist() and counts.cpu().numpy().tolist() == c_ref.tolist()
    for b in range(B):
        ref = _oracle_ffn("swiglu", x[b], S_ref, w, "neuron_major")
        assert_close_rms(y_c[b], ref, dt, f"{knob}: compacted row {b}")
        assert_close_rms(y_g[b], ref, dt, f"{knob}: gathered row {b}")
        assert_close_rms(y_u[b], ref, dt, f"{knob}: union row {b}")


def test_tiny_fp32_configuration_end_to_end(lib):
    """The small fp32 configuration, whole: prefill 32 tokens, select, compact,
    16 decode steps; every stage against the oracle."""
    cfg = wl.WORKLOADS["tiny_relu_f32"]
    t = wl.tiny_relu_f32_numpy()
    g = {k: (None if v is None else torch.from_numpy(v).to(DEV)) for k, v in t.items()}
    Y, A = lib.ffn_dense(g["x_prefill"], g["w_up"], None, g["b_up"], g["w_down"], g["b_down"],
                         "out_major", "relu", want_y=True, want_a=True)
    torch.cuda.synchronize()
    A_ref = orc.score_relu(t["x_prefill"], t["w_up"], t["b_up"])
    assert_close_rms(A, A_ref, torch.float32, "prefill scores")
    assert_close_rms(Y, orc.ffn_relu(t["x_prefill"], None, t["w_up"], t["b_up"], t["w_down"], t["b_down"]),
                     torch.float32, "prefill Y")
    # selection: bit-exact on identical activation bits (the GPU's own fp32 A) ...
    S_gpu, c_gpu = lib.select(A, cfg.alpha, cfg.betas[0])
    torch.cuda.synchronize()
    S_ref, c_ref = orc.select(A.cpu().numpy(), cfg.alpha, cfg.betas[0])
    assert S_gpu.cpu().numpy().tolist() == S_ref.tolist() and len(S_ref) == 410
    assert c_gpu.cpu().numpy().tolist() == c_ref.tolist()
    # ... and on the oracle's activations rounded to fp32
    A32 = A_ref.astype(np.float32)
    S_gpu2, _ = lib.select(torch.from_numpy(A32).to(DEV), cfg.alpha, cfg.betas[0])
    S_ref2, _ = orc.select(A32, cfg.alpha, cfg.betas[0])
    assert S_gpu2.cpu().numpy().tolist() == S_ref2.tolist()
    _say("tiny: core-set similarity GPU-A vs oracle-A:", orc.core_similarity(S_ref, S_ref2))
    # deploy + decode
    c = lib.compact(g["w_up"], None, g["b_up"], g["w_down"], "out_major", "relu", S_gpu)
    ref_c = orc.compact(S_ref, t["w_up"], t["w_down"], None, t["b_up"])
    assert np.array_equal(c["w_up_c"].cpu().numpy(), ref_c["w_up_c"])
    assert np.array_equal(c["w_down_c"].cpu().numpy(), ref_c["w_down_c"])
    assert np.array_equal(c["b_up_c"].cpu().numpy(), ref_c["b_up_c"])
    desc = lib.make_weights(c["w_up_c"], None, c["b_up_c"], c["w_down_c"], g["b_down"])
    for i in range(cfg.decode_tokens):
        y = lib.ffn_decode(g["x_decode"][i], desc, "relu")
        y_ref = orc.ffn_relu(t["x_decode"][i], S_ref, t["w_up"], t["b_up"], t["w_down"], t["b_down"])
        assert_close_rms(y, y_ref, torch.float32, f"decode token {i}")
    # dense decode (one token through ffn_dense) against the dense oracle
    Yd, _ = lib.ffn_dense(g["x_decode"][:1], g["w_up"], None, g["b_up"], g["w_down"], g["b_down"],
                          "out_major", "relu")
    assert_close_rms(Yd[0], orc.ffn_relu(t["x_decode"][0], None, t["w_up"], t["b_up"], t["w_down"], t["b_down"]),
                     torch.float32, "dense decode")


def test_keep_fraction_one_reproduces_the_dense_ffn(lib):
    d, N, M = 512, 1536, 24
    for dt, act in (("f16", "relu"), ("bf16", "swiglu")):
        dtype = DTYPES[dt]
        w = rand_weights(d, N, dtype, act, "out_major", seed=77, device=DEV)
        X = torch.randn(M, d, generator=torch.Generator().manual_seed(4)).to(dtype).to(DEV)
        _, A = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], "out_major", act,
                             want_y=False, want_a=True)
        S, _ = lib.select(A, 0.2, 1.0)
        torch.cuda.synchronize()
        assert S.cpu().numpy().tolist() == list(range(N))
        c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], "out_major", act, S)
        assert torch.equal(c["w_up_c"], w["w_up"]) and torch.equal(c["w_down_c"], w["w_down"].t().contiguous())
        x = X[:1].contiguous()
        y = lib.ffn_decode(x, lib.make_weights(c["w_up_c"], c["w_gate_c"], c["b_up_c"], c["w_down_c"], w["b_down"]), act)
        assert_close_rms(y[0], _oracle_ffn(act, x[0], None, w, "out_major"), dtype, "beta=1 vs dense oracle")


# ---------------------------------------------- full-size layers, bench launch shape

def _layer_ids(names):
    out = []
    for name in names:
        L = wl.WORKLOADS[name].L
        out += [(name, l) for l in (0, L // 2, L - 1)]
    return out


@pytest.mark.parametrize("name,layer", _layer_ids(["opt6.7b_relu_f16", "llama2_7b_swiglu_bf16",
                                                   "llama2_13b_swiglu_bf16"]))
def test_full_size_layer_compacted(lib, name, layer):
    """First, middle and last layer of each compacted workload at its full shape, every keep
    fraction the workload names: prefill scores sampled against the oracle, selection bit-exact,
    decode through both compact layouts (two launches / single launch) against the oracle."""
    cfg = wl.WORKLOADS[name]
    _say("full-size layer", name, "layer", layer)
    dtype = cfg.torch_dtype
    w = wl.layer_weights(cfg, layer, DEV)
    X = wl.prefill_hidden(cfg, layer, DEV)
    _, A = lib.ffn_dense(X, w["w_up"], w["w_gate"], w["b_up"], None, None, cfg.down_layout, cfg.act,
                         want_y=False, want_a=True)
    torch.cuda.synchronize()
    # sampled rows of A against the oracle (full rows would need the whole fp64 product)
    rows = [0, cfg.M // 2, cfg.M - 1]
    Wu, Wg, Wd = f64(w["w_up"]), f64(w["w_gate"]), f64(w["w_down"])
    if cfg.act == "relu":
        A_ref = orc.score_relu(f64(X[rows]), Wu, f64(w["b_up"]))
    else:
        A_ref = orc.score_swiglu(f64(X[rows]), Wg, Wu)
    rms = np.sqrt(np.mean(A_ref ** 2))
    assert np.max(np.abs(f64(A[rows]) - A_ref)) <= score_bound(dtype, cfg.act, A_ref, X[rows], w), "prefill scores"
    A_host = A.cpu().numpy()
    x = wl.decode_hidden(cfg, layer, DEV, tokens=2)
    for beta in cfg.betas:
        S, counts = lib.select(A, cfg.alpha, beta)
        torch.cuda.synchronize()
        # selection bit-exact on the GPU's own activation bits
        S_ref, c_ref = orc.select(A_host, cfg.alpha, beta)
        assert counts.cpu().numpy().tolist() == c_ref.tolist()
        assert S.cpu().numpy().tolist() == S_ref.tolist()
        assert len(S_ref) == orc.keep_count(beta, cfg.N)
        c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], cfg.down_layout, cfg.act, S)
        co = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], cfg.down_layout, cfg.act, S,
                         down_c_layout="out_major")
        desc = lib.make_compact_weights(c, w["b_down"])
        desc_o = lib.make_compact_weights(co, w["b_down"])
        ws = lib.decode_workspace(1, len(S_ref), cfg.d, DEV)
        for i in range(2):
            if cfg.act == "relu":
                y_ref = orc.ffn_relu(f64(x[i]), S_ref, Wu, f64(w["b_up"]), Wd, f64(w["b_down"]))
            else:
                y_ref = orc.ffn_swiglu(f64(x[i]), S_ref, Wg, Wu, Wd, f64(w["b_down"]))
            y = lib.ffn_decode(x[i], desc, cfg.act)
            rel = assert_close_rms(y, y_ref, dtype, f"{name} layer {layer} beta {beta} token {i}, two launches")
            y1 = lib.ffn_decode(x[i], desc_o, cfg.act, ws=ws)
            rel1 = assert_close_rms(y1, y_ref, dtype, f"{name} layer {layer} beta {beta} token {i}, single launch")
            _say(f"  beta {beta} token {i}: max err / rms = {rel:.2e} (two launches), {rel1:.2e} (single launch)")
        assert lib.ffn_decode_status(ws) == 0
        del c, co


@pytest.mark.parametrize("name,beta", [("opt6.7b_relu_f16", 0.4), ("llama2_7b_swiglu_bf16", 0.4),
                                       ("llama2_13b_swiglu_bf16", 0.2), ("opt66b_relu_f16_8sent", 0.4)])
def test_full_size_layer_hidden_ranked(lib, name, beta):
    """The prefill pass without fp32 scores at the workload's full layer shape (for the OPT-66B
    shape all eight prompts as one matrix, selection on the first prompt's rows): selection
    bit-exact against the oracle ranking the hidden values; H sampled against the oracle."""
    cfg = wl.WORKLOADS[name]
    _say("full-size hidden-ranked layer", name)
    w = wl.layer_weights(cfg, 0, DEV)
    X = torch.cat([wl.prefill_hidden(cfg, 0, DEV, sentence=s) for s in range(cfg.sentences)], dim=0).contiguous()
    Y, H = lib.ffn_dense_hidden(X, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], cfg.down_layout,
                                cfg.act)
    Hs = H[:cfg.M]
    S, counts = lib.select_hidden(Hs, cfg.act, cfg.alpha, beta)
    torch.cuda.synchronize()
    ranked = f64(Hs) if cfg.act == "relu" else np.abs(f64(Hs))
    S_ref, c_ref = orc.select(ranked, cfg.alpha, beta)
    assert counts.cpu().numpy().tolist() == c_ref.tolist()
    assert S.cpu().numpy().tolist() == S_ref.tolist()
    # What ranking the 16-bit hidden values instead of the fp32 scores costs: the similarity of
    # Insight-2 (Sec. 3.2) between the two core sets of the same prompt (the rounding merges
    # neighbouring scores, which moves neurons at the Def. 1 and Def. 2 boundaries).
    _, A32 = lib.ffn_dense(X[:cfg.M].contiguous(), w["w_up"], w["w_gate"], w["b_up"], None, None, cfg.down_layout,
                           cfg.act, want_y=False, want_a=True)
    S32, _ = lib.select(A32, cfg.alpha, beta)
    torch.cuda.synchronize()
    sim = orc.core_similarity(S32.cpu().numpy(), S_ref)
    _say(f"  hidden-ranked vs fp32-ranked core set of layer 0, first prompt: similarity {sim:.4f} "
         f"({len(set(S32.cpu().numpy().tolist()) - set(S_ref.tolist()))} of {len(S_ref)} neurons differ)")
    assert sim >= 0.9
    del A32
    # sampled rows and columns of H against the oracle's hidden state
    rng = np.random.default_rng(4)
    rows = np.unique(rng.integers(0, X.shape[0], size=6))
    cols = np.unique(rng.integers(0, cfg.N, size=512))
    ct = torch.from_numpy(cols).to(DEV)
    Xs = f64(X[torch.from_numpy(rows).to(DEV)])
    Wu = f64(w["w_up"][ct])
    if cfg.act == "relu":
        H_ref = orc.score_relu(Xs, Wu, f64(w["b_up"][ct]))
    else:
        H_ref = orc.hidden_swiglu(Xs, f64(w["w_gate"][ct]), Wu)
    got = f64(H[torch.from_numpy(rows).to(DEV)][:, ct])
    ulp = 2.0 ** -11 if cfg.dtype == "f16" else 2.0 ** -8
    assert np.all(np.abs(got - H_ref) <= ulp * np.abs(H_ref) * 1.01 + 2e-5 * np.sqrt(np.mean(H_ref ** 2)) + 1e-7)


def test_full_size_layer_gathered_eight_sentences(lib):
    """OPT-66B-shaped layer, eight sentences with their own core sets, rows
    gathered from the resident weights (four of the sentences checked on the CPU)."""
    cfg = wl.WORKLOADS["opt66b_relu_f16_8sent"]
    _say("full-size gathered layer", cfg.name)
    w = wl.layer_weights(cfg, 0, DEV)
    sets = []
    for s in range(cfg.sentences):
        X = wl.prefill_hidden(cfg, 0, DEV, sentence=s)
        _, A = lib.ffn_dense(X, w["w_up"], None, w["b_up"], None, None, cfg.down_layout, "relu",
                             want_y=False, want_a=True)
        S, counts = lib.select(A, cfg.alpha, cfg.betas[0])
        if s in (0, 3, 5, 7):
            S_ref, c_ref = orc.select(A.cpu().numpy(), cfg.alpha, cfg.betas[0])
            assert counts.cpu().numpy().tolist() == c_ref.tolist()
            assert S.cpu().numpy().tolist() == S_ref.tolist() and len(S_ref) == 14746
        sets.append(S)
        del A, X
    idx = torch.stack(sets).contiguous()
    x = torch.stack([wl.decode_hidden(cfg, 0, DEV, sentence=s, tokens=1)[0] for s in range(cfg.sentences)])
    desc = lib.make_weights(w["w_up"], None, w["b_up"], w["w_down"], w["b_down"], core_idx=idx)
    y = lib.ffn_decode(x, desc, "relu")
    # the same batch through the union of the eight sets
    uidx, umask, ucount = lib.union_build(idx, cfg.N)
    yu = lib.ffn_decode_union(x, lib.make_weights(w["w_up"], None, w["b_up"], w["w_down"], w["b_down"]),
                              uidx, umask, ucount, "relu")
    torch.cuda.synchronize()
    U_ref, owners_ref = orc.union_rows([t.cpu().numpy() for t in sets], cfg.N)
    n_rows = int(ucount.item())
    assert n_rows == U_ref.size
    assert uidx[:n_rows].cpu().numpy().tolist() == U_ref.tolist()
    assert (umask[:n_rows].cpu().numpy().astype(np.int64) & 0xffffffff).tolist() == owners_ref.astype(np.int64).tolist()
    _say(f"  union of 8 sets: {n_rows} of {cfg.N} neurons")
    for s in (0, 3, 5, 7):
        Sn = sets[s].cpu().numpy().astype(np.int64)
        up_rows = f64(w["w_up"][sets[s].long()])
        down_rows = f64(w["w_down"][sets[s].long()])          # neuron-major rows
        # the oracle proper, fed the pre-gathered rows as a dense layer (bounds host memory:
        # the full fp64 matrices would take 5.4 GB); indexing by S is what its own S path does
        y_ref = orc.ffn_relu(f64(x[s]), None, up_rows, f64(w["b_up"])[Sn], down_rows.T, f64(w["b_down"]))
        rel = assert_close_rms(y[s], y_ref, torch.float16, f"gathered sentence {s}")
        _say(f"  sentence {s}: max err / rms = {rel:.2e}")
        rel = assert_close_rms(yu[s], y_ref, torch.float16, f"union-batched sentence {s}")
        _say(f"  sentence {s}, union-batched: max err / rms = {rel:.2e}")


# ------------------------------------------------ union-batched decode (next row)

def _random_sets(rng, B, K, N, overlap):
    """B index lists of length K; `overlap` in [0, 1] draws that share from a common pool."""
    pool = rng.choice(N, size=min(N, max(K, 1)), replace=False)
    out = []
    for _ in range(B):
        k_common = int(round(overlap * K))
        a = rng.choice(pool, size=k_common, replace=False) if k_common else np.zeros(0, dtype=np.int64)
        rest = np.setdiff1d(np.arange(N), a)
        b = rng.choice(rest, size=K - k_common, replace=False)
        S = np.concatenate([a, b])
        rng.shuffle(S)
        out.append(S)
    return np.stack(out) if K else np.zeros((B, 0), dtype=np.int64)


@pytest.mark.parametrize("B,K,N,overlap", [(1, 7, 40, 0.0), (3, 100, 300, 0.5), (8, 410, 1024, 0.0),
                                           (8, 2000, 5000, 0.9), (5, 0, 64, 0.0), (2, 3000, 3000, 1.0),
                                           (4, 30000, 150000, 0.5), (2, 1025, 1 << 20, 0.0)])
def test_union_build_matches_oracle(lib, B, K, N, overlap):
    _say("union build case", B, K, N, overlap)
    S = _random_sets(np.random.default_rng(B * 31 + K), B, K, N, overlap)
    if K >= 7:  # out-of-range entries and a duplicate are ignored / harmless
        S[0, 1], S[B - 1, 2], S[0, 4] = -3, N + 5, S[0, 5]
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    uidx, umask, ucount = lib.union_build(idx, N)
    torch.cuda.synchronize()
    U_ref, owners_ref = orc.union_rows(list(S), N)
    n_rows = int(ucount.item())
    assert n_rows == U_ref.size
    assert uidx[:n_rows].cpu().numpy().tolist() == U_ref.tolist()
    assert (umask[:n_rows].cpu().numpy().astype(np.int64) & 0xffffffff).tolist() == owners_ref.astype(np.int64).tolist()


@pytest.mark.parametrize("dt,act", [("f16", "relu"), ("bf16", "swiglu"), ("f32", "relu"), ("f32", "swiglu")])
@pytest.mark.parametrize("d,N,K,B,overlap", [(512, 2000, 801, 4, 0.3), (9216, 1200, 480, 8, 0.0),
                                             (4352, 900, 300, 5, 0.8), (64, 64, 64, 1, 0.0),
                                             (1000, 700, 33, 8, 0.0), (256, 3000, 1500, 2, 1.0)])
def test_decode_union_matches_oracle_and_gathered(lib, dt, act, d, N, K, B, overlap):
    _say("decode union case", dt, act, d, N, K, B, overlap)
    dtype = DTYPES[dt]
    w = rand_weights(d, N, dtype, act, "neuron_major", seed=d + N + 1, device=DEV)
    S = np.sort(_random_sets(np.random.default_rng(B * 100 + K + 7), B, K, N, overlap), axis=1)
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    x = torch.randn(B, d, generator=torch.Generator().manual_seed(K + 3)).to(dtype).to(DEV)
    uidx, umask, ucount = lib.union_build(idx, N)
    resident = lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"])
    y = lib.ffn_decode_union(x, resident, uidx, umask, ucount, act)
    y2 = lib.ffn_decode_union(x, resident, uidx, umask, ucount, act)
    yg = lib.ffn_decode(x, lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"],
                                            core_idx=idx), act)
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "union-batched decode must be deterministic"
    for b in range(B):
        ref = _oracle_ffn(act, x[b], S[b], w, "neuron_major")
        assert_close_rms(y[b], ref, dtype, f"union b={b}")
        assert_close_rms(yg[b], ref, dtype, f"gathered b={b}")


@pytest.mark.parametrize("dt,act", [("f16", "relu"), ("bf16", "swiglu")])
def test_decode_union_several_drains_per_slice(lib, dt, act):
    """Slices longer than the rows handled between two drains of the load ring (forced small through the
    development hook): equal parts with a ragged last one; the result does not depend on the split."""
    d, N, K, B = 320, 12000, 5000, 3
    dtype = DTYPES[dt]
    _say("union drains case", dt, act, d, N, K, B)
    w = rand_weights(d, N, dtype, act, "neuron_major", seed=77, device=DEV)
    S = np.sort(_random_sets(np.random.default_rng(91), B, K, N, 0.2), axis=1)
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    x = torch.randn(B, d, generator=torch.Generator().manual_seed(4)).to(dtype).to(DEV)
    uidx, umask, ucount = lib.union_build(idx, N)
    resident = lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"])
    y_default = lib.ffn_decode_union(x, resident, uidx, umask, ucount, act)
    torch.cuda.synchronize()
    assert int(ucount.item()) > 256 * 17  # every slice of the up phase has more than 16 rows
    try:
        for cap in (16, 23):
            lib.dev_set_param("union_super", cap)
            y = lib.ffn_decode_union(x, resident, uidx, umask, ucount, act)
            torch.cuda.synchronize()
            assert torch.equal(y, y_default), f"rows between drains capped at {cap}"
    finally:
        lib.dev_set_param("union_super", 0)
    for b in range(B):
        assert_close_rms(y_default[b], _oracle_ffn(act, x[b], S[b], w, "neuron_major"), dtype, f"union b={b}")


def test_decode_union_empty_sets_give_the_output_bias(lib):
    d, N, B = 128, 256, 3
    w = rand_weights(d, N, torch.float16, "relu", "neuron_major", seed=5, device=DEV)
    idx = torch.full((B, 4), -1, dtype=torch.int32, device=DEV)   # no valid entry at all
    uidx, umask, ucount = lib.union_build(idx, N)
    x = torch.randn(B, d).half().to(DEV)
    y = lib.ffn_decode_union(x, lib.make_weights(w["w_up"], None, w["b_up"], w["w_down"], w["b_down"]),
                             uidx, umask, ucount, "relu")
    torch.cuda.synchronize()
    assert int(ucount.item()) == 0
    for b in range(B):
        assert torch.equal(y[b], w["b_down"])


# ------------------------------------------------------------ the documented size limits

def test_select_at_the_size_limits(lib):
    """N = CI_MAX_NEURONS with two tokens, and M = CI_MAX_TOKENS (counts up to 65535) on a narrow layer."""
    A = wl.activation_like(2, 1 << 20, seed=77, kind="relu", levels=0)
    _select_case(lib, A, 0.2, 0.4, "N at its limit")
    A = wl.activation_like(65535, 48, seed=78, kind="relu", levels=4)
    _select_case(lib, A, 0.25, 0.5, "M at its limit")


@pytest.mark.parametrize("dt,act", [("f16", "relu"), ("bf16", "swiglu")])
def test_decode_and_dense_at_the_model_width_limit(lib, dt, act):
    """d = CI_MAX_DMODEL: four 16-byte vectors per thread in the decode kernels."""
    d, N, K = 32768, 200, 71
    dtype = DTYPES[dt]
    _say("width limit", dt, act, d, N, K)
    w = rand_weights(d, N, dtype, act, "neuron_major", seed=3, device=DEV)
    S = np.stack([np.sort(np.random.default_rng(5 + b).choice(N, size=K, replace=False)) for b in range(2)])
    idx = torch.from_numpy(S.astype(np.int32)).to(DEV)
    x = (torch.randn(2, d, generator=torch.Generator().manual_seed(2)) * 0.05).to(dtype).to(DEV)
    yg = lib.ffn_decode(x, lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"],
                                            core_idx=idx), act)
    c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], "neuron_major", act, idx[0].contiguous())
    yc = lib.ffn_decode(x[:1], lib.make_weights(c["w_up_c"], c["w_gate_c"], c["b_up_c"], c["w_down_c"], w["b_down"]), act)
    uidx, umask, ucount = lib.union_build(idx, N)
    yu = lib.ffn_decode_union(x, lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"]),
                              uidx, umask, ucount, act)
    Yd, _ = lib.ffn_dense(x, w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], "neuron_major", act)
    torch.cuda.synchronize()
    for b in range(2):
        ref = _oracle_ffn(act, x[b], S[b], w, "neuron_major")
        assert_close_rms(yg[b], ref, dtype, f"gathered, widest model, b={b}")
        assert_close_rms(yu[b], ref, dtype, f"union-batched, widest model, b={b}")
        assert_close_rms(Yd[b], _oracle_ffn(act, x[b], None, w, "neuron_major"), dtype, f"dense, widest model, b={b}")
    assert_close_rms(yc[0], _oracle_ffn(act, x[0], S[0], w, "neuron_major"), dtype, "compacted, widest model")


# --------------------------------- running counts, group sets, similarity (next rows)

def test_running_counts_and_count_select_match_oracle(lib):
    A_np = wl.activation_like(300, 5000, seed=21, kind="relu", levels=16)
    A = torch.from_numpy(A_np).to(DEV)
    counts = lib.count_tokens(A[:100].contiguous(), 0.2)
    lib.count_tokens(A[100:101].contiguous(), 0.2, counts=counts, accumulate=True)
    lib.count_tokens(A[101:].contiguous(), 0.2, counts=counts, accumulate=True)
    S = lib.count_select(counts, 300, 0.4)
    S_all, c_all = lib.select(A, 0.2, 0.4)
    torch.cuda.synchronize()
    ref = np.zeros(5000, dtype=np.int64)
    for lo, hi in ((0, 100), (100, 101), (101, 300)):
        ref = orc.count_tokens_into(ref, A_np[lo:hi], 0.2)
    assert counts.cpu().numpy().tolist() == ref.tolist()
    assert S.cpu().numpy().tolist() == orc.sentence_core_neurons(ref, 0.4).tolist()
    assert torch.equal(S, S_all) and torch.equal(counts, c_all)
    # count_select on arbitrary counts, small and large bounds, huge tie classes
    rng = np.random.default_rng(3)
    for N, mx, beta in ((1000, 3, 0.5), (16384, 255, 0.4), (16384, 256, 0.4), (40000, 65535, 0.1), (7, 1, 1.0)):
        c = rng.integers(0, mx + 1, size=N).astype(np.int32)
        got = lib.count_select(torch.from_numpy(c).to(DEV), mx, beta)
        torch.cuda.synchronize()
        assert got.cpu().numpy().tolist() == orc.sentence_core_neurons(c, beta).tolist(), (N, mx, beta)


@pytest.mark.parametrize("G,K,N,gamma", [(1, 5, 40, 0.2), (12, 410, 1024, 0.2), (50, 6554, 16384, 0.4), (300, 100, 3000, 0.05)])
def test_group_select_matches_oracle(lib, G, K, N, gamma):
    _say("group select case", G, K, N, gamma)
    rng = np.random.default_rng(G + K)
    # sentences of one semantic group share most of their core neurons
    base = rng.choice(N, size=K, replace=False)
    sets = []
    for _ in range(G):
        s = base.copy()
        swap = rng.random(K) < 0.3
        s[swap] = rng.choice(N, size=int(swap.sum()), replace=False)
        sets.append(np.unique(np.concatenate([s, rng.choice(N, size=K, replace=False)]))[:K])
    sets_np = np.stack([np.sort(rng.permutation(s)) for s in sets]).astype(np.int32)
    S, counts = lib.group_select(torch.from_numpy(sets_np).to(DEV), N, gamma)
    torch.cuda.synchronize()
    S_ref, c_ref = orc.group_core_neurons(sets_np, N, gamma)
    assert counts.cpu().numpy().tolist() == c_ref.tolist()
    assert S.cpu().numpy().tolist() == S_ref.tolist()


def test_core_similarity_matches_oracle(lib):
    rng = np.random.default_rng(17)
    for N, Ka, Kb in ((100, 0, 0), (100, 10, 0), (16384, 6554, 6554), (36864, 14746, 9000), (50, 50, 50)):
        a = np.sort(rng.choice(N, size=Ka, replace=False)).astype(np.int32)
        b = np.sort(rng.choice(N, size=Kb, replace=False)).astype(np.int32)
        out = lib.core_similarity(torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV))
        torch.cuda.synchronize()
        assert tuple(out.cpu().numpy().tolist()) == orc.core_similarity_counts(a, b), (N, Ka, Kb)


@pytest.mark.parametrize("G,K,Kg,N", [(1, 5, 5, 40), (4, 410, 410, 1024), (37, 6554, 3277, 16384), (1500, 20, 30, 300)])
def test_assign_group_matches_oracle(lib, G, K, Kg, N):
    rng = np.random.default_rng(G * 7 + K)
    prompt = np.sort(rng.choice(N, size=K, replace=False))
    groups = np.stack([np.sort(rng.choice(N, size=Kg, replace=False)) for _ in range(G)])
    if G >= 4:                       # two groups with exactly the same similarity: the lower index wins
        groups[G - 1] = groups[1]
    best, iu = lib.assign_group(torch.from_numpy(prompt.astype(np.int32)).to(DEV),
                                torch.from_numpy(groups.astype(np.int32)).to(DEV))
    torch.cuda.synchronize()
    g_ref, pairs = orc.assign_group(prompt, list(groups))
    assert iu.cpu().numpy().tolist() == [list(p) for p in pairs]
    assert int(best.item()) == g_ref


@pytest.mark.parametrize("M,N,G,ld_pad", [(1, 1, 1, 0), (5, 64, 3, 0), (37, 1000, 9, 3), (256, 16384, 40, 0),
                                          (700, 4100, 300, 0), (64, 36864, 2, 8), (130, 257, 1500, 1)])
def test_assign_centroid_matches_oracle(lib, M, N, G, ld_pad):
    """Feature vector and squared distances within fp32 summation error of the fp64 oracle; the
    chosen group is the oracle's whenever the oracle's margin exceeds that error, and in any
    case a group whose distance is within it of the smallest."""
    _say("assign centroid case", M, N, G, ld_pad)
    rng = np.random.default_rng(M + N + G)
    centers = rng.standard_normal((G, N)).astype(np.float32) * 0.5
    own = int(rng.integers(0, G))
    A = np.maximum(centers[own] + rng.standard_normal((M, N)).astype(np.float32), 0).astype(np.float32)
    if G >= 3:
        centers[(own + 1) % G] = centers[own]            # an exact duplicate: the lower index must win
    buf = torch.zeros(M, N + ld_pad, dtype=torch.float32, device=DEV)
    buf[:, :N] = torch.from_numpy(A).to(DEV)
    best, dist, feat = lib.assign_centroid(buf[:, :N], torch.from_numpy(centers).to(DEV))
    torch.cuda.synchronize()
    f_ref = orc.sentence_feature(A)
    g_ref, d_ref = orc.assign_centroid(f_ref, centers)
    scale = max(float(np.max(np.abs(f_ref))), 1e-30)
    assert np.max(np.abs(f64(feat) - f_ref)) <= 2e-6 * scale * max(1.0, np.sqrt(M) / 8)
    tol = 2e-5 * max(float(np.max(d_ref)), 1e-30)
    assert np.max(np.abs(f64(dist) - d_ref)) <= tol
    g = int(best.item())
    assert 0 <= g < G and d_ref[g] <= d_ref[g_ref] + 2 * tol
    others = np.delete(d_ref, g_ref)
    if others.size == 0 or np.min(others) > d_ref[g_ref] + 2 * tol:
        assert g == g_ref
    # the decision itself is taken in the kernel's precision: the oracle's rule (smallest distance,
    # lower index among equal ones) on the kernel's fp32 distances, held exactly in float64 on the host
    assert g == orc.nearest_group(f64(dist))


def test_decode_graph_replays_match_eager(lib):
    """The decode launches captured in a HIP graph give the eager result on every replay,
    with other work and synchronisations in between."""
    d, N, K = 1024, 3000, 1201
    w = rand_weights(d, N, torch.float16, "relu", "out_major", seed=5, device=DEV)
    S = np.sort(np.random.default_rng(1).choice(N, size=K, replace=False))
    c = lib.compact(w["w_up"], None, w["b_up"], w["w_down"], "out_major", "relu",
                    torch.from_numpy(S.astype(np.int32)).to(DEV))
    desc = lib.make_weights(c["w_up_c"], None, c["b_up_c"], c["w_down_c"], w["b_down"])
    x = torch.randn(1, d, generator=torch.Generator().manual_seed(2)).half().to(DEV)
    y = torch.empty_like(x)
    ws = lib.decode_workspace(1, K, d, DEV)
    lib.ffn_decode(x, desc, "relu", y=y, ws=ws)
    torch.cuda.synchronize()
    eager = y.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        lib.ffn_decode(x, desc, "relu", y=y, ws=ws)
    for i in range(4):
        y.zero_()
        ws.fill_(0xFF)                               # stale scratch must not matter
        (torch.randn(256, 256, device=DEV) @ torch.randn(256, 256, device=DEV)).sum().item()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager), f"replay {i}"
    # new input through the same graph
    x.copy_(torch.randn(1, d, generator=torch.Generator().manual_seed(3)).half())
    g.replay()
    torch.cuda.synchronize()
    assert_close_rms(y[0], _oracle_ffn("relu", x[0], S, w, "out_major"), torch.float16, "graph, new input")


def test_prefill_graph_replays_match_eager(lib):
    """Dense FFN, selection, deployment and the union build captured in one HIP graph: every replay
    gives the eager result, with stale workspaces and other work in between (nothing in these
    paths relies on memory being cleared outside the captured kernels)."""
    M, d, N, B = 96, 256, 1536, 3
    dt = torch.float16
    w = rand_weights(d, N, dt, "relu", "neuron_major", seed=11, device=DEV)
    X = torch.randn(M, d, generator=torch.Generator().manual_seed(4)).to(dt).to(DEV)
    K = lib.keep_count(0.3, N)
    A = torch.empty(M, N, dtype=torch.float32, device=DEV)
    Y = torch.empty(M, d, dtype=dt, device=DEV)
    dws = torch.empty(lib.ffn_dense_workspace_size(M, d, N, dt), dtype=torch.uint8, device=DEV)
    sws = torch.empty(lib.select_workspace_size(M, N), dtype=torch.uint8, device=DEV)
    idx = torch.empty(K, dtype=torch.int32, device=DEV)
    cnt = torch.empty(N, dtype=torch.int32, device=DEV)
    bufs = lib.compact(w["w_up"], None, w["b_up"], w["w_down"], "neuron_major", "relu",
                       torch.arange(K, dtype=torch.int32, device=DEV))
    sets = torch.stack([torch.sort(torch.randperm(N, generator=torch.Generator().manual_seed(s))[:K]).values
                        for s in range(B)]).to(torch.int32).to(DEV)
    import ctypes
    need = ctypes.c_size_t(0)
    lib._check(lib.raw.coreinfer_union_workspace_size(N, ctypes.byref(need)), "union_workspace_size")
    uws = torch.empty(need.value, dtype=torch.uint8, device=DEV)
    uidx = torch.empty(N, dtype=torch.int32, device=DEV)
    umask = torch.empty(N, dtype=torch.int32, device=DEV)
    ucount = torch.empty(1, dtype=torch.int32, device=DEV)

    Hh = torch.empty(M, N, dtype=dt, device=DEV)
    Yh = torch.empty(M, d, dtype=dt, device=DEV)
    idx_h = torch.empty(K, dtype=torch.int32, device=DEV)
    cnt_h = torch.empty(N, dtype=torch.int32, device=DEV)
    sws_h = torch.empty(lib.select_workspace_size(M, N), dtype=torch.uint8, device=DEV)

    def run():
        lib.ffn_dense_hidden(X, w["w_up"], None, w["b_up"], w["w_down"], w["b_down"], "neuron_major", "relu",
                             Y=Yh, H=Hh, ws=dws)
        lib.select_hidden(Hh, "relu", 0.2, 0.3, core_idx=idx_h, counts=cnt_h, ws=sws_h)
        lib.ffn_dense(X, w["w_up"], None, w["b_up"], w["w_down"], w["b_down"], "neuron_major", "relu",
                      want_y=True, want_a=True, Y=Y, A=A, ws=dws)
        lib.select(A, 0.2, 0.3, core_idx=idx, counts=cnt, ws=sws)
        lib.compact(w["w_up"], None, w["b_up"], w["w_down"], "neuron_major", "relu", idx, out=bufs)
        lib._check(lib.raw.coreinfer_union_build(sets.data_ptr(), B, K, N, N, uidx.data_ptr(), umask.data_ptr(),
                                                 ucount.data_ptr(), uws.data_ptr(), uws.numel(),
                                                 torch.cuda.current_stream().cuda_stream), "union_build")

    run()
    torch.cuda.synchronize()
    S_ref, c_ref = orc.select(A.cpu().numpy(), 0.2, 0.3)
    assert idx.cpu().numpy().tolist() == S_ref.tolist() and cnt.cpu().numpy().tolist() == c_ref.tolist()
    Sh_ref, ch_ref = orc.select(f64(Hh), 0.2, 0.3)
    assert idx_h.cpu().numpy().tolist() == Sh_ref.tolist() and cnt_h.cpu().numpy().tolist() == ch_ref.tolist()
    want_h = {"idx": idx_h.clone(), "cnt": cnt_h.clone(), "H": Hh.clone(), "Y": Yh.clone()}
    want = {"idx": idx.clone(), "cnt": cnt.clone(), "up": bufs["w_up_c"].clone(), "down": bufs["w_down_c"].clone(),
            "Y": Y.clone(), "uidx": uidx[:int(ucount.item())].clone(), "un": int(ucount.item())}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for i in range(3):
        for t in (dws, sws, uws, sws_h):
            t.fill_(0xA5)                                # stale scratch must not matter
        for t in (idx_h, cnt_h):
            t.fill_(-7)
        Hh.zero_(); Yh.zero_()
        for t in (idx, cnt, uidx, ucount):
            t.fill_(-7)
        bufs["w_up_c"].zero_(); bufs["w_down_c"].zero_(); Y.zero_()
        (torch.randn(128, 128, device=DEV) @ torch.randn(128, 128, device=DEV)).sum().item()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, want["idx"]) and torch.equal(cnt, want["cnt"]), f"replay {i}: selection"
        assert torch.equal(bufs["w_up_c"], want["up"]) and torch.equal(bufs["w_down_c"], want["down"]), f"replay {i}"
        assert torch.equal(Y, want["Y"]), f"replay {i}: dense output"
        assert torch.equal(idx_h, want_h["idx"]) and torch.equal(cnt_h, want_h["cnt"]), f"replay {i}: selection on H"
        assert torch.equal(Hh, want_h["H"]) and torch.equal(Yh, want_h["Y"]), f"replay {i}: hidden pass"
        assert int(ucount.item()) == want["un"] and torch.equal(uidx[:want["un"]], want["uidx"]), f"replay {i}: union"
