"""Pins for the CPU oracle: it is checked here against things other than
itself -- hand-worked examples, brute force by repeated arg-max, closed forms,
invariants that follow from the paper's definitions, and library routines
(torch CPU float64) for the special cases that reduce to them."""

import itertools
import math

import numpy as np
import pytest
import torch

from oracle import coreinfer_oracle as orc
from tests._golden import read_hand_examples


# ---------------------------------------------------------------- keep_count

def test_keep_count_values_quoted_for_the_workloads():
    # K for the five benchmark shapes (beta * d_ff rounded up), as tabulated
    # with the workloads: 0.4*1024 = 409.6, 0.4*16384 = 6553.6, ...
    assert orc.keep_count(0.4, 1024) == 410
    assert orc.keep_count(0.4, 16384) == 6554
    assert orc.keep_count(0.4, 11008) == 4404
    assert [orc.keep_count(b, 13824) for b in (0.2, 0.3, 0.4, 0.6)] == [2765, 4148, 5530, 8295]
    assert orc.keep_count(0.4, 36864) == 14746


def test_keep_count_closed_forms():
    assert orc.keep_count(1.0, 17) == 17
    assert orc.keep_count(0.5, 0) == 0
    assert orc.keep_count(0.5, 1) == 1            # at least one when n >= 1
    assert orc.keep_count(0.1, 30) == 3           # 0.1 * 30 = 3.0000000000000004 in floats
    assert orc.keep_count(0.3, 10) == 3
    assert orc.keep_count(0.7, 10) == 7
    for n in range(0, 200):
        for f in (0.01, 0.2, 0.25, 1 / 3, 0.4, 0.999, 1.0):
            k = orc.keep_count(f, n)
            q = round(f * 10**6)
            assert k * 10**6 >= q * n and (k - 1) * 10**6 < q * n or (n == 0 and k == 0)
            assert 0 <= k <= n
    with pytest.raises(ValueError):
        orc.keep_count(0.0, 5)
    with pytest.raises(ValueError):
        orc.keep_count(1.5, 5)
    with pytest.raises(ValueError):
        orc.keep_count(float("nan"), 5)


# ------------------------------------------------------------ hand examples

@pytest.mark.parametrize("name", ["example1", "example2", "example3"])
def test_hand_worked_examples(name):
    ex = read_hand_examples()[name]
    A, alpha, beta = ex["A"], ex["alpha"], ex["beta"]
    for m, want in enumerate(ex["token_sets"]):
        assert orc.token_core_neurons(A[m], alpha).tolist() == want
    S, counts = orc.select(A, alpha, beta)
    assert counts.tolist() == ex["counts"]
    assert S.tolist() == ex["S"]
    # the literal ">= percentile" reading keeps ties and differs where stated
    for m, want in enumerate(ex["token_sets_threshold"]):
        assert sorted(orc.token_core_neurons(A[m], alpha, rule="threshold").tolist()) == sorted(want)
    S_t, counts_t = orc.select(A, alpha, beta, rule="threshold")
    assert counts_t.tolist() == ex["counts_threshold"]
    assert S_t.tolist() == ex["S_threshold"]


def test_hand_example_alpha_base_readings_differ():
    ex = read_hand_examples()["example3"]
    got = orc.token_core_neurons(ex["A"][0], ex["alpha"], base="all").tolist()
    assert got == [0, 4, 2]        # ceil(0.34 * 8) = 3, capped by the 3 positives


# ------------------------------------------------- brute force on tiny inputs

def _brute_token_set(a, k):
    """k rounds of 'take the largest remaining positive value, lowest index
    among equals' -- no sort involved."""
    a = [float(v) for v in a]
    taken = []
    for _ in range(k):
        best = None
        for n, v in enumerate(a):
            if n in taken or not (v > 0.0):
                continue
            if best is None or v > a[best]:
                best = n
        assert best is not None
        taken.append(best)
    return taken


def _brute_sentence_set(counts, K):
    counts = [int(c) for c in counts]
    taken = []
    for _ in range(K):
        best = None
        for n, c in enumerate(counts):
            if n in taken:
                continue
            if best is None or c > counts[best]:
                best = n
        taken.append(best)
    return sorted(taken)


@pytest.mark.parametrize("seed", range(12))
def test_selection_matches_brute_force(seed):
    rng = np.random.default_rng(1000 + seed)
    M, N = int(rng.integers(1, 9)), int(rng.integers(1, 40))
    alpha = float(rng.choice([0.05, 0.2, 0.34, 0.5, 0.9, 1.0]))
    beta = float(rng.choice([0.1, 0.25, 0.4, 0.77, 1.0]))
    A = rng.standard_normal((M, N))
    if seed % 3 == 0:                       # heavy ties
        A = np.round(A * 2) / 2
    if seed % 4 == 1:
        A[rng.integers(0, M), rng.integers(0, N)] = np.nan
        A[rng.integers(0, M), rng.integers(0, N)] = np.inf
    counts = np.zeros(N, dtype=int)
    for m in range(M):
        P = sum(1 for v in A[m] if v > 0)
        k = 0 if P == 0 else math.ceil(round(alpha * 10**6) * P / 10**6 - 1e-12)
        want = _brute_token_set(A[m], k)
        got = orc.token_core_neurons(A[m], alpha).tolist()
        assert got == want
        for n in want:
            counts[n] += 1
    S, got_counts = orc.select(A, alpha, beta)
    assert got_counts.tolist() == counts.tolist()
    K = math.ceil(round(beta * 10**6) * N / 10**6 - 1e-12)
    assert S.tolist() == _brute_sentence_set(counts, K)


def test_exhaustive_three_level_rows():
    # every row over {-1, 0, 1, 2}^5: selected = the k largest positives, lowest index on ties
    for row in itertools.product([-1.0, 0.0, 1.0, 2.0], repeat=5):
        a = np.array(row)
        P = int((a > 0).sum())
        for alpha in (0.3, 0.5, 1.0):
            k = 0 if P == 0 else -((-round(alpha * 10**6) * P) // 10**6)
            assert orc.token_core_neurons(a, alpha).tolist() == _brute_token_set(a, k)


# ------------------------------------------------------------------ invariants

@pytest.mark.parametrize("kind,levels", [("relu", 0), ("abs", 0), ("raw", 0), ("relu", 6), ("abs", 3)])
def test_token_and_count_invariants(kind, levels):
    from paper_2410_18311_amd.workloads import activation_like
    M, N, alpha, beta = 24, 193, 0.2, 0.4
    A = activation_like(M, N, seed=7, kind=kind, levels=levels)
    counts = np.zeros(N, dtype=int)
    total = 0
    for m in range(M):
        C = orc.token_core_neurons(A[m], alpha)
        P = int((A[m] > 0).sum())
        assert len(C) == orc.keep_count(alpha, P) and len(set(C.tolist())) == len(C)
        assert np.all(A[m][C] > 0)
        rest = np.setdiff1d(np.flatnonzero(A[m] > 0), C)
        if len(C) and len(rest):
            lo = A[m][C].min()
            assert lo >= A[m][rest].max()
            # among the boundary value, the chosen ones are the lowest indices
            tied_in = C[A[m][C] == lo]
            tied_out = rest[A[m][rest] == lo]
            if len(tied_out):
                assert tied_in.max() < tied_out.min()
        counts[C] += 1
        total += len(C)
    S, got = orc.select(A, alpha, beta)
    assert got.tolist() == counts.tolist()
    assert got.sum() == total and got.min() >= 0 and got.max() <= M
    # positive scaling leaves every set unchanged
    S2, got2 = orc.select(A * 3.5, alpha, beta)
    assert S2.tolist() == S.tolist() and got2.tolist() == got.tolist()
    # token order is irrelevant (Eq. 3 is a sum over tokens)
    perm = np.random.default_rng(3).permutation(M)
    S3, got3 = orc.select(A[perm], alpha, beta)
    assert S3.tolist() == S.tolist() and got3.tolist() == got.tolist()
    # concatenating two sentences adds their count sets
    c1 = orc.count_set(A[:10], alpha)
    c2 = orc.count_set(A[10:], alpha)
    assert (c1 + c2).tolist() == got.tolist()


def test_sentence_set_invariants_and_nesting():
    rng = np.random.default_rng(11)
    N, M = 500, 40
    counts = rng.integers(0, M + 1, size=N)
    counts[rng.integers(0, N, size=200)] = 0
    prev = None
    for beta in (0.05, 0.2, 0.3, 0.4, 0.6, 0.99, 1.0):
        S = orc.sentence_core_neurons(counts, beta)
        K = orc.keep_count(beta, N)
        assert len(S) == K and np.all(np.diff(S) > 0)
        out = np.setdiff1d(np.arange(N), S)
        if len(out):
            lo = counts[S].min()
            assert lo >= counts[out].max()
            tied_out = out[counts[out] == lo]
            tied_in = S[counts[S] == lo]
            if len(tied_out):
                assert tied_in.max() < tied_out.min()
        if prev is not None:
            assert set(prev.tolist()) <= set(S.tolist())      # S_beta1 within S_beta2
        prev = S
    assert orc.sentence_core_neurons(counts, 1.0).tolist() == list(range(N))


def test_alpha_one_counts_positive_tokens():
    from paper_2410_18311_amd.workloads import activation_like
    A = activation_like(17, 80, seed=5, kind="relu")
    assert orc.count_set(A, 1.0).tolist() == (A > 0).sum(axis=0).tolist()


def test_never_positive_neuron_has_zero_count_and_nan_is_skipped():
    A = np.abs(np.random.default_rng(2).standard_normal((6, 10)))
    A[:, 4] = 0.0
    A[:, 7] = -1.0
    A[2, 3] = np.nan
    c = orc.count_set(A, 1.0)
    assert c[4] == 0 and c[7] == 0 and c[3] == 5
    A[1, 0] = np.inf
    assert orc.token_core_neurons(A[1], 0.01).tolist() == [0]


def test_core_similarity_hand_values():
    assert orc.core_similarity([0, 1, 2], [1, 2, 3]) == 0.5
    assert orc.core_similarity([5, 6], [5, 6]) == 1.0
    assert orc.core_similarity([1], [2]) == 0.0


# ----------------------------------------------------------------------- FFN

def _rand_ffn(seed, d=7, N=13, B=3):
    rng = np.random.default_rng(seed)
    return dict(
        x=rng.standard_normal((B, d)), W_up=rng.standard_normal((N, d)) * 0.3,
        W_gate=rng.standard_normal((N, d)) * 0.3, b_up=rng.standard_normal(N) * 0.1,
        W_down=rng.standard_normal((d, N)) * 0.3, b_down=rng.standard_normal(d) * 0.1)


def test_silu_against_library_and_identities():
    z = np.linspace(-9, 9, 181)
    want = torch.nn.functional.silu(torch.from_numpy(z)).numpy()
    np.testing.assert_allclose(orc.silu(z), want, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(orc.silu(z) - orc.silu(-z), z, rtol=1e-13, atol=1e-14)
    assert orc.silu(np.array([0.0]))[0] == 0.0


def test_dense_ffn_reduces_to_library_routines():
    t = _rand_ffn(0)
    T = {k: torch.from_numpy(v) for k, v in t.items()}
    F = torch.nn.functional
    want_relu = F.linear(F.relu(F.linear(T["x"], T["W_up"], T["b_up"])), T["W_down"], T["b_down"]).numpy()
    got_relu = orc.ffn_relu(t["x"], None, t["W_up"], t["b_up"], t["W_down"], t["b_down"])
    np.testing.assert_allclose(got_relu, want_relu, rtol=1e-12, atol=1e-13)
    want_sw = F.linear(F.silu(F.linear(T["x"], T["W_gate"])) * F.linear(T["x"], T["W_up"]), T["W_down"]).numpy()
    got_sw = orc.ffn_swiglu(t["x"], None, t["W_gate"], t["W_up"], t["W_down"])
    np.testing.assert_allclose(got_sw, want_sw, rtol=1e-12, atol=1e-13)
    # the ranked activations are the library's too
    np.testing.assert_allclose(orc.score_relu(t["x"], t["W_up"], t["b_up"]),
                               F.relu(F.linear(T["x"], T["W_up"], T["b_up"])).numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.score_swiglu(t["x"], t["W_gate"], t["W_up"]),
                               (F.silu(F.linear(T["x"], T["W_gate"])) * F.linear(T["x"], T["W_up"])).abs().numpy(),
                               rtol=1e-12, atol=1e-13)


def test_sparse_ffn_neuron_by_neuron():
    """The restricted FFN written as an explicit sum over the core neurons."""
    t = _rand_ffn(1)
    S = [1, 4, 5, 11]
    for b in range(t["x"].shape[0]):
        y_relu = t["b_down"].copy()
        y_sw = np.zeros_like(t["b_down"])
        for n in S:
            z = float(np.dot(t["W_up"][n], t["x"][b])) + t["b_up"][n]
            y_relu += max(z, 0.0) * t["W_down"][:, n]
            g = float(np.dot(t["W_gate"][n], t["x"][b]))
            u = float(np.dot(t["W_up"][n], t["x"][b]))
            y_sw += (g / (1.0 + math.exp(-g))) * u * t["W_down"][:, n]
        np.testing.assert_allclose(orc.ffn_relu(t["x"][b], S, t["W_up"], t["b_up"], t["W_down"], t["b_down"]),
                                   y_relu, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(orc.ffn_swiglu(t["x"][b], S, t["W_gate"], t["W_up"], t["W_down"]),
                                   y_sw, rtol=1e-12, atol=1e-13)
        # an output bias (Llama has none, the interface allows one) is added once, in full
        np.testing.assert_allclose(orc.ffn_swiglu(t["x"][b], S, t["W_gate"], t["W_up"], t["W_down"], t["b_down"]),
                                   y_sw + t["b_down"], rtol=1e-12, atol=1e-13)


def test_beta_one_is_the_dense_ffn_and_masked_dense_formulation():
    t = _rand_ffn(2, d=9, N=21, B=4)
    N = 21
    A = orc.score_relu(t["x"], t["W_up"], t["b_up"])
    S_all, _ = orc.select(A, 0.3, 1.0)
    assert S_all.tolist() == list(range(N))
    dense = orc.ffn_relu(t["x"], None, t["W_up"], t["b_up"], t["W_down"], t["b_down"])
    assert np.array_equal(orc.ffn_relu(t["x"], S_all, t["W_up"], t["b_up"], t["W_down"], t["b_down"]), dense)
    S, _ = orc.select(A, 0.3, 0.4)
    mask = np.zeros(N)
    mask[S] = 1.0
    h = np.maximum(t["x"] @ t["W_up"].T + t["b_up"], 0.0) * mask
    np.testing.assert_allclose(orc.ffn_relu(t["x"], S, t["W_up"], t["b_up"], t["W_down"], t["b_down"]),
                               h @ t["W_down"].T + t["b_down"], rtol=1e-12, atol=1e-13)
    hs = orc.hidden_swiglu(t["x"], t["W_gate"], t["W_up"]) * mask
    np.testing.assert_allclose(orc.ffn_swiglu(t["x"], S, t["W_gate"], t["W_up"], t["W_down"]),
                               hs @ t["W_down"].T, rtol=1e-12, atol=1e-13)
    # no core neurons at all: only the output bias is left
    empty = np.zeros(0, dtype=np.int64)
    assert np.array_equal(orc.ffn_relu(t["x"][0], empty, t["W_up"], t["b_up"], t["W_down"], t["b_down"]), t["b_down"])
    assert np.array_equal(orc.ffn_swiglu(t["x"][0], empty, t["W_gate"], t["W_up"], t["W_down"]), np.zeros(9))


def test_compact_is_plain_indexing_and_feeds_the_same_ffn():
    t = _rand_ffn(3, d=6, N=15, B=2)
    S = [0, 3, 4, 9, 14]
    c = orc.compact(S, t["W_up"], t["W_down"], t["W_gate"], t["b_up"])
    for k, n in enumerate(S):
        for j in range(6):
            assert c["w_up_c"][k, j] == t["W_up"][n, j]
            assert c["w_gate_c"][k, j] == t["W_gate"][n, j]
            assert c["w_down_c"][k, j] == t["W_down"][j, n]
        assert c["b_up_c"][k] == t["b_up"][n]
    # the dense FFN over the deployed buffers equals the FFN restricted to S
    y = orc.ffn_relu(t["x"], None, c["w_up_c"], c["b_up_c"], c["w_down_c"].T, t["b_down"])
    np.testing.assert_allclose(y, orc.ffn_relu(t["x"], S, t["W_up"], t["b_up"], t["W_down"], t["b_down"]),
                               rtol=1e-13, atol=1e-14)


def test_sparse_error_shrinks_as_beta_grows():
    # information only in the benchmark, but monotone set nesting makes beta = 1 exact
    t = _rand_ffn(4, d=16, N=64, B=8)
    A = orc.score_relu(t["x"], t["W_up"], t["b_up"])
    dense = orc.ffn_relu(t["x"], None, t["W_up"], t["b_up"], t["W_down"], t["b_down"])
    S, _ = orc.select(A, 0.5, 1.0)
    assert np.abs(orc.ffn_relu(t["x"], S, t["W_up"], t["b_up"], t["W_down"], t["b_down"]) - dense).max() == 0.0


# ------------------------------------------- group sets, running counts, similarity

def test_group_core_neurons_hand_example_and_identity():
    # three sentences' core sets over 6 neurons: neuron 1 in all three, 0 and 4 in two, 3 in one
    sets = [[0, 1, 4], [1, 4, 3], [0, 1, 5]]
    S, counts = orc.group_core_neurons(sets, 6, 0.5)
    assert counts.tolist() == [2, 3, 0, 1, 2, 1]
    assert S.tolist() == [0, 1, 4]                      # K = 3: counts 3, 2, 2
    S2, _ = orc.group_core_neurons(sets, 6, 0.67)       # K = ceil(4.02) = 5: tie at count 1 -> lower index 3
    assert S2.tolist() == [0, 1, 3, 4, 5][:5] and len(S2) == 5
    # identity: the group step equals Def. 1-2 applied to the 0/1 membership matrix with alpha = 1
    rng = np.random.default_rng(8)
    N, G, K = 50, 7, 12
    sets = [np.sort(rng.choice(N, size=K, replace=False)) for _ in range(G)]
    member = np.zeros((G, N))
    for g, S_g in enumerate(sets):
        member[g, S_g] = 1.0
    for gamma in (0.1, 0.3, 0.8):
        S_a, c_a = orc.group_core_neurons(sets, N, gamma)
        S_b, c_b = orc.select(member, 1.0, gamma)
        assert S_a.tolist() == S_b.tolist() and c_a.tolist() == c_b.tolist()


def test_running_counts_equal_counts_of_the_whole_sentence():
    from paper_2410_18311_amd.workloads import activation_like
    A = activation_like(20, 64, seed=4, kind="relu")
    whole = orc.count_set(A, 0.25)
    run = np.zeros(64, dtype=np.int64)
    for lo, hi in ((0, 7), (7, 8), (8, 20)):
        run = orc.count_tokens_into(run, A[lo:hi], 0.25)
    assert run.tolist() == whole.tolist()


def test_similarity_counts_hand_values():
    assert orc.core_similarity_counts([0, 1, 2], [1, 2, 3]) == (2, 4)
    assert orc.core_similarity_counts([], []) == (0, 0)
    assert orc.core_similarity_counts([5], [5]) == (1, 1)
    i, u = orc.core_similarity_counts([1, 4, 9], [2, 4])
    assert (i, u) == (1, 4) and orc.core_similarity([1, 4, 9], [2, 4]) == 0.25


def test_union_rows_hand_example_and_set_identities():
    # three sentences over 8 neurons; 9 and -1 name no neuron
    sets = [[0, 3, 5], [3, 4, 9], [-1, 5, 7]]
    U, owners = orc.union_rows(sets, 8)
    assert U.tolist() == [0, 3, 4, 5, 7]
    assert owners.tolist() == [0b001, 0b011, 0b010, 0b101, 0b100]
    # against Python set algebra on random sets: U is the sorted union, and the
    # rows tagged with bit s are exactly sentence s's set
    rng = np.random.default_rng(11)
    sets = [rng.choice(50, size=12, replace=False) for _ in range(6)]
    U, owners = orc.union_rows(sets, 50)
    assert U.tolist() == sorted(set().union(*[set(map(int, S)) for S in sets]))
    for s, S in enumerate(sets):
        assert U[(owners >> np.uint32(s)) & np.uint32(1) == 1].tolist() == sorted(map(int, S))
    assert sum(bin(int(m)).count("1") for m in owners) == 6 * 12
    # one sentence: the union is its own set, every owner mask is 1
    U, owners = orc.union_rows([[4, 2, 2, 6]], 8)
    assert U.tolist() == [2, 4, 6] and owners.tolist() == [1, 1, 1]
    U, owners = orc.union_rows([[], []], 8)
    assert U.size == 0 and owners.size == 0


def test_assign_group_hand_example_and_identities():
    prompt = [1, 2, 3, 4]
    groups = [[1, 2, 9, 10], [2, 3, 4, 8], [5, 6, 7, 11]]
    # identical / involved: 2/6, 3/5, 0/8 -> group 1
    g, pairs = orc.assign_group(prompt, groups)
    assert g == 1 and pairs == [(2, 6), (3, 5), (0, 8)]
    # a group equal to the prompt's set has similarity 1 and wins; ties go to the lower index
    g, _ = orc.assign_group(prompt, [[7, 8, 9, 10], [1, 2, 3, 4], [1, 2, 3, 4]])
    assert g == 1
    g, _ = orc.assign_group(prompt, [[1, 2, 5, 6], [3, 4, 7, 8]])     # both 2/6
    assert g == 0
    # reordering the groups moves the answer with them
    rng = np.random.default_rng(3)
    groups = [np.sort(rng.choice(200, size=40, replace=False)) for _ in range(7)]
    prompt = np.sort(rng.choice(200, size=40, replace=False))
    g, pairs = orc.assign_group(prompt, groups)
    sims = [orc.core_similarity(prompt, G) for G in groups]
    assert g == int(np.argmax(sims)) and sims.count(max(sims)) == 1
    perm = rng.permutation(7)
    g2, _ = orc.assign_group(prompt, [groups[i] for i in perm])
    assert perm[g2] == g
    assert orc.assign_group([], [[], [1]])[0] == 0


def test_compact_update_slots_hand_example_and_invariants():
    # rows hold neurons 2 5 7 9; new set 2 3 9 11: 5 and 7 leave (rows 1, 2), 3 and 11 enter
    out, changed = orc.compact_update_slots([2, 5, 7, 9], [2, 3, 9, 11])
    assert out.tolist() == [2, 3, 11, 9] and changed == 2
    out, changed = orc.compact_update_slots([2, 5, 7, 9], [9, 7, 5, 2])
    assert out.tolist() == [2, 5, 7, 9] and changed == 0
    rng = np.random.default_rng(8)
    slots = rng.permutation(300)[:120]
    for _ in range(5):           # a chain of updates
        new = np.sort(rng.choice(300, size=120, replace=False))
        out, changed = orc.compact_update_slots(slots, new)
        assert sorted(out.tolist()) == new.tolist()                      # exactly the new set, once each
        stay = np.isin(slots, new)
        assert (out[stay] == slots[stay]).all()                          # who stays keeps the row
        assert changed == int((~stay).sum()) == len(set(new) - set(slots))
        # the FFN over the rows in slot order is the FFN over the new set (a sum over neurons)
        slots = out
    d, N = 16, 300
    W1, W2, x = rng.standard_normal((N, d)), rng.standard_normal((d, N)), rng.standard_normal(d)
    b1 = rng.standard_normal(N)
    y_slots = orc.ffn_relu(x, slots, W1, b1, W2)
    y_sorted = orc.ffn_relu(x, np.sort(slots), W1, b1, W2)
    assert np.allclose(y_slots, y_sorted, rtol=1e-12, atol=1e-12)


def test_assign_centroid_hand_example_library_and_invariances():
    # hand example: three centroids on a line, feature at 1.9 -> nearest is the one at 2; an exact
    # midpoint goes to the lower index
    C = np.array([[0.0, 0.0], [2.0, 0.0], [5.0, 0.0]])
    g, d2 = orc.assign_centroid(np.array([1.9, 0.0]), C)
    assert g == 1 and np.allclose(d2, [3.61, 0.01, 9.61])
    assert orc.assign_centroid(np.array([1.0, 0.0]), C)[0] == 0          # tie between 0 and 1
    assert orc.assign_centroid(np.array([3.5, 0.0]), C)[0] == 1          # tie between 1 and 2
    assert orc.assign_centroid(np.array([7.0, 3.0]), C[:1])[0] == 0      # a single group
    # the library's vector-quantisation step (nearest code book entry, Euclidean)
    from scipy.cluster.vq import vq
    rng = np.random.default_rng(5)
    book = rng.standard_normal((9, 40))
    obs = rng.standard_normal((60, 40)) * 1.5
    code, dist = vq(obs, book)
    for i in range(60):
        g, d2 = orc.assign_centroid(obs[i], book)
        assert g == code[i]
        np.testing.assert_allclose(np.sqrt(d2[g]), dist[i], rtol=1e-12)
        # brute force, term by term
        want = [sum((obs[i, n] - book[k, n]) ** 2 for n in range(40)) for k in range(9)]
        np.testing.assert_allclose(d2, want, rtol=1e-12)
    # moving everything by the same vector, or rotating the axes, changes no assignment
    shift = rng.standard_normal(40)
    Q, _ = np.linalg.qr(rng.standard_normal((40, 40)))
    for i in range(20):
        g = orc.assign_centroid(obs[i], book)[0]
        assert orc.assign_centroid(obs[i] + shift, book + shift)[0] == g
        assert orc.assign_centroid(obs[i] @ Q, book @ Q)[0] == g
    # a centroid is its own nearest centroid, at distance zero
    for k in range(9):
        g, d2 = orc.assign_centroid(book[k], book)
        assert g == k and d2[k] == 0.0


def test_sentence_feature_is_the_token_mean():
    A = np.array([[1.0, 0.0, 4.0], [3.0, 0.0, 0.0], [2.0, 6.0, 2.0], [2.0, 2.0, 2.0]])
    assert orc.sentence_feature(A).tolist() == [2.0, 2.0, 2.0]
    rng = np.random.default_rng(2)
    B = rng.standard_normal((7, 5))
    f = orc.sentence_feature(B)
    for n in range(5):
        assert abs(f[n] - sum(B[m, n] for m in range(7)) / 7) < 1e-15
    # one token: the feature is that token's row; repeating the sentence changes nothing;
    # the token order does not matter
    assert np.array_equal(orc.sentence_feature(B[:1]), B[0])
    np.testing.assert_allclose(orc.sentence_feature(np.vstack([B, B])), f, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(orc.sentence_feature(B[::-1]), f, rtol=1e-14, atol=1e-15)
    # K-Means fixed point: with centroids = means of two well separated sets of sentences, every
    # sentence is assigned to its own set
    left = [rng.standard_normal((4, 6)) * 0.1 - 3.0 for _ in range(5)]
    right = [rng.standard_normal((4, 6)) * 0.1 + 3.0 for _ in range(5)]
    cents = np.stack([np.mean([orc.sentence_feature(a) for a in left], axis=0),
                      np.mean([orc.sentence_feature(a) for a in right], axis=0)])
    assert all(orc.assign_centroid(orc.sentence_feature(a), cents)[0] == 0 for a in left)
    assert all(orc.assign_centroid(orc.sentence_feature(a), cents)[0] == 1 for a in right)
