"""Plain CPU oracle for CoreInfer's hot path (arXiv 2410.18311).

TEST INFRASTRUCTURE, NOT PRODUCT.  Slow, float64, written straight from the
paper's definitions so it can be checked against them by eye.  It shares no
code, tables or helpers with the HIP library, and imports nothing from it.
Only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

What is here, and the passage each part follows:

* ``token_core_neurons``    -- Definition 1 / Eq. 1 (Sec. 3.1): the token-wise
  core neurons, the top-alpha share of the positively activated neurons.
* ``count_set``             -- Eq. 3 (Sec. 3.1): how many of the sentence's
  tokens have each neuron in their token-wise core set.
* ``sentence_core_neurons`` -- Definition 2 / Eq. 2 (Sec. 3.1): the top-beta
  share of neurons by that count.
* ``select``                -- the three above chained (prefill stage, Fig. 1,
  Sec. 4.2); stability-guided prediction (Sec. 4.1) freezes the result.
* ``ffn_relu`` / ``ffn_swiglu`` -- the decode-stage FFN restricted to the
  frozen core set (Sec. 4.2; Sec. 5.3 "only a static subset of neurons take
  part"): the standard OPT / Llama FFN with every neuron outside S removed.
* ``score_relu`` / ``score_swiglu`` -- the per-token activation vector
  A(x) that Definition 1 ranks.
* ``compact``               -- Sec. 5.3 "deploy the necessary neurons during
  pre-filling": the rows / columns of the weights that S names.
* ``core_similarity``       -- Insight-2 (Sec. 3.2): identical neurons over
  all neurons involved.
* ``group_core_neurons``    -- similarity-guided prediction, group step
  (Sec. 4.1): top-gamma of neurons by how many of the group's sentences have
  them in their core set.
* ``assign_group``          -- similarity-guided prediction, choosing the group
  (Sec. 4.1 says only "once the input sentence's group is determined"): the
  group whose core set is most similar to the prompt's own under Insight-2's
  metric.
* ``sentence_feature`` / ``assign_centroid`` -- similarity-guided prediction
  when the groups come from K-Means on a layer's activation (App. A.2.3): the
  vector a sentence is clustered by, and the K-Means assignment step (nearest
  centroid) that puts a new prompt into a group.
* ``count_tokens_into``     -- Eq. 3 as a running sum when a sentence grows.
* ``compact_update_slots``  -- re-deploying after the core set changed
  (Fig. 1 "stability estimation ... how to update"; the paper gives no rule):
  only the rows whose neuron left the set are rewritten.
* ``union_rows``            -- batching several sentences that share resident
  weights (the Sec. 5.3 large-model scenario): the neurons any sentence
  needs, each tagged with the sentences that own it.  The decode result of a
  batch is by definition each sentence's own ``ffn_relu`` / ``ffn_swiglu``.

Readings taken where the paper is silent or ambiguous (each is also listed in
the design document):

* alpha, beta are KEEP fractions ("top alpha ... largest"), not percentiles
  counted from the bottom.
* alpha is a share of the POSITIVE neurons of that token (Eq. 1 takes the
  percentile over A+).  ``base="all"`` gives the other reading.
* Set sizes are fixed: ``keep_count(f, n) = ceil(round(f * 1e6) * n / 1e6)``
  in integers (Fig. 1 speaks of "top-k selection").  ``rule="threshold"``
  gives the literal ">= percentile" reading, which keeps all ties.
* Ties (equal activation, equal count) go to the lower neuron index.
* Neurons with count zero are admitted, in index order, when fewer than K
  neurons were ever token-core; |S| is always K.  S is reported ascending.
* NaN is never positive, so never selected; +inf ranks first.
* For SiLU-gated FFNs the ranked activation is |SiLU(gate) * up|, the
  magnitude of what the down projection consumes.
* b_down is not neuron-indexed and is always added in full.

Parity pins: every function here is pinned by tests/test_oracle_pins.py
(brute force by repeated arg-max, a hand-worked example, permutation and
scaling invariances, count identities, nesting in beta, beta = 1 equals the
dense FFN, masked-dense formulation, empty-set limit).  The approximation
quality of the sparse FFN on synthetic data is parity unpinned: the paper's
accuracy claims need trained weights.
"""

from __future__ import annotations

import math

import numpy as np

_PPM = 10**6


def keep_count(frac: float, n: int) -> int:
    """Size of "the top ``frac`` of ``n`` items": the smallest integer k with
    k / n >= frac, where frac is first rounded to parts per million so that
    0.1 * 3-style float noise cannot move the result.  (Reading of the
    rounding that Def. 1 / Def. 2 leave open.)"""
    n = int(n)
    if n < 0:
        raise ValueError("n must be >= 0")
    if not (frac > 0.0 and frac <= 1.0):
        raise ValueError("fraction must lie in (0, 1]")
    q = int(math.floor(float(frac) * 1e6 + 0.5))
    if q < 1:
        raise ValueError("fraction below one part per million")
    return -((-q * n) // _PPM)


def token_core_neurons(a, alpha: float, base: str = "positive", rule: str = "topk") -> np.ndarray:
    """Definition 1 / Eq. 1: core neurons of ONE token.

    ``a`` is the activation vector A(x) = [a_1 .. a_N].  A+ is the set of
    neurons with a_n > 0.  The result holds the top-alpha share of A+ by
    activation value, largest first; equal values are ordered by index.
    """
    a = np.asarray(a, dtype=np.float64)
    if a.ndim != 1:
        raise ValueError("one token's activation vector expected")
    positive = np.flatnonzero(a > 0.0)                # NaN > 0 is False
    if positive.size == 0:
        return positive.astype(np.int64)
    if base == "positive":
        k = keep_count(alpha, positive.size)
    elif base == "all":
        k = min(keep_count(alpha, a.size), positive.size)
    else:
        raise ValueError(base)
    # full sort: value descending, index ascending among equals (stable sort
    # of the negated values keeps index order inside a tie).
    ranked = positive[np.argsort(-a[positive], kind="stable")]
    if rule == "topk":
        return ranked[:k]
    if rule == "threshold":                           # literal Eq. 1
        percentile = a[ranked[k - 1]]
        return positive[a[positive] >= percentile]
    raise ValueError(rule)


def count_set(A, alpha: float, base: str = "positive", rule: str = "topk") -> np.ndarray:
    """Eq. 3: f_alpha(n; s) = sum over the sentence's tokens m of
    1[n in C_alpha(x^m)].  ``A`` is [M, N], one activation row per token."""
    A = np.asarray(A, dtype=np.float64)
    if A.ndim != 2:
        raise ValueError("A must be [M, N]")
    counts = np.zeros(A.shape[1], dtype=np.int64)
    for m in range(A.shape[0]):
        counts[token_core_neurons(A[m], alpha, base, rule)] += 1
    return counts


def sentence_core_neurons(counts, beta: float, rule: str = "topk") -> np.ndarray:
    """Definition 2 / Eq. 2: the top-beta share of all N neurons by count,
    equal counts ordered by index; reported in ascending index order."""
    counts = np.asarray(counts)
    if counts.ndim != 1:
        raise ValueError("counts must be [N]")
    n = counts.size
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    k = keep_count(beta, n)
    ranked = np.argsort(-counts.astype(np.int64), kind="stable")
    if rule == "topk":
        chosen = ranked[:k]
    elif rule == "threshold":                         # literal Eq. 2
        percentile = counts[ranked[k - 1]]
        chosen = np.flatnonzero(counts >= percentile)
    else:
        raise ValueError(rule)
    return np.sort(chosen).astype(np.int64)


def select(A, alpha: float, beta: float, base: str = "positive", rule: str = "topk"):
    """Prefill-stage core-neuron selection for one layer of one sentence
    (Fig. 1; Def. 1 -> Eq. 3 -> Def. 2).  Returns (S ascending, counts)."""
    counts = count_set(A, alpha, base, rule)
    return sentence_core_neurons(counts, beta, rule), counts


# --------------------------------------------------------------------------
# FFN arithmetic.  Weights use the nn.Linear convention of the models the
# paper runs (OPT, Llama): W_up, W_gate are [N, d]; W_down is [d, N].
# --------------------------------------------------------------------------

def _f64(t):
    return np.asarray(t, dtype=np.float64)


def silu(z):
    z = _f64(z)
    return z / (1.0 + np.exp(-z))


def score_relu(X, W_up, b_up=None):
    """A(x) for a ReLU FFN (OPT): max(W_up x + b_up, 0), one row per token."""
    Z = _f64(X) @ _f64(W_up).T
    if b_up is not None:
        Z = Z + _f64(b_up)
    return np.maximum(Z, 0.0)


def hidden_swiglu(X, W_gate, W_up):
    """What the down projection of a SiLU-gated FFN (Llama) consumes."""
    return silu(_f64(X) @ _f64(W_gate).T) * (_f64(X) @ _f64(W_up).T)


def score_swiglu(X, W_gate, W_up):
    """A(x) for a SiLU-gated FFN: |SiLU(W_gate x) * (W_up x)|."""
    return np.abs(hidden_swiglu(X, W_gate, W_up))


def ffn_relu(x, S, W_up, b_up, W_down, b_down=None):
    """Decode-stage FFN over the frozen core set S (Sec. 4.2):
    y = W_down[:, S] max(W_up[S, :] x + b_up[S], 0) + b_down.
    ``x`` is [d] or [B, d]; S = None means every neuron (the dense FFN)."""
    x = _f64(x)
    W_up, W_down = _f64(W_up), _f64(W_down)
    if S is None:
        S = np.arange(W_up.shape[0])
    S = np.asarray(S, dtype=np.int64)
    z = x @ W_up[S, :].T
    if b_up is not None:
        z = z + _f64(b_up)[S]
    h = np.maximum(z, 0.0)
    y = h @ W_down[:, S].T
    if b_down is not None:
        y = y + _f64(b_down)
    return y


def ffn_swiglu(x, S, W_gate, W_up, W_down, b_down=None):
    """Decode-stage SiLU-gated FFN over the frozen core set S:
    y = W_down[:, S] (SiLU(W_gate[S, :] x) * (W_up[S, :] x)) [+ b_down]."""
    x = _f64(x)
    W_gate, W_up, W_down = _f64(W_gate), _f64(W_up), _f64(W_down)
    if S is None:
        S = np.arange(W_up.shape[0])
    S = np.asarray(S, dtype=np.int64)
    h = silu(x @ W_gate[S, :].T) * (x @ W_up[S, :].T)
    y = h @ W_down[:, S].T
    if b_down is not None:
        y = y + _f64(b_down)
    return y


def compact(S, W_up, W_down, W_gate=None, b_up=None):
    """Sec. 5.3: the neurons deployed for decoding -- rows S of the up (and
    gate) projection, entries S of its bias, columns S of the down
    projection (returned neuron-major, i.e. transposed, [K, d])."""
    S = np.asarray(S, dtype=np.int64)
    out = {"w_up_c": np.asarray(W_up)[S, :], "w_down_c": np.asarray(W_down)[:, S].T}
    if W_gate is not None:
        out["w_gate_c"] = np.asarray(W_gate)[S, :]
    if b_up is not None:
        out["b_up_c"] = np.asarray(b_up)[S]
    return out


def count_tokens_into(counts, A, alpha: float) -> np.ndarray:
    """Running form of Eq. 3: the count set of a sentence that grew by the
    tokens in A is the old count set plus the new tokens' contributions."""
    return np.asarray(counts, dtype=np.int64) + count_set(A, alpha)


def group_core_neurons(core_sets, n_neurons: int, gamma: float):
    """Similarity-guided prediction, group step (Sec. 4.1): the top-gamma share
    of neurons that appear most often in the core sets of the group's
    sentences.  Returns (S ascending, counts)."""
    counts = np.zeros(int(n_neurons), dtype=np.int64)
    for S in core_sets:
        for n in S:
            if 0 <= int(n) < n_neurons:
                counts[int(n)] += 1
    return sentence_core_neurons(counts, gamma), counts


def compact_update_slots(slot_idx, new_set):
    """Updating deployed neurons in place when the core set changes (the paper
    names the update in Fig. 1 but gives no rule; this one rewrites as little
    as possible).  ``slot_idx[j]`` is the neuron held by row j of the compact
    buffers.  Neurons that stay keep their row; the rows of neurons that left
    (ascending row) take the neurons that entered (ascending neuron).
    Returns (new slot_idx, number of rows rewritten)."""
    slot_idx = [int(v) for v in slot_idx]
    new = sorted(set(int(v) for v in new_set))
    if len(new) != len(slot_idx):
        raise ValueError("the core set keeps its size")
    newset = set(new)
    seen, free = set(), []
    for j, n in enumerate(slot_idx):
        if n in newset and n not in seen:
            seen.add(n)
        else:
            free.append(j)
    entering = [n for n in new if n not in seen]
    out = list(slot_idx)
    for j, n in zip(free, entering):
        out[j] = n
    return np.asarray(out, dtype=np.int64), len(free)


def union_rows(core_sets, n_neurons: int):
    """Rows of the weight matrices that a batch of sentences needs: U = the
    union of the sentences' core sets (ascending) and, per row of U, a bit
    mask whose bit s says that sentence s owns the row.  Indices outside
    [0, n_neurons) name no neuron and are ignored.  At most 32 sentences."""
    if len(core_sets) > 32:
        raise ValueError("at most 32 sentences")
    owners = np.zeros(int(n_neurons), dtype=np.uint32)
    for s, S in enumerate(core_sets):
        for n in S:
            if 0 <= int(n) < n_neurons:
                owners[int(n)] |= np.uint32(1 << s)
    U = np.flatnonzero(owners).astype(np.int64)
    return U, owners[U]


def core_similarity_counts(S1, S2):
    """(identical neurons, neurons involved) of Insight-2's similarity."""
    a, b = set(int(v) for v in S1), set(int(v) for v in S2)
    return len(a & b), len(a | b)


def assign_group(prompt_set, group_sets):
    """Similarity-guided prediction, group choice (Sec. 4.1; the rule is a
    reading, the paper leaves it open): the group whose core set has the
    largest Insight-2 similarity (identical / involved neurons) with the
    prompt's own core set; equal similarities go to the lower group index;
    two empty sets count as similarity 1.  Returns (group, [(identical,
    involved) per group]).  Compared as exact fractions."""
    from fractions import Fraction
    pairs = [core_similarity_counts(prompt_set, G) for G in group_sets]
    best, best_sim = -1, None
    for g, (i, u) in enumerate(pairs):
        sim = Fraction(1) if u == 0 else Fraction(i, u)
        if best_sim is None or sim > best_sim:
            best, best_sim = g, sim
    return best, pairs


def sentence_feature(A) -> np.ndarray:
    """The vector a sentence is clustered by.  App. A.2.3 runs K-Means on "the
    activation" of one layer without saying how a sentence's tokens are
    summarised; the reading taken here is the mean over the sentence's tokens
    of the layer's activation rows A [M, N] (the vector Def. 1 ranks)."""
    A = np.asarray(A, dtype=np.float64)
    if A.ndim != 2 or A.shape[0] < 1:
        raise ValueError("A must be [M, N] with M >= 1")
    return A.sum(axis=0) / A.shape[0]


def assign_centroid(feature, centroids):
    """Group of a new prompt when the groups are K-Means clusters (App. A.2.3):
    the K-Means assignment step, i.e. the centroid nearest to the prompt's
    feature vector in Euclidean distance; equal distances go to the lower
    group index.  Returns (group, squared distances [G])."""
    f = np.asarray(feature, dtype=np.float64)
    C = np.asarray(centroids, dtype=np.float64)
    if C.ndim != 2 or f.ndim != 1 or C.shape[1] != f.shape[0] or C.shape[0] < 1:
        raise ValueError("feature [N], centroids [G, N] with G >= 1")
    d2 = np.zeros(C.shape[0])
    for g in range(C.shape[0]):
        diff = f - C[g]
        d2[g] = float(np.dot(diff, diff))
    return nearest_group(d2), d2


def nearest_group(d2) -> int:
    """The decision of the K-Means assignment step (App. A.2.3) on given squared
    distances: the smallest one, the lower group index among equal ones."""
    d2 = np.asarray(d2, dtype=np.float64)
    if d2.ndim != 1 or d2.shape[0] < 1:
        raise ValueError("squared distances [G] with G >= 1")
    best = 0
    for g in range(1, d2.shape[0]):
        if d2[g] < d2[best]:
            best = g
    return best


def core_similarity(S1, S2) -> float:
    """Insight-2 (Sec. 3.2): identical neurons / all neurons involved."""
    a, b = set(int(v) for v in S1), set(int(v) for v in S2)
    if not a and not b:
        return 1.0
    return len(a & b) / len(a | b)
