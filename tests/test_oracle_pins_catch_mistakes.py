"""The pins are only worth something if a wrong oracle fails them.  Each case
here plants one plausible mistake (a dropped term, a flipped comparison, a
wrong index or tie-break, swapped operands) in a copy of the oracle's source,
on the CPU, and checks that at least one pin in test_oracle_pins.py rejects
the copy.  The unmodified source must pass every pin through the same runner."""

import inspect
import itertools
import os
import types

import pytest

from tests import test_oracle_pins as pins

ORACLE_SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle",
                          "coreinfer_oracle.py")

# (name, text in the oracle, replacement, which occurrence)
MISTAKES = [
    ("zero counts as positive", "np.flatnonzero(a > 0.0)", "np.flatnonzero(a >= 0.0)", 0),
    ("keep count rounds down", "return -((-q * n) // _PPM)", "return (q * n) // _PPM", 0),
    ("keep count off by one", "return -((-q * n) // _PPM)", "return -((-q * n) // _PPM) + 1", 0),
    ("Def. 1 takes the smallest", "ranked = positive[np.argsort(-a[positive], kind=\"stable\")]",
     "ranked = positive[np.argsort(a[positive], kind=\"stable\")]", 0),
    ("Def. 1 ties to the higher index", "ranked = positive[np.argsort(-a[positive], kind=\"stable\")]",
     "ranked = positive[::-1][np.argsort(-a[positive[::-1]], kind=\"stable\")]", 0),
    ("alpha as a share of all neurons", "        k = keep_count(alpha, positive.size)\n",
     "        k = min(keep_count(alpha, a.size), positive.size)\n", 0),
    ("Def. 1 threshold rule drops ties", "return positive[a[positive] >= percentile]",
     "return positive[a[positive] > percentile]", 0),
    ("counts saturate at one", "counts[token_core_neurons(A[m], alpha, base, rule)] += 1",
     "counts[token_core_neurons(A[m], alpha, base, rule)] = 1", 0),
    ("first token not counted", "for m in range(A.shape[0]):", "for m in range(1, A.shape[0]):", 0),
    ("Def. 2 takes the rarest", "ranked = np.argsort(-counts.astype(np.int64), kind=\"stable\")",
     "ranked = np.argsort(counts.astype(np.int64), kind=\"stable\")", 0),
    ("Def. 2 ties to the higher index", "ranked = np.argsort(-counts.astype(np.int64), kind=\"stable\")",
     "ranked = (n - 1 - np.argsort(-counts.astype(np.int64)[::-1], kind=\"stable\"))", 0),
    ("beta as a share of the counted neurons", "    k = keep_count(beta, n)\n",
     "    k = max(1, keep_count(beta, int((counts > 0).sum())))\n", 0),
    ("S not ascending", "return np.sort(chosen).astype(np.int64)", "return chosen.astype(np.int64)", 0),
    ("Def. 2 threshold rule drops ties", "chosen = np.flatnonzero(counts >= percentile)",
     "chosen = np.flatnonzero(counts > percentile)", 0),
    ("SiLU sign", "return z / (1.0 + np.exp(-z))", "return z / (1.0 + np.exp(z))", 0),
    ("SiLU without the gate factor", "return z / (1.0 + np.exp(-z))", "return 1.0 / (1.0 + np.exp(-z))", 0),
    ("score bias sign", "Z = Z + _f64(b_up)", "Z = Z - _f64(b_up)", 0),
    ("score without the ReLU", "return np.maximum(Z, 0.0)", "return Z", 0),
    ("gated score keeps the sign", "return np.abs(hidden_swiglu(X, W_gate, W_up))",
     "return hidden_swiglu(X, W_gate, W_up)", 0),
    ("gate and up swapped in the hidden vector",
     "return silu(_f64(X) @ _f64(W_gate).T) * (_f64(X) @ _f64(W_up).T)",
     "return silu(_f64(X) @ _f64(W_up).T) * (_f64(X) @ _f64(W_gate).T)", 0),
    ("ReLU FFN: bias of the first K neurons", "z = z + _f64(b_up)[S]", "z = z + _f64(b_up)[:S.size]", 0),
    ("ReLU FFN: bias dropped", "z = z + _f64(b_up)[S]", "z = z", 0),
    ("ReLU FFN: magnitude instead of ReLU", "h = np.maximum(z, 0.0)", "h = np.abs(z)", 0),
    ("ReLU FFN: down columns of the first K neurons", "y = h @ W_down[:, S].T", "y = h @ W_down[:, :S.size].T", 0),
    ("gated FFN: down columns of the first K neurons", "y = h @ W_down[:, S].T", "y = h @ W_down[:, :S.size].T", 1),
    ("ReLU FFN: output bias dropped", "y = y + _f64(b_down)", "y = y", 0),
    ("gated FFN: output bias dropped", "y = y + _f64(b_down)", "y = y", 1),
    ("gated FFN: gate and up swapped", "h = silu(x @ W_gate[S, :].T) * (x @ W_up[S, :].T)",
     "h = silu(x @ W_up[S, :].T) * (x @ W_gate[S, :].T)", 0),
    ("gated FFN: up rows of the first K neurons", "h = silu(x @ W_gate[S, :].T) * (x @ W_up[S, :].T)",
     "h = silu(x @ W_gate[S, :].T) * (x @ W_up[:S.size, :].T)", 0),
    ("compact: rows in reverse order", "\"w_up_c\": np.asarray(W_up)[S, :]", "\"w_up_c\": np.asarray(W_up)[S[::-1], :]", 0),
    ("compact: down columns off by one", "np.asarray(W_down)[:, S].T", "np.asarray(W_down)[:, (S + 1) % np.asarray(W_down).shape[1]].T", 0),
    ("compact: bias of the first K neurons", "out[\"b_up_c\"] = np.asarray(b_up)[S]", "out[\"b_up_c\"] = np.asarray(b_up)[:S.size]", 0),
    ("running counts forget the past", "return np.asarray(counts, dtype=np.int64) + count_set(A, alpha)",
     "return count_set(A, alpha)", 0),
    ("group counts saturate", "                counts[int(n)] += 1", "                counts[int(n)] = 1", 0),
    ("update pairs rows with entering neurons in reverse", "for j, n in zip(free, entering):",
     "for j, n in zip(free, reversed(entering)):", 0),
    ("update moves neurons that stay", "if n in newset and n not in seen:", "if n in newset and n not in seen and j % 2:", 0),
    ("union keeps only the last owner", "owners[int(n)] |= np.uint32(1 << s)", "owners[int(n)] = np.uint32(1 << s)", 0),
    ("union owner bit off by one", "owners[int(n)] |= np.uint32(1 << s)", "owners[int(n)] |= np.uint32(1 << (s + 1))", 0),
    ("similarity counts: union as a sum", "return len(a & b), len(a | b)", "return len(a & b), len(a) + len(b)", 0),
    ("group choice: ties to the higher index", "if best_sim is None or sim > best_sim:",
     "if best_sim is None or sim >= best_sim:", 0),
    ("group choice: least similar", "if best_sim is None or sim > best_sim:", "if best_sim is None or sim < best_sim:", 0),
    ("feature: sum instead of mean", "return A.sum(axis=0) / A.shape[0]", "return A.sum(axis=0)", 0),
    ("feature: mean over neurons", "return A.sum(axis=0) / A.shape[0]", "return A.sum(axis=1) / A.shape[1]", 0),
    ("feature: last token dropped", "return A.sum(axis=0) / A.shape[0]", "return A[:-1].sum(axis=0) / A.shape[0]", 0),
    ("centroid: farthest", "if d2[g] < d2[best]:", "if d2[g] > d2[best]:", 0),
    ("centroid: ties to the higher index", "if d2[g] < d2[best]:", "if d2[g] <= d2[best]:", 0),
    ("centroid: sum of absolute differences", "d2[g] = float(np.dot(diff, diff))", "d2[g] = float(np.abs(diff).sum())", 0),
    ("centroid: first coordinate skipped", "d2[g] = float(np.dot(diff, diff))", "d2[g] = float(np.dot(diff[1:], diff[1:]))", 0),
    ("centroid: similarity instead of distance", "d2[g] = float(np.dot(diff, diff))", "d2[g] = -float(np.dot(f, C[g]))", 0),
    ("similarity over the larger set", "return len(a & b) / len(a | b)", "return len(a & b) / max(len(a), len(b))", 0),
]


def _oracle_with(old, new, occurrence):
    src = open(ORACLE_SRC).read()
    if old is not None:
        parts = src.split(old)
        assert len(parts) > occurrence + 1, f"oracle source no longer contains {old!r}"
        src = old.join(parts[:occurrence + 1]) + new + old.join(parts[occurrence + 1:])
    mod = types.ModuleType("oracle_copy")
    mod.__file__ = ORACLE_SRC
    exec(compile(src, ORACLE_SRC, "exec"), mod.__dict__)
    return mod


def _pin_cases():
    """Every pin with every parameter set it is run with."""
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not inspect.isfunction(fn):
            continue
        axes = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                names = [n.strip() for n in mark.args[0].split(",")]
                rows = [v if len(names) > 1 else (v,) for v in mark.args[1]]
                axes.append([dict(zip(names, row)) for row in rows])
        for combo in itertools.product(*axes):
            kwargs = {}
            for part in combo:
                kwargs.update(part)
            yield name, fn, kwargs


def _first_pin_that_fails(oracle_module, monkeypatch):
    monkeypatch.setattr(pins, "orc", oracle_module)
    for name, fn, kwargs in _pin_cases():
        try:
            fn(**kwargs)
        except Exception as exc:  # an assertion, or the mistake made the oracle raise
            return f"{name}{kwargs or ''}: {type(exc).__name__}"
    return None


def test_runner_passes_the_real_oracle(monkeypatch):
    assert sum(1 for _ in _pin_cases()) >= 30
    assert _first_pin_that_fails(_oracle_with(None, None, 0), monkeypatch) is None


@pytest.mark.parametrize("mistake", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_some_pin(mistake, monkeypatch):
    name, old, new, occurrence = mistake
    caught_by = _first_pin_that_fails(_oracle_with(old, new, occurrence), monkeypatch)
    assert caught_by is not None, f"no pin notices: {name}"
