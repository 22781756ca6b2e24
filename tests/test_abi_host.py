"""Host-side checks of the C ABI that need no GPU: the library loads, exports
what include/coreinfer.h declares, and rejects bad arguments before touching
the device (validation precedes every HIP call)."""

import ctypes
import os
import re

import pytest

from oracle import coreinfer_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "coreinfer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(coreinfer_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib.raw, n), n
    assert set(names) == set(lib.EXPORTS)
    assert lib.version() >= 2


def test_strerror_names_every_status(lib):
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6):
        s = lib.strerror(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 7
    assert lib.strerror(-99) == "unknown status"


def test_keep_count_agrees_with_the_oracle_rule(lib):
    for n in (0, 1, 2, 3, 7, 10, 30, 1024, 11008, 13824, 16384, 36864):
        for f in (1e-6, 0.01, 0.1, 0.2, 0.25, 0.3, 1 / 3, 0.34, 0.4, 0.5, 0.6, 0.999999, 1.0):
            assert lib.keep_count(f, n) == orc.keep_count(f, n), (f, n)
    assert lib.keep_count(0.4, 16384) == 6554 and lib.keep_count(0.4, 36864) == 14746
    k = ctypes.c_int64(0)
    for bad in (0.0, -0.1, 1.0000001, float("nan"), 1e-9):
        assert lib.raw.coreinfer_keep_count(bad, 10, ctypes.byref(k)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_keep_count(0.5, -1, ctypes.byref(k)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_keep_count(0.5, 10, None) == lib.CI_ERR_INVALID_ARG


def test_workspace_sizes(lib):
    assert lib.select_workspace_size(256, 16384) >= 16384 * 4
    assert lib.ffn_decode_workspace_size(1, 6554, 4096) >= 1024 * 4096 * 4
    assert lib.ffn_decode_workspace_size(1, 10, 256) >= 10 * 256 * 4
    assert lib.ffn_decode_workspace_size(8, 14746, 9216) >= 8 * 1024 * 9216 * 4
    import torch
    assert lib.ffn_dense_workspace_size(256, 4096, 16384, torch.float16) >= 256 * 16384 * 2
    b = ctypes.c_size_t(0)
    assert lib.raw.coreinfer_select_workspace_size(0, 10, ctypes.byref(b)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_select_workspace_size(70000, 10, ctypes.byref(b)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_select_workspace_size(4, 10, None) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_ffn_decode_workspace_size(0, 10, 64, ctypes.byref(b)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_ffn_dense_workspace_size(4, 64, 64, 9, ctypes.byref(b)) == lib.CI_ERR_BAD_DTYPE


FAKE = 0x10000  # a non-null, 16-byte aligned address that is never dereferenced on these paths


def test_select_rejects_bad_arguments_without_a_gpu(lib):
    r = lib.raw.coreinfer_select
    ok_ws = 1 << 20
    assert r(None, 4, 64, 64, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 4, 64, 64, 0.2, 0.4, None, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 0, 64, 64, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 4, 64, 64, 0.0, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 4, 64, 64, 0.2, 1.5, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 4, 64, 32, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(FAKE + 2, 4, 64, 64, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(FAKE, 4, 64, 64, 0.2, 0.4, FAKE, None, None, ok_ws, None) == lib.CI_ERR_WORKSPACE
    assert r(FAKE, 4, 64, 64, 0.2, 0.4, FAKE, None, FAKE, 16, None) == lib.CI_ERR_WORKSPACE


def test_compact_rejects_bad_arguments_without_a_gpu(lib):
    r = lib.raw.coreinfer_compact
    F = FAKE
    # (w_up, w_gate, b_up, w_down, layout, dtype, act, d, N, idx, K, up_c, gate_c, b_c, down_c, down_c_layout,
    #  status, stream)
    assert r(F, None, None, F, 0, 7, 0, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, None, None, F, 0, 1, 5, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, None, None, F, 3, 1, 0, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(None, None, None, F, 0, 1, 0, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 200, F, None, None, F, 1, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 0, 64, 128, None, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_INVALID_ARG
    # gate given for ReLU / missing for SwiGLU; bias in without bias out
    assert r(F, F, None, F, 0, 1, 0, 64, 128, F, 8, F, F, None, F, 1, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 1, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, F, F, 0, 1, 0, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_INVALID_ARG
    # d not a multiple of 8 halfs; misaligned pointer
    assert r(F, None, None, F, 0, 1, 0, 60, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F + 8, None, None, F, 0, 1, 0, 64, 128, F, 8, F, None, None, F, 1, None, None) == lib.CI_ERR_BAD_LAYOUT
    # layout of the compact down matrix out of range; up bias with a gated FFN
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 8, F, None, None, F, 2, None, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, F, F, F, 0, 1, 1, 64, 128, F, 8, F, F, F, F, 0, None, None) == lib.CI_ERR_INVALID_ARG
    ld = ctypes.c_int64(0)
    assert lib.raw.coreinfer_compact_down_ld(6554, 1, ctypes.byref(ld)) == lib.CI_OK and ld.value == 6560
    assert lib.raw.coreinfer_compact_down_ld(410, 0, ctypes.byref(ld)) == lib.CI_OK and ld.value == 412
    assert lib.raw.coreinfer_compact_down_ld(0, 2, ctypes.byref(ld)) == lib.CI_OK and ld.value == 0
    assert lib.raw.coreinfer_compact_down_ld(8, 5, ctypes.byref(ld)) == lib.CI_ERR_BAD_DTYPE
    assert lib.raw.coreinfer_compact_down_ld(-1, 1, ctypes.byref(ld)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_compact_down_ld(8, 1, None) == lib.CI_ERR_INVALID_ARG


def test_preferred_compact_layout_and_its_arguments(lib):
    """Pure host function: small layers -> neuron-major, large ones -> output-major, shapes the
    single-launch decode does not take -> neuron-major."""
    import torch
    out = ctypes.c_int(-1)
    r = lib.raw.coreinfer_compact_preferred_layout
    assert r(2765, 5120, lib.CI_BF16, lib.CI_ACT_SWIGLU, ctypes.byref(out)) == lib.CI_OK
    assert out.value == lib.CI_DOWN_NEURON_MAJOR
    assert r(8295, 5120, lib.CI_BF16, lib.CI_ACT_SWIGLU, ctypes.byref(out)) == lib.CI_OK
    assert out.value == lib.CI_DOWN_OUT_MAJOR
    assert r(20000, 32768, lib.CI_F16, lib.CI_ACT_RELU, ctypes.byref(out)) == lib.CI_OK   # d beyond the single launch
    assert out.value == lib.CI_DOWN_NEURON_MAJOR
    assert r(0, 4096, lib.CI_F16, lib.CI_ACT_RELU, ctypes.byref(out)) == lib.CI_OK and out.value == lib.CI_DOWN_NEURON_MAJOR
    assert r(10, 4096, 9, lib.CI_ACT_RELU, ctypes.byref(out)) == lib.CI_ERR_BAD_DTYPE
    assert r(10, 0, lib.CI_F16, lib.CI_ACT_RELU, ctypes.byref(out)) == lib.CI_ERR_INVALID_ARG
    assert r(-1, 64, lib.CI_F16, lib.CI_ACT_RELU, ctypes.byref(out)) == lib.CI_ERR_INVALID_ARG
    assert r(10, 64, lib.CI_F16, lib.CI_ACT_RELU, None) == lib.CI_ERR_INVALID_ARG
    assert lib.compact_preferred_layout(6554, 4096, torch.float16, "relu") in ("neuron_major", "out_major")
    plan = lib.dev_fused_plan(6554, 4096, torch.float16, "relu")
    assert plan["chunks"] >= 2 and plan["chunks"] * plan["chunk_neurons"] >= 6554 and plan["loads_per_row"] == 1
    assert (plan["chunks"] - 1) * plan["chunk_neurons"] < 6554


def test_select_batch_rejects_bad_arguments_without_a_gpu(lib):
    r = lib.raw.coreinfer_select_batch
    ok_ws = 1 << 22
    b = ctypes.c_size_t(0)
    assert lib.raw.coreinfer_select_batch_workspace_size(8, 512, 36864, ctypes.byref(b)) == lib.CI_OK
    assert b.value >= 8 * 36864 * 4 + 8 * 512 * 8
    assert lib.select_batch_workspace_size(1, 256, 16384) == lib.select_workspace_size(256, 16384)
    assert lib.raw.coreinfer_select_batch_workspace_size(0, 4, 64, ctypes.byref(b)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_select_batch_workspace_size(70000, 4, 64, ctypes.byref(b)) == lib.CI_ERR_INVALID_ARG
    assert lib.raw.coreinfer_select_batch_workspace_size(2, 4, 64, None) == lib.CI_ERR_INVALID_ARG
    # (act, B, M, N, ld, alpha, beta, core_idx, counts, ws, ws_bytes, stream)
    assert r(None, 2, 4, 64, 64, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 2, 4, 64, 64, 0.2, 0.4, None, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 0, 4, 64, 64, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 2, 4, 64, 64, 0.2, 2.0, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_INVALID_ARG
    assert r(FAKE, 2, 4, 64, 32, 0.2, 0.4, FAKE, None, FAKE, ok_ws, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(FAKE, 2, 4, 64, 64, 0.2, 0.4, FAKE + 2, None, FAKE, ok_ws, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(FAKE, 2, 4, 64, 64, 0.2, 0.4, FAKE, None, None, ok_ws, None) == lib.CI_ERR_WORKSPACE
    assert r(FAKE, 2, 4, 64, 64, 0.2, 0.4, FAKE, None, FAKE, 16, None) == lib.CI_ERR_WORKSPACE


def test_static_decode_rejects_bad_arguments_without_a_gpu(lib):
    """coreinfer_ffn_decode_static validates like coreinfer_ffn_decode and turns down what its
    scratch cannot hold before any HIP call."""
    r = lib.raw.coreinfer_ffn_decode_static
    F = FAKE
    def desc(K=8, d=64, N=128, layout=1, ld=0, core=None, gate=None, bias=None):
        return lib.ci_ffn_weights(F, gate, bias, F, None, core, K, d, N, ld, layout)
    # (x, B, w, dtype, act, y, status_out, stream)
    assert r(F, 1, None, 1, 0, F, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(None, 1, ctypes.byref(desc()), 1, 0, F, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, ctypes.byref(desc()), 7, 0, F, None, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, 1, ctypes.byref(desc(layout=5)), 1, 0, F, None, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 1, ctypes.byref(desc(gate=F)), 1, 0, F, None, None) == lib.CI_ERR_INVALID_ARG       # gate with ReLU
    assert r(F, 1, ctypes.byref(desc(gate=F, bias=F)), 1, 1, F, None, None) == lib.CI_ERR_INVALID_ARG  # bias with SwiGLU
    assert r(F, 1, ctypes.byref(desc(d=60)), 1, 0, F, None, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 1, ctypes.byref(desc(layout=0, ld=4)), 1, 0, F, None, None) == lib.CI_ERR_BAD_LAYOUT  # ld < K
    assert r(F, 1, ctypes.byref(desc()), 1, 0, F, F + 2, None) == lib.CI_ERR_BAD_LAYOUT               # status_out misaligned
    assert r(F, 1, ctypes.byref(desc(K=200000, N=200000, layout=0, ld=200000)), 1, 0, F, None, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 8, ctypes.byref(desc(K=4096, d=32768, N=4096)), 1, 0, F, None, None) == lib.CI_ERR_WORKSPACE


def test_compact_update_rejects_bad_arguments_without_a_gpu(lib):
    r = lib.raw.coreinfer_compact_update
    F = FAKE
    big = 1 << 24
    # (w_up, w_gate, b_up, w_down, layout, dtype, act, d, N, new_idx, K, slot_idx, w_up_c, w_gate_c, b_up_c,
    #  w_down_c, down_c_layout, changed, ws, ws_bytes, stream)
    assert r(F, None, None, F, 0, 6, 0, 64, 128, F, 8, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, None, None, F, 3, 1, 0, 64, 128, F, 8, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, None, None, F, 0, 1, 0, 64, 128, None, 8, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 8, None, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 200, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 1, 64, 128, F, 8, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, F, F, 0, 1, 0, 64, 128, F, 8, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, None, None, F, 0, 1, 0, 60, 128, F, 8, F, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 8, F + 2, F, None, None, F, 1, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 8, F, F, None, None, F, 1, None, None, big, None) == lib.CI_ERR_WORKSPACE
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 8, F, F, None, None, F, 1, None, F, 100, None) == lib.CI_ERR_WORKSPACE
    assert r(F, None, None, F, 0, 1, 0, 64, 128, F, 8, F, F, None, None, F, 7, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    n = ctypes.c_size_t(0)
    assert lib.raw.coreinfer_compact_update_workspace_size(128, 8, ctypes.byref(n)) == lib.CI_OK
    assert n.value >= (128 + 3 * 8 + 1) * 4
    assert lib.raw.coreinfer_compact_update_workspace_size(128, 129, ctypes.byref(n)) == lib.CI_ERR_INVALID_ARG


def test_ffn_decode_rejects_bad_arguments_without_a_gpu(lib):
    r = lib.raw.coreinfer_ffn_decode
    F = FAKE
    big = 1 << 30

    def W(**kw):
        base = dict(w_up=F, w_gate=None, b_up=None, w_down=F, b_down=None, core_idx=None, K=16, d=64, N=16,
                    ld_down=0, down_layout=1)
        base.update(kw)
        return ctypes.byref(lib.ci_ffn_weights(**base))

    assert r(F, 1, None, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, W(), 9, 0, F, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, 1, W(), 1, 2, F, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(None, 1, W(), 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, W(), 1, 0, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 0, W(), 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, W(w_up=None), 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, W(), 1, 1, F, F, big, None) == lib.CI_ERR_INVALID_ARG          # SwiGLU without gate
    assert r(F, 1, W(w_gate=F), 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG   # ReLU with gate
    assert r(F, 1, W(d=60), 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 1, W(d=62), 0, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F + 4, 1, W(), 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 1, W(core_idx=F, N=0), 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, W(), 1, 0, F, None, big, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 1, W(), 1, 0, F, F, 64, None) == lib.CI_ERR_WORKSPACE
    # up bias with a gated FFN; layout enum; output-major compact matrix: row length, gathered rows
    assert r(F, 1, W(w_gate=F, b_up=F), 1, 1, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, W(down_layout=2), 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 1, W(down_layout=0, ld_down=8), 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT     # shorter than K
    assert r(F, 1, W(down_layout=0, ld_down=20), 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT    # not whole vectors
    assert r(F, 1, W(down_layout=0, ld_down=16, core_idx=F), 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    st = lib.raw.coreinfer_ffn_decode_status
    assert st(None, F, None) == lib.CI_ERR_INVALID_ARG and st(F, None, None) == lib.CI_ERR_INVALID_ARG
    assert st(F + 4, F, None) == lib.CI_ERR_BAD_LAYOUT


def test_ffn_dense_rejects_bad_arguments_without_a_gpu(lib):
    r = lib.raw.coreinfer_ffn_dense
    F = FAKE
    big = 1 << 30
    # (X, M, w_up, w_gate, b_up, w_down, b_down, layout, dtype, act, d, N, Y, A, ws, ws_bytes, stream)
    assert r(F, 8, F, None, None, F, None, 0, 5, 0, 64, 128, F, None, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, 8, F, None, None, F, None, 2, 1, 0, 64, 128, F, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(None, 8, F, None, None, F, None, 0, 1, 0, 64, 128, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 8, F, None, None, F, None, 0, 1, 0, 64, 128, None, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 8, F, None, None, None, None, 0, 1, 0, 64, 128, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 8, F, None, None, F, None, 0, 1, 1, 64, 128, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 8, F, None, None, F, None, 0, 1, 0, 64, 100, F, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 8, F, None, None, F, None, 0, 1, 0, 64, 128, F, None, None, big, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 8, F, None, None, F, None, 0, 1, 0, 64, 128, F, None, F, 100, None) == lib.CI_ERR_WORKSPACE


def test_next_row_entry_points_reject_bad_arguments_without_a_gpu(lib):
    F = FAKE
    r = lib.raw.coreinfer_count_tokens
    assert r(None, 4, 64, 64, 0.2, F, 0, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 64, 0.2, None, 0, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 64, 1.2, F, 0, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 10, 0.2, F, 0, F, 1 << 20, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 4, 64, 64, 0.2, F, 0, None, 1 << 20, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 4, 64, 64, 0.2, F, 0, F, 16, None) == lib.CI_ERR_WORKSPACE
    r = lib.raw.coreinfer_count_select
    assert r(None, 64, 10, 0.4, F, F, 256, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 64, 70000, 0.4, F, F, 256, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 64, 10, 0.0, F, F, 256, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 64, 10, 0.4, F, None, 256, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 64, 10, 0.4, F, F, 8, None) == lib.CI_ERR_WORKSPACE
    r = lib.raw.coreinfer_group_select
    big = 1 << 20
    assert r(None, 3, 8, 64, 0.2, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 0, 8, 64, 0.2, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 3, 80, 64, 0.2, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 3, 8, 64, 2.0, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 3, 8, 64, 0.2, F, None, F, 16, None) == lib.CI_ERR_WORKSPACE
    r = lib.raw.coreinfer_assign_group
    assert r(F, 4, F, 0, 4, F, F, None) == lib.CI_ERR_INVALID_ARG
    assert r(None, 4, F, 3, 4, F, F, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, None, 3, 4, F, F, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, F, 3, 4, None, F, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, F, 3, 4, F, F + 2, None) == lib.CI_ERR_BAD_LAYOUT
    r = lib.raw.coreinfer_select_hidden
    big = 1 << 22
    assert r(None, 1, 0, 4, 64, 64, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, 0, 4, 64, 64, 0.2, 0.4, None, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 9, 0, 4, 64, 64, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, 1, 7, 4, 64, 64, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, 1, 0, 0, 64, 64, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, 0, 4, 64, 64, 0.0, 0.4, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 1, 0, 4, 64, 32, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F + 1, 1, 0, 4, 64, 64, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F + 2, 0, 0, 4, 64, 64, 0.2, 0.4, F, None, F, big, None) == lib.CI_ERR_BAD_LAYOUT   # fp32 needs 4 bytes
    assert r(F, 1, 0, 4, 64, 64, 0.2, 0.4, F, None, None, big, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 1, 0, 4, 64, 64, 0.2, 0.4, F, None, F, 16, None) == lib.CI_ERR_WORKSPACE
    r = lib.raw.coreinfer_ffn_dense_hidden
    ok = dict(X=F, M=8, up=F, gate=None, bup=None, down=F, bdown=None, layout=0, dt=1, act=0, d=64, N=128, Y=F, H=F,
              ws=F, wsb=big)
    def call(**kw):
        a = dict(ok); a.update(kw)
        return r(a["X"], a["M"], a["up"], a["gate"], a["bup"], a["down"], a["bdown"], a["layout"], a["dt"], a["act"],
                 a["d"], a["N"], a["Y"], a["H"], a["ws"], a["wsb"], None)
    assert call(H=None) == lib.CI_ERR_INVALID_ARG
    assert call(X=None) == lib.CI_ERR_INVALID_ARG
    assert call(down=None) == lib.CI_ERR_INVALID_ARG          # Y wanted without a down matrix
    assert call(act=1) == lib.CI_ERR_INVALID_ARG              # gated FFN without a gate matrix
    assert call(dt=5) == lib.CI_ERR_BAD_DTYPE
    assert call(layout=3) == lib.CI_ERR_BAD_LAYOUT
    assert call(d=60) == lib.CI_ERR_BAD_LAYOUT
    assert call(H=F + 8) == lib.CI_ERR_BAD_LAYOUT
    assert call(ws=None) == lib.CI_ERR_WORKSPACE
    assert call(M=0) == lib.CI_ERR_INVALID_ARG
    r = lib.raw.coreinfer_assign_centroid
    assert r(None, 4, 64, 64, F, 3, F, F, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 64, None, 3, F, F, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 64, F, 3, None, F, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 64, F, 3, F, None, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 0, 64, 64, F, 3, F, F, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 64, F, 0, F, F, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 0, 64, F, 3, F, F, F, 1 << 20, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 4, 64, 32, F, 3, F, F, F, 1 << 20, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 4, 64, 64, F + 2, 3, F, F, F, 1 << 20, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 4, 64, 64, F, 3, F, F, None, 1 << 20, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 4, 64, 64, F, 3, F, F, F, 100, None) == lib.CI_ERR_WORKSPACE
    r = lib.raw.coreinfer_core_similarity
    assert r(F, 4, F, 4, None, None) == lib.CI_ERR_INVALID_ARG
    assert r(None, 4, F, 4, F, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, -1, F, 4, F, None) == lib.CI_ERR_INVALID_ARG
    assert r(F + 2, 4, F, 4, F, None) == lib.CI_ERR_BAD_LAYOUT


def test_union_entry_points_reject_bad_arguments_without_a_gpu(lib):
    F = FAKE
    big = 1 << 30
    r = lib.raw.coreinfer_union_build
    # (core_idx, B, K, N, max_rows, union_idx, union_mask, union_count, ws, ws_bytes, stream)
    assert r(None, 2, 8, 64, 16, F, F, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 9, 8, 64, 64, F, F, F, F, big, None) == lib.CI_ERR_INVALID_ARG      # more than 8 sentences
    assert r(F, 0, 8, 64, 64, F, F, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 2, 80, 64, 64, F, F, F, F, big, None) == lib.CI_ERR_INVALID_ARG     # K > N
    assert r(F, 2, 8, 64, 15, F, F, F, F, big, None) == lib.CI_ERR_INVALID_ARG      # max_rows < min(N, B*K)
    assert r(F, 2, 8, 64, 16, None, F, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 2, 8, 64, 16, F, F, None, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F + 2, 2, 8, 64, 16, F, F, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 2, 8, 64, 16, F, F, F, None, big, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 2, 8, 64, 16, F, F, F, F, 64, None) == lib.CI_ERR_WORKSPACE
    n = ctypes.c_size_t(0)
    assert lib.raw.coreinfer_union_workspace_size(36864, ctypes.byref(n)) == lib.CI_OK and n.value >= 36864 * 4
    assert lib.raw.coreinfer_union_workspace_size(0, ctypes.byref(n)) == lib.CI_ERR_INVALID_ARG

    q = lib.raw.coreinfer_ffn_decode_union_workspace_size
    assert q(8, 36864, 9216, 1, 0, ctypes.byref(n)) == lib.CI_OK
    # partial dots [1 chunk][1][36864][8] + partial sums [8][256][9216], fp32
    assert n.value >= (36864 * 8 + 8 * 256 * 9216) * 4
    assert q(9, 64, 64, 1, 0, ctypes.byref(n)) == lib.CI_ERR_INVALID_ARG
    assert q(8, 64, 60, 1, 0, ctypes.byref(n)) == lib.CI_ERR_BAD_LAYOUT
    assert q(8, 64, 64, 7, 0, ctypes.byref(n)) == lib.CI_ERR_BAD_DTYPE

    r = lib.raw.coreinfer_ffn_decode_union

    def W(**kw):
        base = dict(w_up=F, w_gate=None, b_up=None, w_down=F, b_down=None, core_idx=None, K=0, d=64, N=128)
        base.update(kw)
        return ctypes.byref(lib.ci_ffn_weights(**base))

    # (x, B, w, union_idx, union_mask, union_count, max_rows, dtype, act, y, ws, ws_bytes, stream)
    assert r(F, 2, None, F, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(None, 2, W(), F, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 2, W(), None, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 2, W(), F, F, None, 128, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 9, W(), F, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 2, W(N=0), F, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_INVALID_ARG
    assert r(F, 2, W(), F, F, F, 128, 1, 1, F, F, big, None) == lib.CI_ERR_INVALID_ARG   # SwiGLU without gate
    assert r(F, 2, W(d=60), F, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 2, W(), F + 2, F, F, 128, 1, 0, F, F, big, None) == lib.CI_ERR_BAD_LAYOUT
    assert r(F, 2, W(), F, F, F, 128, 4, 0, F, F, big, None) == lib.CI_ERR_BAD_DTYPE
    assert r(F, 2, W(), F, F, F, 128, 1, 0, F, None, big, None) == lib.CI_ERR_WORKSPACE
    assert r(F, 2, W(), F, F, F, 128, 1, 0, F, F, 1024, None) == lib.CI_ERR_WORKSPACE


def test_development_hook_validation(lib):
    """csrc/coreinfer_dev.h: launch-shape parameters, not declared in the installed header."""
    r = lib.raw.coreinfer_dev_set_param
    assert r(b"no_such_knob", 1) == lib.CI_ERR_INVALID_ARG
    assert r(b"decode_wgs_per_cu", 0) == lib.CI_ERR_INVALID_ARG
    assert r(None, 1) == lib.CI_ERR_INVALID_ARG
    assert r(b"decode_wgs_per_cu", 2) == lib.CI_OK and r(b"decode_wgs_per_cu", 1) == lib.CI_OK
    # no setting makes a call skip its output: the two that did are gone
    assert r(b"decode_skip_reduce", 1) == lib.CI_ERR_INVALID_ARG
    assert r(b"select_debug", 1) == lib.CI_ERR_INVALID_ARG
    assert "coreinfer_dev_set_param" not in _declared_symbols()


def test_development_probes_validate_before_launching(lib):
    """csrc/coreinfer_dev.h: the load-stream probes reject anything that would read outside the buffer."""
    import ctypes
    vp, i64, ci_ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    sp = lib.raw.coreinfer_dev_stream_probe
    sp.restype = ci_
    sp.argtypes = [vp, i64, i64, ci_, ci_, ci_, ci_, ci_, vp, vp]
    F = 0x100000
    assert sp(None, 1 << 20, 1 << 16, 0, 4, 64, 8, 1, F, None) == lib.CI_ERR_INVALID_ARG
    assert sp(F, 1 << 20, 1 << 16, 1, 17, 64, 8, 1, F, None) == lib.CI_ERR_INVALID_ARG   # 17 windows of 64 KB > 1 MB
    assert sp(F, 1 << 20, 512, 0, 4, 64, 8, 1, F, None) == lib.CI_ERR_INVALID_ARG         # window < 16 * threads
    assert sp(F, 1 << 20, 1 << 16, 0, 4, 96, 8, 1, F, None) == lib.CI_ERR_INVALID_ARG     # threads not whole waves
    assert sp(F, 1 << 20, 1 << 16, 0, 4, 64, 3, 1, F, None) == lib.CI_ERR_INVALID_ARG     # depth
    assert sp(F + 8, 1 << 20, 1 << 16, 0, 4, 64, 8, 1, F, None) == lib.CI_ERR_BAD_LAYOUT
    tp = lib.raw.coreinfer_dev_tile_probe
    tp.restype = ci_
    tp.argtypes = [vp, i64, i64, ci_, ci_, ci_, ci_, ci_, vp, vp]
    # 256 rows of 8 KB per workgroup: two workgroups need 4 MB - 8 KB + 64 * 128 bytes
    assert tp(F, (4 << 20) - 1, 8192, 0, 2, 8, 64, 1, F, None) == lib.CI_ERR_INVALID_ARG
    assert tp(F, 1 << 20, 8192, 1, 2, 8, 64, 1, F, None) == lib.CI_ERR_INVALID_ARG        # shared rows: 2 MB needed
    assert tp(F, 1 << 30, 64, 1, 2, 8, 1, 1, F, None) == lib.CI_ERR_INVALID_ARG           # pitch < 128
    assert tp(F, 1 << 30, 8192, 1, 2, 5, 64, 1, F, None) == lib.CI_ERR_INVALID_ARG        # depth
    assert "coreinfer_dev_stream_probe" not in _declared_symbols()


def test_workloads_module_has_the_five_configurations():
    from paper_2410_18311_amd import workloads as wl
    assert len(wl.WORKLOADS) == 5
    c2 = wl.WORKLOADS["opt6.7b_relu_f16"]
    assert (c2.d, c2.N, c2.L, c2.M, c2.alpha, c2.betas) == (4096, 16384, 32, 256, 0.2, (0.4,))
    t = wl.tiny_relu_f32_numpy()
    assert t["w_up"].shape == (1024, 256) and t["w_down"].shape == (256, 1024)
    assert t["x_prefill"].shape == (32, 256) and t["x_decode"].shape == (16, 256)
    small = c2.scaled(d=64, N=128, M=4, L=1)
    w = wl.layer_weights(small, 0)
    assert w["w_up"].shape == (128, 64) and w["w_down"].shape == (64, 128) and w["w_gate"] is None
    again = wl.layer_weights(small, 0)
    assert (w["w_up"] == again["w_up"]).all()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_bench_line_fields_are_built_from_the_documented_pieces():
    """The traffic note is only used for the launch size it was measured at."""
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    assert bench.read_traffic_note("opt6.7b_relu_f16", 0.4, 107410228) is not None
    assert bench.read_traffic_note("opt6.7b_relu_f16", 0.4, 2 * 107410228) is None
    assert bench.read_traffic_note("no_such_workload", 0.4, 1) is None
