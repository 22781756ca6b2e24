"""coreinfer_ffn_decode_static -- the decode entry point that allocates nothing -- against
coreinfer_ffn_decode on the same inputs: two calls in a row on the library's static scratch, the
second with a smaller input, for the neuron-major (two launches), output-major (single launch)
and gathered forms.  Same kernels on both sides, so the outputs must be identical bit for bit;
the first is also held to the oracle."""
import numpy as np
import pytest
import torch

from oracle import coreinfer_oracle as orc
from tests._util import assert_close_rms, down_out_major64, f64, rand_weights

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


def _case(lib, d, N, K, B, dtype, act, form, seed):
    w = rand_weights(d, N, dtype, act, "out_major" if form != "gathered" else "neuron_major", seed=seed, device=DEV)
    rng = np.random.default_rng(seed)
    x = torch.randn(B, d, generator=torch.Generator().manual_seed(seed)).to(dtype).to(DEV)
    if form == "gathered":
        sets = np.stack([np.sort(rng.choice(N, size=K, replace=False)) for _ in range(B)])
        idx = torch.from_numpy(sets.astype(np.int32)).to(DEV)
        desc = lib.make_weights(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], w["b_down"], core_idx=idx)
        keep = (w, idx)
    else:
        S = np.sort(rng.choice(N, size=K, replace=False))
        sets = np.stack([S] * B)
        c = lib.compact(w["w_up"], w["w_gate"], w["b_up"], w["w_down"], "out_major", act,
                        torch.from_numpy(S.astype(np.int32)).to(DEV),
                        down_c_layout="out_major" if form == "single" else "neuron_major")
        desc = lib.make_compact_weights(c, w["b_down"])
        keep = (w, c)
    return w, sets, x, desc, keep


def _oracle(act, x, S, w, layout):
    Wd = down_out_major64(w, layout)
    if act == "relu":
        return orc.ffn_relu(f64(x), S, f64(w["w_up"]), f64(w["b_up"]), Wd, f64(w["b_down"]))
    return orc.ffn_swiglu(f64(x), S, f64(w["w_gate"]), f64(w["w_up"]), Wd, f64(w["b_down"]))


@pytest.mark.parametrize("form,dt,act", [("two", torch.float16, "relu"), ("single", torch.bfloat16, "swiglu"),
                                         ("single", torch.float32, "relu"), ("gathered", torch.float16, "relu")])
def test_static_scratch_decode_matches_workspace_decode(lib, form, dt, act):
    shapes = [(1024, 3000, 1201, 3), (512, 900, 77, 1)]     # the second call is the smaller one
    status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    for call, (d, N, K, B) in enumerate(shapes):
        _say("no-alloc decode case", form, dt, act, "call", call, d, N, K, B)
        w, sets, x, desc, keep = _case(lib, d, N, K, B, dt, act, form, seed=100 + call)
        y_ws = lib.ffn_decode(x, desc, act)                      # existing entry point, its own zeroed workspace
        y_st = torch.empty_like(x)
        lib.ffn_decode_static(x, desc, act, y=y_st, status=status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert torch.equal(y_st, y_ws), f"{form}: call {call} differs from coreinfer_ffn_decode"
        layout = "neuron_major" if form == "gathered" else "out_major"
        for b in range(B):
            assert_close_rms(y_st[b], _oracle(act, x[b], sets[b], w, layout), dt, f"{form} call {call} sentence {b}")


def test_static_scratch_rejects_sizes_beyond_its_limit(lib):
    """Nothing is launched and no memory is touched: the pointers only need to look valid."""
    import ctypes
    dummy = torch.zeros(64, dtype=torch.float16, device=DEV)
    big = lib.ci_ffn_weights(dummy.data_ptr(), None, None, dummy.data_ptr(), None, None, 200000, 64, 200000, 200000,
                             lib.CI_DOWN_OUT_MAJOR)
    rc = lib.raw.coreinfer_ffn_decode_static(dummy.data_ptr(), 1, ctypes.byref(big), lib.CI_F16, lib.CI_ACT_RELU,
                                             dummy.data_ptr(), None, None)
    assert rc == lib.CI_ERR_WORKSPACE
    wide = lib.ci_ffn_weights(dummy.data_ptr(), None, None, dummy.data_ptr(), None, None, 4096, 32768, 4096, 0,
                              lib.CI_DOWN_NEURON_MAJOR)
    rc = lib.raw.coreinfer_ffn_decode_static(dummy.data_ptr(), 8, ctypes.byref(wide), lib.CI_F16, lib.CI_ACT_RELU,
                                             dummy.data_ptr(), None, None)
    assert rc == lib.CI_ERR_WORKSPACE
