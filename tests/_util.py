"""Helpers shared by the GPU parity tests (conversion and tolerances only)."""
import numpy as np
import torch

# max |y_gpu - y_oracle| <= TOL * rms(y_oracle): the bar set for this build
# (2e-2 for 16-bit element types, 1e-5 for fp32).
TOL = {torch.float32: 1e-5, torch.float16: 2e-2, torch.bfloat16: 2e-2}


def f64(t):
    """Exact float64 copy of a tensor (any device / dtype), or None."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float64).numpy()


def score_bound(dtype, act, A_ref, X=None, w=None):
    """Largest absolute error allowed on the fp32 prefill scores.  fp32 layers: the fp32 bar,
    max(1e-5, 8 sqrt(d) 2^-24) (the second term is the rounding of a length-d fp32 sum, which
    passes 1e-5 beyond d = 440), times the scale of what is rounded -- the RMS of the scores for
    ReLU; for SwiGLU, whose score is the product of two rounded dots (its error grows with the
    dots, and the RMS of a SiLU-gated product is several times smaller than theirs),
    RMS(gate dot) * RMS(up dot).  16-bit inputs: 1e-4 of the scores' RMS."""
    rms = float(np.sqrt(np.mean(np.asarray(A_ref, dtype=np.float64) ** 2)))
    if dtype != torch.float32:
        return 1e-4 * rms
    d = X.shape[-1]
    bar = max(1e-5, 8.0 * np.sqrt(d) * 2.0 ** -24)
    if act == "swiglu":
        Xd = f64(X)
        g = Xd @ f64(w["w_gate"]).T
        u = Xd @ f64(w["w_up"]).T
        return bar * max(rms, float(np.sqrt(np.mean(g ** 2)) * np.sqrt(np.mean(u ** 2))))
    return bar * rms


def assert_close_rms(got, want, dtype, what=""):
    got = f64(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    rms = float(np.sqrt(np.mean(want ** 2)))
    err = float(np.max(np.abs(got - want))) if want.size else 0.0
    bound = TOL[dtype] * max(rms, 1e-30)
    assert err <= bound, f"{what}: max abs err {err:.3e} > {TOL[dtype]} * rms ({rms:.3e})"
    return err / max(rms, 1e-30)


def rand_weights(d, N, dtype, act, layout, seed, device, bias=True):
    """Random FFN layer (N(0, 0.02^2) weights like the workloads, non-constant
    biases so that a dropped or mis-indexed bias shows)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)

    def rn(*shape, scale=0.02):
        return (torch.randn(*shape, generator=g) * scale).to(dtype).to(device)

    w = {"w_up": rn(N, d), "w_gate": rn(N, d) if act == "swiglu" else None,
         "w_down": rn(d, N) if layout == "out_major" else rn(N, d)}
    if bias and act == "relu":
        w["b_up"] = rn(N, scale=0.1)
        w["b_down"] = rn(d, scale=0.1)
    else:
        w["b_up"] = None
        w["b_down"] = rn(d, scale=0.1) if bias else None
    return w


def down_out_major64(w, layout):
    """w_down as float64 [d, N] whatever the stored layout."""
    m = f64(w["w_down"])
    return m if layout == "out_major" else m.T
