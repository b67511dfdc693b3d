"""Shared test plumbing: drives the oracle over a workload with the seeded inputs.

Holds no attention arithmetic of its own.
"""

import os

import numpy as np
import torch

from oracle.mixattn_oracle import LayerSpec, OracleStack
from paper_2409_15012_amd import workloads as wl


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_for(w: wl.Workload, **kw) -> OracleStack:
    return OracleStack([LayerSpec(*t) for t in w.layers], w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, **kw)


def config0_inputs():
    """Tensors of the tiny fp32 configuration: per layer prefill q (and k, v for writers),
    then per decode step per layer q (and k, v for writers).  All on the CPU."""
    w = wl.config(0)
    B, S, Hq, Hkv, d = w.batch, w.prefill_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    writers = set(w.writer_layers())
    pre = []
    for li in range(len(w.layers)):
        q = wl.randn(wl.layer_seed(w.seed, li, "q"), (B, S, Hq, d), w.torch_dtype)
        k = v = None
        if li in writers:
            k = wl.randn(wl.layer_seed(w.seed, li, "k"), (B, S, Hkv, d), w.torch_dtype)
            v = wl.randn(wl.layer_seed(w.seed, li, "v"), (B, S, Hkv, d), w.torch_dtype)
        pre.append((q, k, v))
    steps = []
    for t in range(1, w.decode_steps + 1):
        per_layer = []
        for li in range(len(w.layers)):
            q = wl.randn(wl.layer_seed(w.seed, li, "q", t), (B, Hq, d), w.torch_dtype)
            k = v = None
            if li in writers:
                k = wl.randn(wl.layer_seed(w.seed, li, "k", t), (B, Hkv, d), w.torch_dtype)
                v = wl.randn(wl.layer_seed(w.seed, li, "v", t), (B, Hkv, d), w.torch_dtype)
            per_layer.append((q, k, v))
        steps.append(per_layer)
    return w, pre, steps


def config0_oracle():
    """Oracle outputs for the tiny configuration: (prefill outs per layer, decode outs [step][layer], stack)."""
    w, pre, steps = config0_inputs()
    st = oracle_for(w)
    pre_out = []
    for li, (q, k, v) in enumerate(pre):
        pre_out.append(st.prefill(li, to_f64(q), None if k is None else to_f64(k), None if v is None else to_f64(v)))
    dec_out = []
    for per_layer in steps:
        outs = []
        for li, (q, k, v) in enumerate(per_layer):
            if k is not None:
                st.append(li, to_f64(k), to_f64(v))
            outs.append(st.decode(li, to_f64(q)))
        dec_out.append(outs)
    return pre_out, dec_out, st


# ----------------------------------------------------------------- comparison helpers
BF16_MAX_ABS = 2e-3   # bf16 inputs, fp32 accumulation and fp32 output
BF16_REL_L2 = 1e-3
F32_TOL = 1e-5
# bf16 OUTPUT: the fp32 result is rounded once more, to 8 significant bits.  That rounding alone moves an element
# by up to 2^-9 |x| (half an ulp), which exceeds 2e-3 as soon as |x| >= 1, so the bound per element becomes
# 2e-3 + 2^-8 |ref| (one ulp of slack: the value being rounded is itself off by up to 2e-3) and the relative L2
# bound 1e-3 + 2^-9 (every element within 2^-9 of its magnitude bounds the L2 ratio by the same figure).
BF16_OUT_ULP = 2.0 ** -8


def errors(out: torch.Tensor, ref: np.ndarray):
    o = to_f64(out)
    diff = o - ref
    max_abs = float(np.abs(diff).max()) if diff.size else 0.0
    denom = float(np.linalg.norm(ref.ravel()))
    rel_l2 = float(np.linalg.norm(diff.ravel())) / denom if denom > 0 else 0.0
    return max_abs, rel_l2


def _report(what, dtype, out_dtype, max_abs, rel_l2):
    """With MIXATTN_TEST_REPORT=<file> every comparison appends its errors there (how far the tests are from their
    bounds; nothing reads the file)."""
    path = os.environ.get("MIXATTN_TEST_REPORT")
    if path:
        with open(path, "a") as f:
            f.write("%s\t%s\t%s\t%.4g\t%.4g\n" % (what, dtype, out_dtype, max_abs, rel_l2))


def assert_matches(out: torch.Tensor, ref: np.ndarray, dtype: str, what: str = ""):
    assert not torch.isnan(out).any(), "NaN in output " + what
    max_abs, rel_l2 = errors(out, ref)
    _report(what, dtype, str(out.dtype), max_abs, rel_l2)
    if out.dtype == torch.bfloat16:
        base_abs, base_rel = (F32_TOL, F32_TOL) if dtype == "f32" else (BF16_MAX_ABS, BF16_REL_L2)
        excess = np.abs(to_f64(out) - ref) - (base_abs + BF16_OUT_ULP * np.abs(ref))
        assert float(excess.max()) <= 0.0 and rel_l2 <= base_rel + 2.0 ** -9, \
            "%s (bf16 output): worst excess over the bound %.3g, max_abs %.3g rel_l2 %.3g" % (
                what, float(excess.max()), max_abs, rel_l2)
        return max_abs, rel_l2
    if dtype == "f32":
        assert max_abs <= F32_TOL and rel_l2 <= F32_TOL, "%s: max_abs %.3g rel_l2 %.3g" % (what, max_abs, rel_l2)
    else:
        assert max_abs <= BF16_MAX_ABS and rel_l2 <= BF16_REL_L2, "%s: max_abs %.3g rel_l2 %.3g" % (what, max_abs, rel_l2)
    return max_abs, rel_l2
