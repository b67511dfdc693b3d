"""Shared test plumbing: drives the oracle over a workload with the seeded inputs.

Holds no attention arithmetic of its own.
"""

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
