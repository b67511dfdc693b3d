"""mixattn_decode_noalloc (split-K partials in the library's static device area, no allocation) against
mixattn_decode (partials in the layout's scratch): two calls in a row, the second on a smaller input, so that the
second finds the first call's contents in the shared area."""

import numpy as np
import pytest
import torch

from helpers import assert_matches, to_f64
from oracle.mixattn_oracle import LayerSpec, OracleStack
from paper_2409_15012_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
D = 128


@pytest.fixture(scope="module")
def mx():
    from paper_2409_15012_amd import binding
    binding.load()
    return binding


def _stack(mx, B, Hq, Hkv, W, lens, out_dtype):
    # full writer, ring writer, ring reader, sliding reader of the full cache
    layers = [(0, 0, 0), (1, W, 1), (1, W, 1), (1, 200, 0)]
    lay = mx.Layout(layers, B, Hq, Hkv, D, capacity=[n + 1 for n in lens], kv_dtype="bf16", out_dtype=out_dtype)
    ora = OracleStack([LayerSpec(*t) for t in layers], B, Hq, Hkv, D)
    for li in (0, 1):
        k = wl.randn(31 + li + B, (sum(lens), Hkv, D), torch.bfloat16, DEV)
        v = wl.randn(41 + li + B, (sum(lens), Hkv, D), torch.bfloat16, DEV)
        lay.load_kv(li, k, v, lens)
        ora.load(li, to_f64(k), to_f64(v), lens)
    return layers, lay, ora


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_noalloc_decode_matches_decode_two_calls_second_smaller(mx, out_dtype):
    Hq, Hkv = 8, 2
    big = _stack(mx, 3, Hq, Hkv, 1024, [6000, 2500, 4100], out_dtype)   # every launch is split: partials in use
    small = _stack(mx, 2, Hq, Hkv, 1024, [900, 1300], out_dtype)       # fewer rows, fewer chunks, same area
    for name, (layers, lay, ora) in (("first call", big), ("second call, smaller", small)):
        lay.set_param(mx.PARAM_BALANCED, 0)   # same per-sequence chunks in both entry points: results bit-identical
        for li in range(len(layers)):
            q = wl.randn(500 + li + lay.batch, (lay.batch, Hq, D), torch.bfloat16, DEV)
            want = lay.decode(li, q)
            got = torch.full_like(want, float("nan"))
            lay.decode_noalloc(li, q, got)
            torch.cuda.synchronize()
            assert torch.equal(got, want), "%s layer %d: differs from mixattn_decode" % (name, li)
            assert_matches(got, ora.decode(li, to_f64(q)), "bf16", "%s layer %d" % (name, li))
        lay.set_param(mx.PARAM_BALANCED, 1)   # default plan of mixattn_decode (balanced runs): same result to rounding
        q = wl.randn(600 + lay.batch, (lay.batch, Hq, D), torch.bfloat16, DEV)
        want = lay.decode(0, q)
        got = torch.empty_like(want)
        lay.decode_noalloc(0, q, got)
        assert float((got.float() - want.float()).abs().max()) <= (2e-5 if out_dtype == "f32" else 2.0 ** -7)
    # a call whose partials would not fit the static area is refused before anything is enqueued
    B, n = 64, 40000
    lay = mx.Layout([(0, 0, 0)], B, 32, 8, D, capacity=[n] * B, kv_dtype="bf16", out_dtype=out_dtype)
    k = torch.zeros((B * 64, 8, D), dtype=torch.bfloat16, device=DEV)
    lay.load_kv(0, k, k, [64] * B)
    lay.account_replays(n - 64)           # host-side lengths only: plans as for 40000-token sequences
    lay.set_param(mx.PARAM_CHUNK_KEYS, 1024)   # 40 chunks x 2048 rows x 520 B = 42 MB > 16 MiB
    q = torch.zeros((B, 32, D), dtype=torch.bfloat16, device=DEV)
    out = torch.full((B, 32, D), 7.0, dtype=lay.out_torch, device=DEV)
    with pytest.raises(mx.MixAttnError) as ei:
        lay.decode_noalloc(0, q, out)
    assert ei.value.status == mx.ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    for _, l, _ in (big, small):
        l.close()
    lay.close()


def test_noalloc_decode_inside_a_captured_graph(mx):
    """The callers this entry point is for include code under graph capture: the calls of a reader step are captured
    (nothing in them allocates, synchronises or records a memset) and replayed three times with new queries, with the
    program's own eager work between the replays; every replay must equal the eager result for the same queries."""
    Hq, Hkv = 8, 2
    layers, lay, ora = _stack(mx, 3, Hq, Hkv, 1024, [6000, 2500, 4100], "f32")
    lay.set_param(mx.PARAM_BALANCED, 0)
    qs = [torch.zeros((lay.batch, Hq, D), dtype=torch.bfloat16, device=DEV) for _ in layers]
    outs = [torch.zeros((lay.batch, Hq, D), dtype=torch.float32, device=DEV) for _ in layers]

    def step():
        for li in range(len(layers)):
            lay.decode_noalloc(li, qs[li], outs[li])

    step()   # warm-up outside the capture (kernel modules, planner memo)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for r in range(3):
        for li in range(len(layers)):
            qs[li].copy_(wl.randn(900 + 10 * r + li, (lay.batch, Hq, D), torch.bfloat16, DEV))
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        for li in range(len(layers)):
            want = lay.decode(li, qs[li])          # eager, the layout's own scratch
            torch.cuda.synchronize()
            assert torch.equal(got[li], want), "replay %d layer %d differs from the eager call" % (r, li)
            assert_matches(got[li], ora.decode(li, to_f64(qs[li])), "bf16", "replay %d layer %d" % (r, li))
    del graph
    lay.close()
