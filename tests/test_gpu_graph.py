"""A decode step captured into a HIP graph and replayed: every replay appends one token per sequence and attends one
position further, with kernel arguments frozen at capture (lengths are read from device memory, launch plans adapt
on the device).  Every replay is compared with the CPU oracle; afterwards the host-side bookkeeping must agree with
the device again and eager calls carry on."""

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


@pytest.mark.parametrize("Hq,Hkv,W,lens,chunk_keys,paged,out_dtype,two_call", [
    (8, 2, 48, [20, 700, 3], 0, 0, "f32", False),        # ragged: balanced launches; a ring that wraps; block crossings
    (8, 2, 48, [20, 700, 3], 0, 64, "bf16", False),      # the same with paged full caches
    (8, 2, 100, [3000], 0, 0, "f32", False),             # one long sequence: split-K plan frozen at capture
    (8, 2, 64, [250, 251], 128, 0, "f32", False),        # fixed chunk length: chunk count grows past the captured grid
    (4, 4, 33, [31, 95], 0, 0, "f32", True),             # append_kv + decode as two captured launches
])
def test_captured_decode_step_replayed_40_times(mx, Hq, Hkv, W, lens, chunk_keys, paged, out_dtype, two_call):
    B, R = len(lens), 40
    # full writer, ring writer, ring reader, full reader, sliding reader of the full cache
    layers = [(0, 0, 0), (1, W, 1), (1, W, 1), (0, 0, 0), (1, W, 0)]
    cap = [n + R + 3 for n in lens]
    kw = dict(page_tokens=paged, pool_tokens=sum((c + paged - 1) // paged for c in cap) * paged) if paged else {}
    lay = mx.Layout(layers, B, Hq, Hkv, D, capacity=cap, kv_dtype="bf16", out_dtype=out_dtype, **kw)
    lay.set_param(mx.PARAM_CHUNK_KEYS, chunk_keys)
    ora = OracleStack([LayerSpec(*t) for t in layers], B, Hq, Hkv, D)
    writers = [li for li in range(len(layers)) if lay.cache_of(li)[1]]
    for li in writers:
        k = wl.randn(100 + li, (sum(lens), Hkv, D), torch.bfloat16, DEV)
        v = wl.randn(200 + li, (sum(lens), Hkv, D), torch.bfloat16, DEV)
        lay.load_kv(li, k, v, lens)
        ora.load(li, to_f64(k), to_f64(v), lens)
    # static buffers the captured launches read and write
    qs = [torch.zeros((B, Hq, D), dtype=torch.bfloat16, device=DEV) for _ in layers]
    ks = {li: torch.zeros((B, Hkv, D), dtype=torch.bfloat16, device=DEV) for li in writers}
    vs = {li: torch.zeros((B, Hkv, D), dtype=torch.bfloat16, device=DEV) for li in writers}
    outs = [torch.zeros((B, Hq, D), dtype=lay.out_torch, device=DEV) for _ in layers]

    def step():
        for li in range(len(layers)):
            if li in ks:
                if two_call:
                    lay.append_kv(li, ks[li], vs[li])
                    lay.decode(li, qs[li], outs[li])
                else:
                    lay.append_decode(li, ks[li], vs[li], qs[li], outs[li])
            else:
                lay.decode(li, qs[li], outs[li])

    def fill_inputs(t):
        for li in range(len(layers)):
            qs[li].copy_(wl.randn(1000 + 10 * t + li, (B, Hq, D), torch.bfloat16, DEV))
            if li in ks:
                ks[li].copy_(wl.randn(3000 + 10 * t + li, (B, Hkv, D), torch.bfloat16, DEV))
                vs[li].copy_(wl.randn(5000 + 10 * t + li, (B, Hkv, D), torch.bfloat16, DEV))

    def check(t, what):
        for li in range(len(layers)):
            if li in ks:
                ora.append(li, to_f64(ks[li]), to_f64(vs[li]))
            assert_matches(outs[li], ora.decode(li, to_f64(qs[li])), "bf16", "%s %d layer %d" % (what, t, li))

    # one eager step first (graph and eager calls mix freely)
    fill_inputs(0)
    step()
    torch.cuda.synchronize()
    check(0, "eager step")

    lay.reserve_steps(R)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for r in range(R):
        fill_inputs(1 + r)
        torch.cuda.synchronize()
        graph.replay()
        if r > 0:
            lay.account_replays(1)
        torch.cuda.synchronize()
        check(1 + r, "replay")
    # host and device bookkeeping agree, cache contents are those of R + 1 appends
    for li in writers:
        ci, _ = lay.cache_of(li)
        assert lay.device_lens(ci) == [ora.seq_len(li, b) for b in range(B)]
        assert [lay.seq_len(ci, b) for b in range(B)] == [ora.seq_len(li, b) for b in range(B)]
        for b in range(B):
            K, V = ora.history(li, b)
            for slot, pos in ora.cache_view(li, b)[-(R + 2):]:
                k_row, v_row = lay.read_cache(ci, b, Hkv - 1, slot)
                assert np.array_equal(k_row.double().numpy(), K[pos, Hkv - 1]), (li, b, slot, pos)
                assert np.array_equal(v_row.double().numpy(), V[pos, Hkv - 1]), (li, b, slot, pos)
    # eager calls carry on from there
    fill_inputs(900)
    step()
    torch.cuda.synchronize()
    check(900, "eager step after the replays")
    # the reservation is what makes replays safe: one more than the capacity allows is refused, nothing changes
    with pytest.raises(mx.MixAttnError) as ei:
        lay.reserve_steps(2)
    assert ei.value.status == -5
    lay.reserve_steps(1)
    with pytest.raises(mx.MixAttnError) as ei:
        lay.account_replays(2)
    assert ei.value.status == -5
    del graph
    lay.close()
