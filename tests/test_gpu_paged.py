"""GPU parity for paged layouts (FULL caches held as pools of pages): every result must equal the contiguous
layout's bit for bit (same kernels, same order of arithmetic; only the addresses differ) and match the CPU oracle;
pages are recycled out of order on purpose."""

import numpy as np
import pytest
import torch

from helpers import assert_matches, to_f64
from oracle import mixattn_oracle as mo
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


def _layers(W):
    # full (cache 0), sliding (1), sliding sharing 1, full sharing 0, sliding layer reading the full cache 0
    return [(0, 0, 0), (1, W, 1), (1, W, 1), (0, 0, 0), (1, W, 0)]


def _check_full_cache(lay, ora, layer, heads):
    ci, _ = lay.cache_of(layer)
    for b in range(lay.batch):
        assert lay.seq_len(ci, b) == ora.seq_len(layer, b)
        K, V = ora.history(layer, b)
        for pos in range(K.shape[0]):
            for h in heads:
                k_row, v_row = lay.read_cache(ci, b, h, pos)
                assert np.array_equal(k_row.double().numpy(), K[pos, h]), (b, h, pos)
                assert np.array_equal(v_row.double().numpy(), V[pos, h]), (b, h, pos)
    assert lay.device_lens(ci) == [ora.seq_len(layer, b) for b in range(lay.batch)]


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("page_tokens", [32, 64, 256, 1024])
def test_paged_decode_and_prefill_equal_contiguous_and_oracle(mx, page_tokens, out_dtype):
    Hq, Hkv, W, B = 8, 2, 48, 3
    layers = _layers(W)
    lens = [5, 700, 257]
    chunk = [33, 1, 130]          # a varlen prefill chunk on top of the loaded histories
    steps = 3
    cap = [lens[b] + chunk[b] + steps for b in range(B)]
    pool = sum((c + page_tokens - 1) // page_tokens for c in cap) * page_tokens
    lays = [mx.Layout(layers, B, Hq, Hkv, D, capacity=cap, kv_dtype="bf16", out_dtype=out_dtype),
            mx.Layout(layers, B, Hq, Hkv, D, capacity=cap, kv_dtype="bf16", out_dtype=out_dtype,
                      page_tokens=page_tokens, pool_tokens=pool)]
    ora = OracleStack([LayerSpec(*t) for t in layers], B, Hq, Hkv, D)
    for li in (0, 1):
        k = wl.randn(10 + li, (sum(lens), Hkv, D), torch.bfloat16, DEV)
        v = wl.randn(20 + li, (sum(lens), Hkv, D), torch.bfloat16, DEV)
        for lay in lays:
            lay.load_kv(li, k, v, lens)
        ora.load(li, to_f64(k), to_f64(v), lens)
    # varlen prefill chunk through all layers
    T = sum(chunk)
    kv = {}
    for li in range(len(layers)):
        wr = lays[0].writer_of(li)
        if wr == li:
            kv[li] = (wl.randn(30 + li, (T, Hkv, D), torch.bfloat16, DEV), wl.randn(40 + li, (T, Hkv, D), torch.bfloat16, DEV))
        q = wl.randn(50 + li, (T, Hq, D), torch.bfloat16, DEV)
        k, v = kv[wr]
        reuse = wr == li - 1
        outs = [lay.prefill_varlen(li, q, None if reuse else k, None if reuse else v, chunk) for lay in lays]
        assert torch.equal(outs[0], outs[1]), "prefill layer %d differs between paged and contiguous" % li
        ref = ora.prefill_ragged(li, to_f64(q), to_f64(k) if wr == li else None, to_f64(v) if wr == li else None, chunk)
        assert_matches(outs[1], ref, "bf16", "prefill layer %d" % li)
    # decode steps: two-call form and fused form alternate
    for t in range(steps):
        for li in range(len(layers)):
            q = wl.randn(100 + 10 * t + li, (B, Hq, D), torch.bfloat16, DEV)
            if lays[0].writer_of(li) == li:
                k = wl.randn(200 + 10 * t + li, (B, Hkv, D), torch.bfloat16, DEV)
                v = wl.randn(300 + 10 * t + li, (B, Hkv, D), torch.bfloat16, DEV)
                ora.append(li, to_f64(k), to_f64(v))
                if t % 2 == 0:
                    outs = [lay.append_decode(li, k, v, q) for lay in lays]
                else:
                    for lay in lays:
                        lay.append_kv(li, k, v)
                    outs = [lay.decode(li, q) for lay in lays]
            else:
                outs = [lay.decode(li, q) for lay in lays]
            assert torch.equal(outs[0], outs[1]), "decode step %d layer %d differs" % (t, li)
            assert_matches(outs[1], ora.decode(li, to_f64(q)), "bf16", "decode step %d layer %d" % (t, li))
    _check_full_cache(lays[1], ora, 0, heads=[0, Hkv - 1])
    live = lays[1].kv_bytes_live()
    assert live == lays[0].kv_bytes_live()
    for lay in lays:
        lay.close()


def test_pages_are_recycled_out_of_order_and_the_pool_runs_dry(mx):
    """Three sequence slots over a pool that cannot hold all of them at full length: requests come and go, pages
    change hands in scrambled order, and a call that would overdraw the pool fails without touching anything."""
    Hq, Hkv, W, B, page = 8, 2, 40, 3, 64
    layers = [(0, 0, 0), (1, W, 1), (0, 0, 0)]
    cap = [600] * B
    pool_pages = 12                      # 768 tokens for 3 x 600 of capacity
    lay = mx.Layout(layers, B, Hq, Hkv, D, capacity=cap, kv_dtype="bf16", out_dtype="f32",
                    page_tokens=page, pool_tokens=pool_pages * page)
    ora = OracleStack([LayerSpec(*t) for t in layers], B, Hq, Hkv, D)
    seed = [1000]

    def feed(lens):
        T = sum(lens)
        kv = {}
        for li in range(len(layers)):
            wr = lay.writer_of(li)
            if wr == li:
                seed[0] += 2
                kv[li] = (wl.randn(seed[0], (T, Hkv, D), torch.bfloat16, DEV), wl.randn(seed[0] + 1, (T, Hkv, D), torch.bfloat16, DEV))
            seed[0] += 1
            q = wl.randn(seed[0], (T, Hq, D), torch.bfloat16, DEV)
            k, v = kv[wr]
            out = lay.prefill_varlen(li, q, k, v, lens)
            ref = ora.prefill_ragged(li, to_f64(q), to_f64(k) if wr == li else None, to_f64(v) if wr == li else None, lens)
            assert_matches(out, ref, "bf16", "layer %d lens %s" % (li, lens))

    def step():
        for li in range(len(layers)):
            seed[0] += 3
            q = wl.randn(seed[0], (B, Hq, D), torch.bfloat16, DEV)
            if lay.writer_of(li) == li:
                k = wl.randn(seed[0] + 1, (B, Hkv, D), torch.bfloat16, DEV)
                v = wl.randn(seed[0] + 2, (B, Hkv, D), torch.bfloat16, DEV)
                out = lay.append_decode(li, k, v, q)
                ora.append(li, to_f64(k), to_f64(v))
            else:
                out = lay.decode(li, q)
            assert_matches(out, ora.decode(li, to_f64(q)), "bf16", "decode layer %d" % li)

    feed([200, 130, 65])     # 4 + 3 + 2 pages
    step()
    lay.release_sequence(1); ora.release_sequence(1)     # its 3 pages go back
    feed([100, 0, 130])      # sequence 0: 300 tokens (5 pages: takes one of the freed), sequence 2: 195 (4 pages)
    lay.release_sequence(0); ora.release_sequence(0)
    feed([10, 320, 0])       # sequence 1 restarts on pages freed by 1 and 0, out of order
    step()
    _check_full_cache(lay, ora, 0, heads=[1])
    # the pool holds 12 pages: sequence 0 has 1, sequence 1 has 6 (321 tokens), sequence 2 has 4 (196): one left
    q = wl.randn(1, (200, Hq, D), torch.bfloat16, DEV)
    k = wl.randn(2, (200, Hkv, D), torch.bfloat16, DEV)
    before = [lay.seq_len(0, b) for b in range(B)]
    with pytest.raises(mx.MixAttnError) as ei:
        lay.prefill_varlen(0, q, k, k, [200, 0, 0])      # needs 3 more pages
    assert ei.value.status == -5
    assert [lay.seq_len(0, b) for b in range(B)] == before
    step()                                                 # nothing was disturbed
    # beyond a sequence's own capacity (the table width): CAPACITY as for a contiguous layout
    lay.release_sequence(1); ora.release_sequence(1)
    lay.release_sequence(2); ora.release_sequence(2)
    q = wl.randn(3, (601, Hq, D), torch.bfloat16, DEV)
    k = wl.randn(4, (601, Hkv, D), torch.bfloat16, DEV)
    with pytest.raises(mx.MixAttnError) as ei:
        lay.prefill_varlen(0, q, k, k, [0, 601, 0])
    assert ei.value.status == -5
    lay.reset()
    assert lay.kv_bytes_live() == 0
    lay.close()


def test_paged_layout_rejects_what_it_cannot_hold(mx):
    layers = [(0, 0, 0), (1, 16, 1)]
    for kwargs in (dict(page_tokens=48, pool_tokens=4800), dict(page_tokens=16, pool_tokens=1600),
                   dict(page_tokens=64, pool_tokens=32)):
        with pytest.raises(mx.MixAttnError) as ei:
            mx.Layout(layers, 1, 8, 2, D, capacity=[100], kv_dtype="bf16", **kwargs)
        assert ei.value.status == -2
    with pytest.raises(mx.MixAttnError) as ei:   # row-major shapes have no paged form
        mx.Layout(layers, 1, 4, 4, 64, capacity=[100], kv_dtype="f32", page_tokens=64, pool_tokens=640)
    assert ei.value.status == -2


@pytest.mark.parametrize("kv_dtype,d,paged,balanced", [("bf16", 128, 0, 1), ("bf16", 128, 64, 2), ("bf16", 128, 0, 0),
                                                       ("f32", 64, 0, 1)])
def test_idle_slots_of_the_batch_are_passed_over(mx, kv_dtype, d, paged, balanced):
    """Requests end at different times: a released sequence is idle (decode-step tokens pass over it, its output
    rows are zero, its batch mates are unaffected) until a prompt chunk starts a new request in its slot."""
    Hq, Hkv, W, B = 8, 2, 40, 4
    tdt = torch.bfloat16 if kv_dtype == "bf16" else torch.float32
    tol = "bf16" if kv_dtype == "bf16" else "f32"
    # full writer, ring writer, ring reader, full reader, sliding reader of the full cache
    layers = [(0, 0, 0), (1, W, 1), (1, W, 1), (0, 0, 0), (1, W, 0)]
    lens = [300, 77, 5, 130]
    cap = [n + 400 for n in lens]
    kw = {}
    if paged:
        kw = dict(page_tokens=paged, pool_tokens=sum((c + paged - 1) // paged for c in cap) * paged)
    lay = mx.Layout(layers, B, Hq, Hkv, d, capacity=cap, kv_dtype=kv_dtype, out_dtype="f32", **kw)
    lay.set_param(mx.PARAM_BALANCED, balanced)
    ora = OracleStack([LayerSpec(*t) for t in layers], B, Hq, Hkv, d)
    for li in (0, 1):
        k = wl.randn(10 + li, (sum(lens), Hkv, d), tdt, DEV)
        v = wl.randn(20 + li, (sum(lens), Hkv, d), tdt, DEV)
        lay.load_kv(li, k, v, lens)
        ora.load(li, to_f64(k), to_f64(v), lens)
    seed = [5000]

    def step(fused, group=False):
        seed[0] += 10
        outs = {}
        for li in range(len(layers)):
            q = wl.randn(seed[0] + li, (B, Hq, d), tdt, DEV)
            if lay.writer_of(li) == li:
                k = wl.randn(seed[0] + 100 + li, (B, Hkv, d), tdt, DEV)
                v = wl.randn(seed[0] + 200 + li, (B, Hkv, d), tdt, DEV)
                ora.append(li, to_f64(k), to_f64(v))
                if group and li == 1:
                    q2 = torch.stack([q, wl.randn(seed[0] + 2, (B, Hq, d), tdt, DEV)]).contiguous()
                    out2 = lay.decode_group([1, 2], q2, k, v)
                    outs[1], outs[2] = (out2[0], q2[0]), (out2[1], q2[1])
                    continue
                if fused:
                    out = lay.append_decode(li, k, v, q)
                else:
                    lay.append_kv(li, k, v)
                    out = lay.decode(li, q)
            elif group and li == 2:
                continue
            else:
                out = lay.decode(li, q)
            outs[li] = (out, q)
        for li, (out, q) in outs.items():
            ref = ora.decode(li, to_f64(q))
            assert_matches(out, ref, tol, "layer %d" % li)
            for b in range(B):
                if ora.is_idle(li, b):
                    assert torch.count_nonzero(out[b]) == 0, (li, b)

    step(fused=True)
    for b in (1, 3):
        lay.release_sequence(b); ora.release_sequence(b)
    step(fused=True)
    step(fused=False)
    if kv_dtype == "bf16":
        step(fused=True, group=True)
    ci0, _ = lay.cache_of(0)
    ci1, _ = lay.cache_of(1)
    assert [lay.seq_len(ci0, b) for b in range(B)] == [ora.seq_len(0, b) for b in range(B)]
    assert lay.device_lens(ci0)[1] == -1 and lay.device_lens(ci1)[3] == -1      # idle on the device too
    # a new request starts in slot 3 (a prompt of 90 tokens, fed in two chunks); slot 1 stays idle
    for chunk in ([0, 0, 0, 60], [0, 0, 0, 30]):
        T = sum(chunk)
        kv = {}
        for li in range(len(layers)):
            wr = lay.writer_of(li)
            seed[0] += 7
            if wr == li:
                kv[li] = (wl.randn(seed[0], (T, Hkv, d), tdt, DEV), wl.randn(seed[0] + 1, (T, Hkv, d), tdt, DEV))
            q = wl.randn(seed[0] + 2, (T, Hq, d), tdt, DEV)
            k, v = kv[wr]
            ring_reader = wr != li and layers[li][0] == 1 and layers[wr][0] == 1
            if ring_reader and kv_dtype == "bf16":
                out = lay.prefill_varlen(li, q, None, None, chunk)
            elif ring_reader and chunk[3] == 30:
                continue    # the scalar path has no staged copy for a ring reader past the first chunk
            else:
                out = lay.prefill_varlen(li, q, k, v, chunk)
            ref = ora.prefill_ragged(li, to_f64(q), to_f64(k) if wr == li else None, to_f64(v) if wr == li else None, chunk)
            assert_matches(out, ref, tol, "restart chunk %s layer %d" % (chunk, li))
    step(fused=True)
    step(fused=False)
    assert [lay.seq_len(ci0, b) for b in range(B)] == [ora.seq_len(0, b) for b in range(B)]
    assert lay.device_lens(ci0)[1] == -1 and lay.device_lens(ci0)[3] == ora.seq_len(0, 3)
    # everybody idle: the calls still run and write zeros
    for b in (0, 2, 3):
        lay.release_sequence(b); ora.release_sequence(b)
    step(fused=True)
    step(fused=False)
    assert lay.kv_bytes_live() == 0
    lay.close()
