"""GPU parity at the full benchmark sizes, on sampled outputs the oracle can compute one by one.

The library runs the whole workload through the calls bench.py times: same layout, batch and context, the automatic
split-K plan, writer layers through mixattn_append_decode (one fused launch) and bf16 output; an fp32-output pass
of the same sequence keeps the strict bound, and one pass uses the two-call form (append_kv, then decode).  The
oracle recomputes a sample of (sequence, kv head) pairs / query rows from the same bytes (copied back from the
device)."""

import numpy as np
import pytest
import torch

from helpers import assert_matches, to_f64
from oracle.mixattn_oracle import LayerSpec, OracleStack
from paper_2409_15012_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def mx():
    from paper_2409_15012_amd import binding
    binding.load()
    return binding


def _decode_sampled(mx, w, sample, steps=2, seed_shift=0, out_dtype="bf16", fused=True, layers=None):
    """Loads w.seq_lens[b] - steps tokens, runs `steps` decode steps of the whole stack, checks sampled (b, kv head).
    fused: writer layers append and decode in one call (what the benchmark times); otherwise append_kv + decode."""
    B, Hq, Hkv, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    G = Hq // Hkv
    layers = layers or w.layers
    lens = [n - steps for n in w.seq_lens]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    lay = mx.Layout(layers, B, Hq, Hkv, d, capacity=list(w.seq_lens), kv_dtype="bf16", out_dtype=out_dtype)
    # one oracle per sampled (b, h): batch 1, one KV head, its G query heads
    oras = {s: OracleStack([LayerSpec(*t) for t in layers], 1, G, 1, d) for s in sample}
    seed = w.seed + seed_shift
    writers = [li for li in range(len(layers)) if lay.cache_of(li)[1]]
    for li in writers:
        k = wl.randn(wl.layer_seed(seed, li, "k", 1), (int(offs[-1]), Hkv, d), torch.bfloat16, DEV)
        v = wl.randn(wl.layer_seed(seed, li, "v", 1), (int(offs[-1]), Hkv, d), torch.bfloat16, DEV)
        lay.load_kv(li, k, v, lens)
        for (b, h), ora in oras.items():
            sl = slice(int(offs[b]), int(offs[b + 1]))
            ora.load(li, to_f64(k[sl, h:h + 1]), to_f64(v[sl, h:h + 1]), [lens[b]])
        del k, v
        torch.cuda.empty_cache()
    worst = [0.0, 0.0]
    for t in range(steps):
        for li in range(len(layers)):
            ci, is_writer = lay.cache_of(li)
            q = wl.randn(wl.layer_seed(seed, li, "q", 10 + t), (B, Hq, d), torch.bfloat16, DEV)
            if is_writer:
                k = wl.randn(wl.layer_seed(seed, li, "k", 10 + t), (B, Hkv, d), torch.bfloat16, DEV)
                v = wl.randn(wl.layer_seed(seed, li, "v", 10 + t), (B, Hkv, d), torch.bfloat16, DEV)
                for (b, h), ora in oras.items():
                    ora.append(li, to_f64(k[b:b + 1, h:h + 1]), to_f64(v[b:b + 1, h:h + 1]))
                if fused:
                    out = lay.append_decode(li, k, v, q)
                else:
                    lay.append_kv(li, k, v)
                    out = lay.decode(li, q)
            else:
                out = lay.decode(li, q)
            assert out.dtype == lay.out_torch and not torch.isnan(out).any()
            got = torch.stack([out[b, h * G:(h + 1) * G] for (b, h) in oras])
            ref = np.stack([ora.decode(li, to_f64(q[b:b + 1, h * G:(h + 1) * G]))[0] for (b, h), ora in oras.items()])
            e = assert_matches(got, ref, "bf16", "step %d layer %d" % (t, li))
            worst = [max(worst[0], e[0]), max(worst[1], e[1])]
    # bit-exact cache rows at a few slots of the sampled pairs (first, middle, and the slots the appended tokens went
    # to), host and device lengths
    for li in sorted({writers[0], writers[1 % len(writers)], writers[-1]}):
        ci, _ = lay.cache_of(li)
        dev_lens = lay.device_lens(ci)
        for (b, h), ora in oras.items():
            view = dict(ora.cache_view(li, 0))
            pos_of_slot = sorted(view.items(), key=lambda sp: sp[1])   # by position
            K, V = ora.history(li, 0)
            for slot, pos in [pos_of_slot[0], pos_of_slot[len(pos_of_slot) // 2]] + pos_of_slot[-steps:]:
                k_row, v_row = lay.read_cache(ci, b, h, slot)
                assert np.array_equal(k_row.double().numpy(), K[pos, 0]) and np.array_equal(v_row.double().numpy(), V[pos, 0])
            assert lay.seq_len(ci, b) == ora.seq_len(li, 0) == dev_lens[b]
    print("worst max_abs %.3g rel_l2 %.3g" % tuple(worst))
    lay.close()
    torch.cuda.empty_cache()


# (output dtype, fused append): the benchmark's form first; fp32 output for the strict bound; the two-call form
FORMS = [("bf16", True), ("f32", True), ("f32", False)]


@pytest.mark.parametrize("out_dtype,fused", FORMS)
def test_config1_decode_b8_ctx4096(mx, out_dtype, fused):
    _decode_sampled(mx, wl.config(1), [(0, 0), (3, 5), (7, 7)], out_dtype=out_dtype, fused=fused)


@pytest.mark.parametrize("out_dtype,fused", FORMS)
def test_config2_decode_b32_ctx32768(mx, out_dtype, fused):
    _decode_sampled(mx, wl.config(2), [(0, 0), (17, 3), (31, 7)], out_dtype=out_dtype, fused=fused)


@pytest.mark.parametrize("out_dtype,fused", FORMS)
def test_config4_ragged_b64(mx, out_dtype, fused):
    """The ragged batch takes the balanced launch (equal runs of blocks per workgroup), with the append fused in."""
    w = wl.config(4)
    order = np.argsort(w.seq_lens)
    sample = [(int(order[0]), 1), (int(order[len(order) // 2]), 4), (int(order[-1]), 7)]  # shortest, median, longest
    _decode_sampled(mx, w, sample, steps=2, out_dtype=out_dtype, fused=fused)


def test_config4_standard_stack_layers_ragged_b64(mx):
    """The all-full comparison stack of the ragged configuration (three of its 24 identical layers are enough to
    cover its launch; every layer has a private cache)."""
    w = wl.config(4)
    order = np.argsort(w.seq_lens)
    sample = [(int(order[1]), 0), (int(order[-2]), 5)]
    _decode_sampled(mx, w, sample, steps=1, layers=wl.layout_full24()[:3])


@pytest.mark.parametrize("out_dtype", ["bf16", "f32"])
def test_config3_prefill_s32768_sampled_rows(mx, out_dtype):
    w = wl.config(3)
    B, S, Hq, Hkv, d, W = 1, w.prefill_len, w.n_q_heads, w.n_kv_heads, w.head_dim, 1024
    G = Hq // Hkv
    # one full layer (cache 0) and one sliding group (writer 1, reader 2) are enough to cover both kernels paths
    layers = [(0, 0, 0), (1, W, 1), (1, W, 1)]
    lay = mx.Layout(layers, B, Hq, Hkv, d, capacity=[S + 1], kv_dtype="bf16", out_dtype=out_dtype)
    rows = sorted(set([0, 1, 31, 32, 63, 64, 127, 128, W - 1, W, W + 1, W + 63, W + 64, 4095, 4096, 16383, 20000,
                       S - 129, S - 128, S - 1]))
    heads = [0, 13, 31]
    kv = {}
    for li in range(3):
        wr = lay.writer_of(li)
        if wr == li:
            kv[li] = (wl.randn(wl.layer_seed(w.seed, li, "k"), (B, S, Hkv, d), torch.bfloat16, DEV),
                      wl.randn(wl.layer_seed(w.seed, li, "v"), (B, S, Hkv, d), torch.bfloat16, DEV))
        k, v = kv[wr]
        q = wl.randn(wl.layer_seed(w.seed, li, "q"), (B, S, Hq, d), torch.bfloat16, DEV)
        # readers reuse the prompt copy their writer staged, as the benchmark's layer loop does
        out = lay.prefill(li, q, k, v) if wr == li else lay.prefill(li, q, None, None)
        assert out.dtype == lay.out_torch and not torch.isnan(out).any()
        got, ref = [], []
        for j in heads:
            h = j // G
            ora = OracleStack([LayerSpec(*layers[li])], 1, 1, 1, d)
            res = ora.prefill(0, to_f64(q[:, :, j:j + 1]), to_f64(k[:, :, h:h + 1]), to_f64(v[:, :, h:h + 1]),
                              rows=[(0, i, 0) for i in rows])
            ref.append(res[0, rows, 0])
            got.append(out[0, rows, j])
        assert_matches(torch.stack(got), np.stack(ref), "bf16", "prefill layer %d" % li)
    # caches: full holds every position, ring the last W at p mod W
    for (ci, li) in ((0, 0), (1, 1)):
        k, v = kv[li]
        for pos in (0, 1000, S - W, S - 1):
            if ci == 1 and pos < S - W:
                continue
            slot = lay.slot_of(ci, pos)
            assert slot == (pos if ci == 0 else pos % W)
            k_row, v_row = lay.read_cache(ci, 0, 5, slot)
            assert torch.equal(k_row, k[0, pos, 5].cpu()) and torch.equal(v_row, v[0, pos, 5].cpu())
    # one decode step on top of the prefilled caches
    for li in range(3):
        wr = lay.writer_of(li)
        if wr == li:
            kn = wl.randn(77 + li, (B, Hkv, d), torch.bfloat16, DEV)
            vn = wl.randn(87 + li, (B, Hkv, d), torch.bfloat16, DEV)
            qn = wl.randn(97 + li, (B, Hq, d), torch.bfloat16, DEV)
            out = lay.append_decode(li, kn, vn, qn)
            kv[li] = (torch.cat([kv[li][0], kn.view(B, 1, Hkv, d)], 1), torch.cat([kv[li][1], vn.view(B, 1, Hkv, d)], 1))
        k, v = kv[wr]
        q = wl.randn(97 + li, (B, Hq, d), torch.bfloat16, DEV)
        if wr != li:
            out = lay.decode(li, q)
        got, ref = [], []
        for j in heads:
            h = j // G
            ora = OracleStack([LayerSpec(*layers[li])], 1, 1, 1, d)
            ora.load(0, to_f64(k[0, :, h:h + 1]), to_f64(v[0, :, h:h + 1]), [S + 1])
            ref.append(ora.decode(0, to_f64(q[:, j:j + 1]))[0, 0])
            got.append(out[0, j])
        assert_matches(torch.stack(got), np.stack(ref), "bf16", "decode after prefill layer %d" % li)
    lay.close()
