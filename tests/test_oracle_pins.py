"""Pins for the CPU oracle: closed forms, invariants, a library special case, brute
force on tiny inputs, and planted mistakes that the pins must catch.

Passages (arXiv 2409.15012): Section 1 (causal attention over the cached context),
Section 3 "Sliding Window Attention Layers" (last s keys), Section 3 "KV cache reuse"
(a layer reads an earlier layer's cache), Section 3 last paragraph (GQA).
"""

import math

import numpy as np
import pytest
import torch

from oracle import mixattn_oracle as mo
from oracle.mixattn_oracle import FULL, SLIDING, LayerSpec, OracleStack

RNG = np.random.default_rng(20240915)


def _stack(layers, B=1, Hq=2, Hkv=2, d=8, **kw):
    return OracleStack([LayerSpec(*t) for t in layers], B, Hq, Hkv, d, **kw)


def _feed(st, layer, n, B, Hkv, d, rng):
    ks, vs = [], []
    for _ in range(n):
        k = rng.standard_normal((B, Hkv, d))
        v = rng.standard_normal((B, Hkv, d))
        st.append(layer, k, v)
        ks.append(k)
        vs.append(v)
    return np.stack(ks, 1), np.stack(vs, 1)  # [B, n, Hkv, d]


# ------------------------------------------------------------------ closed forms
def test_single_key_returns_its_value():
    st = _stack([(FULL, 0, 0)])
    k = RNG.standard_normal((1, 2, 8))
    v = RNG.standard_normal((1, 2, 8))
    st.append(0, k, v)
    out = st.decode(0, RNG.standard_normal((1, 2, 8)))
    np.testing.assert_allclose(out, v, rtol=0, atol=1e-15)


def test_constant_keys_give_mean_of_values_full_and_window():
    # equal keys => equal scores => uniform weights over the attended set
    B, H, d, n, W = 1, 2, 8, 23, 5
    st = _stack([(FULL, 0, 0), (SLIDING, W, 1)], B, H, H, d)
    kc = RNG.standard_normal((1, H, d))
    vs = []
    for _ in range(n):
        v = RNG.standard_normal((B, H, d))
        st.append(0, kc, v)
        st.append(1, kc, v)
        vs.append(v)
    V = np.stack(vs, 1)
    q = RNG.standard_normal((B, H, d))
    np.testing.assert_allclose(st.decode(0, q), V.mean(axis=1), atol=1e-13)
    np.testing.assert_allclose(st.decode(1, q), V[:, n - W:].mean(axis=1), atol=1e-13)


@pytest.mark.parametrize("W", [1, 2, 4, 7])
def test_window_is_exactly_W_keys_including_self(W):
    # constant keys, value at position p equals p  =>  output = mean(max(0,i-W+1) .. i),
    # a hand-countable number that moves if the window is W+1 keys or excludes the query's token.
    d = 4
    st = _stack([(SLIDING, W, 0)], 1, 1, 1, d)
    kc = np.ones((1, 1, d))
    for i in range(12):
        st.append(0, kc, np.full((1, 1, d), float(i)))
        out = st.decode(0, np.ones((1, 1, d)))
        lo = max(0, i - W + 1)
        expect = (lo + i) / 2.0
        np.testing.assert_allclose(out, expect, atol=1e-13)


def test_two_key_logistic_closed_form_pins_scale_and_sign():
    # two keys a*e0 and b*e0, query c*e0: weight of key 0 is sigmoid(scale*c*(a-b))
    d = 16
    a, b, c = 1.5, -0.25, 2.0
    st = _stack([(FULL, 0, 0)], 1, 1, 1, d)
    e0 = np.zeros((1, 1, d)); e0[..., 0] = 1.0
    v0 = RNG.standard_normal((1, 1, d)); v1 = RNG.standard_normal((1, 1, d))
    st.append(0, a * e0, v0)
    st.append(0, b * e0, v1)
    out = st.decode(0, c * e0)
    w0 = 1.0 / (1.0 + math.exp(-(c * (a - b)) / math.sqrt(d)))
    np.testing.assert_allclose(out, w0 * v0 + (1 - w0) * v1, atol=1e-14)
    # an explicit scale replaces 1/sqrt(d)
    st2 = _stack([(FULL, 0, 0)], 1, 1, 1, d, scale=0.7)
    st2.append(0, a * e0, v0); st2.append(0, b * e0, v1)
    w0 = 1.0 / (1.0 + math.exp(-0.7 * c * (a - b)))
    np.testing.assert_allclose(st2.decode(0, c * e0), w0 * v0 + (1 - w0) * v1, atol=1e-14)


def test_dominant_key_selects_its_value():
    d, n = 8, 9
    st = _stack([(FULL, 0, 0)], 1, 1, 1, d)
    K, V = _feed(st, 0, n, 1, 1, d, RNG)
    q = RNG.standard_normal((1, 1, d))
    big = 1e4 * q / np.linalg.norm(q)
    vb = RNG.standard_normal((1, 1, d))
    st.append(0, big, vb)
    K2, V2 = _feed(st, 0, 3, 1, 1, d, RNG)
    np.testing.assert_allclose(st.decode(0, q), vb, atol=1e-12)


# -------------------------------------------------------------------- invariants
def test_key_shift_invariance_and_linearity_in_values():
    B, H, d, n = 2, 2, 8, 17
    rng = np.random.default_rng(5)
    K = rng.standard_normal((B, n, H, d)); V = rng.standard_normal((B, n, H, d))
    V2 = rng.standard_normal((B, n, H, d))
    q = rng.standard_normal((B, H, d))
    delta = rng.standard_normal((1, 1, 1, d))

    def run(Kx, Vx):
        st = _stack([(FULL, 0, 0)], B, H, H, d)
        for p in range(n):
            st.append(0, Kx[:, p], Vx[:, p])
        return st.decode(0, q)

    base = run(K, V)
    np.testing.assert_allclose(run(K + delta, V), base, atol=1e-12)
    np.testing.assert_allclose(run(K, 2.0 * V - 3.0 * V2), 2.0 * base - 3.0 * run(K, V2), atol=1e-12)


def test_window_at_least_context_equals_full():
    B, H, d, n = 2, 2, 8, 19
    for W in (n, n + 1, 1000):
        rng = np.random.default_rng(6)
        st = _stack([(FULL, 0, 0), (SLIDING, W, 1)], B, H, H, d)
        for _ in range(n):
            k = rng.standard_normal((B, H, d)); v = rng.standard_normal((B, H, d))
            st.append(0, k, v); st.append(1, k, v)
        q = rng.standard_normal((B, H, d))
        np.testing.assert_array_equal(st.decode(0, q), st.decode(1, q))


def test_shared_cache_equals_duplicated_cache():
    B, Hq, Hkv, d, W = 2, 4, 2, 8, 6
    layers = [(FULL, 0, 0), (SLIDING, W, 1), (SLIDING, W, 1), (FULL, 0, 0)]
    sh = _stack(layers, B, Hq, Hkv, d)
    du = _stack(layers, B, Hq, Hkv, d, duplicate=True)
    rng = np.random.default_rng(7)
    S = 9
    kv = {w: (rng.standard_normal((B, S, Hkv, d)), rng.standard_normal((B, S, Hkv, d))) for w in (0, 1)}
    wr = {0: 0, 1: 1, 2: 1, 3: 0}
    for li in range(4):
        q = rng.standard_normal((B, S, Hq, d))
        k, v = kv[wr[li]]
        a = sh.prefill(li, q, k if sh.is_writer(li) else None, v if sh.is_writer(li) else None)
        b = du.prefill(li, q, k, v)
        np.testing.assert_array_equal(a, b)
    for step in range(11):
        new = {w: (rng.standard_normal((B, Hkv, d)), rng.standard_normal((B, Hkv, d))) for w in (0, 1)}
        for li in range(4):
            if sh.is_writer(li):
                sh.append(li, *new[wr[li]])
            du.append(li, *new[wr[li]])
            q = rng.standard_normal((B, Hq, d))
            np.testing.assert_array_equal(sh.decode(li, q), du.decode(li, q))
    with pytest.raises(ValueError):
        sh.append(2, *new[1])  # a reader appends nothing


def test_permuting_positions_inside_the_window_changes_nothing():
    # the softmax-weighted mean is a sum over the attended set: the order keys are visited in is irrelevant
    d, n, W = 8, 40, 16
    rng = np.random.default_rng(8)
    st = _stack([(SLIDING, W, 0)], 1, 1, 1, d)
    K, V = _feed(st, 0, n, 1, 1, d, rng)
    q = rng.standard_normal((1, 1, d))
    ref = st.decode(0, q)
    perm = rng.permutation(W)
    Kw = K[0, n - W:, 0][perm]; Vw = V[0, n - W:, 0][perm]
    np.testing.assert_allclose(mo.attend_row(q[0, 0], Kw, Vw, st.scale), ref[0, 0], atol=1e-14)
    # ring order: slot s holds position p = s mod W; reading slots 0..W-1 is one such permutation
    view = mo.ring_view(SLIDING, W, n)
    Kr = np.stack([K[0, p, 0] for p in view]); Vr = np.stack([V[0, p, 0] for p in view])
    np.testing.assert_allclose(mo.attend_row(q[0, 0], Kr, Vr, st.scale), ref[0, 0], atol=1e-14)


def test_gqa_equals_replicated_kv_heads():
    B, Hq, Hkv, d, n = 2, 8, 2, 8, 13
    G = Hq // Hkv
    rng = np.random.default_rng(9)
    a = _stack([(FULL, 0, 0)], B, Hq, Hkv, d)
    b = _stack([(FULL, 0, 0)], B, Hq, Hq, d)
    for _ in range(n):
        k = rng.standard_normal((B, Hkv, d)); v = rng.standard_normal((B, Hkv, d))
        a.append(0, k, v)
        b.append(0, np.repeat(k, G, axis=1), np.repeat(v, G, axis=1))
    q = rng.standard_normal((B, Hq, d))
    np.testing.assert_array_equal(a.decode(0, q), b.decode(0, q))


def test_prefill_row_equals_decode_after_that_many_appends():
    B, Hq, Hkv, d, S, W = 2, 4, 2, 8, 21, 5
    rng = np.random.default_rng(10)
    q = rng.standard_normal((B, S, Hq, d))
    k = rng.standard_normal((B, S, Hkv, d)); v = rng.standard_normal((B, S, Hkv, d))
    for layers in ([(FULL, 0, 0)], [(SLIDING, W, 0)]):
        pf = _stack(layers, B, Hq, Hkv, d).prefill(0, q, k, v)
        st = _stack(layers, B, Hq, Hkv, d)
        for i in range(S):
            st.append(0, k[:, i], v[:, i])
            np.testing.assert_array_equal(st.decode(0, q[:, i]), pf[:, i])


def test_ragged_batch_mates_are_independent():
    B, H, d = 3, 2, 8
    lens = [5, 1, 12]
    rng = np.random.default_rng(11)
    st = _stack([(SLIDING, 4, 0)], B, H, H, d)
    k = rng.standard_normal((sum(lens), H, d)); v = rng.standard_normal((sum(lens), H, d))
    st.load(0, k, v, lens)
    q = rng.standard_normal((B, H, d))
    out = st.decode(0, q)
    off = 0
    for b, n in enumerate(lens):
        solo = _stack([(SLIDING, 4, 0)], 1, H, H, d)
        solo.load(0, k[off:off + n], v[off:off + n], [n])
        np.testing.assert_array_equal(solo.decode(0, q[b:b + 1])[0], out[b])
        off += n


# ------------------------------------------------------- library special case
@pytest.mark.parametrize("kind,W", [(FULL, 0), (SLIDING, 7), (SLIDING, 1)])
def test_against_torch_cpu_fp64_sdpa_with_explicit_mask(kind, W):
    B, Hq, Hkv, d, S = 2, 4, 2, 16, 33
    G = Hq // Hkv
    rng = np.random.default_rng(12)
    q = rng.standard_normal((B, S, Hq, d)); k = rng.standard_normal((B, S, Hkv, d)); v = rng.standard_normal((B, S, Hkv, d))
    mine = _stack([(kind, W, 0)], B, Hq, Hkv, d).prefill(0, q, k, v)
    i = torch.arange(S)[:, None]; j = torch.arange(S)[None, :]
    mask = j <= i
    if kind == SLIDING:
        mask = mask & (j > i - W)
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    tk = torch.from_numpy(np.repeat(k, G, axis=2)).permute(0, 2, 1, 3)
    tv = torch.from_numpy(np.repeat(v, G, axis=2)).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(mine, ref, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------- brute force, tiny inputs
def test_brute_force_python_loops_tiny():
    B, Hq, Hkv, d, S, W = 1, 2, 1, 3, 7, 3
    rng = np.random.default_rng(13)
    q = rng.standard_normal((B, S, Hq, d)); k = rng.standard_normal((B, S, Hkv, d)); v = rng.standard_normal((B, S, Hkv, d))
    for kind in (FULL, SLIDING):
        mine = _stack([(kind, W, 0)], B, Hq, Hkv, d).prefill(0, q, k, v)
        for i in range(S):
            for jh in range(Hq):
                num = [0.0] * d; den = 0.0
                for p in range(S):
                    allowed = p <= i and (kind == FULL or i - p < W)
                    if not allowed:
                        continue
                    s = sum(q[0, i, jh, e] * k[0, p, jh // 2, e] for e in range(d)) / math.sqrt(d)
                    w = math.exp(s)
                    den += w
                    for e in range(d):
                        num[e] += w * v[0, p, jh // 2, e]
                for e in range(d):
                    assert abs(mine[0, i, jh, e] - num[e] / den) < 1e-12


# ------------------------------------------------------------- ring bookkeeping
def test_ring_slots_against_a_simulated_ring():
    for W in (1, 3, 8):
        ring = [None] * W
        for n in range(1, 30):
            p = n - 1
            assert mo.ring_slot(SLIDING, W, p) == p % W
            ring[p % W] = p
            view = mo.ring_view(SLIDING, W, n)
            assert view == [x for x in ring[:min(n, W)]]
            assert sorted(view) == list(range(max(0, n - W), n))
    assert mo.ring_view(FULL, 0, 5) == [0, 1, 2, 3, 4]
    assert mo.ring_slot(FULL, 0, 123456789012) == 123456789012


def test_cache_view_against_simulated_storage():
    """cache_view (what the GPU cache-content checks iterate over) against storage simulated token by token: a ring
    of W slots overwritten at p mod W, a list for a standard cache.  Covers a ring's writer and reader, a standard
    cache's writer and reader, and a sliding reader of a standard cache, which stores nothing of its own: its view
    is the writer's (every position, slot = position), however small its window."""
    W, B = 5, 2
    layers = [(FULL, 0, 0), (SLIDING, W, 1), (SLIDING, W, 1), (FULL, 0, 0), (SLIDING, 3, 0)]
    st = _stack(layers, B=B, Hq=2, Hkv=2, d=4)
    rng = np.random.default_rng(77)
    ring = [[None] * W for _ in range(B)]
    full = [[] for _ in range(B)]
    st.load(0, rng.standard_normal((2, 2, 4)), rng.standard_normal((2, 2, 4)), [2, 0])  # sequence 0 starts ahead
    st.load(1, rng.standard_normal((2, 2, 4)), rng.standard_normal((2, 2, 4)), [2, 0])
    for p in range(2):
        ring[0][p % W] = p
        full[0].append(p)
    for step in range(17):
        for li in (0, 1):
            st.append(li, rng.standard_normal((B, 2, 4)), rng.standard_normal((B, 2, 4)))
        for b in range(B):
            p = len(full[b])
            ring[b][p % W] = p
            full[b].append(p)
            want_ring = [(s, ring[b][s]) for s in range(W) if ring[b][s] is not None]
            want_full = list(enumerate(full[b]))
            assert st.cache_view(1, b) == want_ring and st.cache_view(2, b) == want_ring
            assert st.cache_view(0, b) == want_full and st.cache_view(3, b) == want_full
            assert st.cache_view(4, b) == want_full      # mixed-kind reader: the writer's storage
            # every listed position is where the slot arithmetic puts it, and its row is the history's row
            for li in range(len(layers)):
                wk = layers[st.writer[layers[li][2]]]
                for slot, pos in st.cache_view(li, b):
                    assert mo.ring_slot(wk[0], wk[1], pos) == slot
                assert len(st.cache_view(li, b)) == (min(st.seq_len(li, b), W) if wk[0] == SLIDING else st.seq_len(li, b))
    st.release_sequence(1)
    assert st.cache_view(1, 1) == [] and st.cache_view(4, 1) == []


def test_kv_accounting_matches_the_section3_ratios():
    # every l layers sharing one cache => 1/l of the caches; a sliding cache holds min(n, s) tokens
    n = 5000
    full = [LayerSpec(FULL, 0, i) for i in range(24)]
    shared4 = [LayerSpec(FULL, 0, i // 4) for i in range(24)]
    assert mo.resident_kv_tokens(shared4, [n]) * 4 == mo.resident_kv_tokens(full, [n])
    slid = [LayerSpec(SLIDING, 1024, i) for i in range(24)]
    assert mo.resident_kv_tokens(slid, [n]) == 24 * 1024
    assert mo.resident_kv_tokens(slid, [100]) == 24 * 100
    assert mo.step_read_tokens(shared4, [n]) == 24 * n
    assert mo.kv_bytes_per_token(8, 128, 2) == 4096


# ----------------------------------------------------------- planted mistakes
class _WindowPlusOne(OracleStack):
    def _attend(self, layer, b, q_row, j, i, K, V):
        sp = self.layers[layer]
        h = j // self.G
        lo = max(0, i - sp.window) if sp.kind == SLIDING else 0  # W+1 keys: wrong
        return mo.attend_row(q_row, K[lo:i + 1, h, :], V[lo:i + 1, h, :], self.scale)


class _WrongHeadMap(OracleStack):
    def _attend(self, layer, b, q_row, j, i, K, V):
        h = j % self.Hkv  # interleaved instead of grouped: wrong
        return mo.attend_row(q_row, K[:i + 1, h, :], V[:i + 1, h, :], self.scale)


def test_pins_catch_planted_mistakes():
    d = 4
    st = _WindowPlusOne([LayerSpec(SLIDING, 3, 0)], 1, 1, 1, d)
    for i in range(6):
        st.append(0, np.ones((1, 1, d)), np.full((1, 1, d), float(i)))
    assert abs(st.decode(0, np.ones((1, 1, d)))[0, 0, 0] - 4.0) > 0.4  # right answer is mean(3,4,5) = 4

    rng = np.random.default_rng(14)
    B, Hq, Hkv, n = 1, 4, 2, 6
    good = OracleStack([LayerSpec(FULL, 0, 0)], B, Hq, Hkv, d)
    bad = _WrongHeadMap([LayerSpec(FULL, 0, 0)], B, Hq, Hkv, d)
    for _ in range(n):
        k = rng.standard_normal((B, Hkv, d)); v = rng.standard_normal((B, Hkv, d))
        good.append(0, k, v); bad.append(0, k, v)
    q = rng.standard_normal((B, Hq, d))
    assert np.abs(good.decode(0, q) - bad.decode(0, q)).max() > 1e-3


def test_sliding_reader_of_a_full_cache_sees_the_last_window_positions():
    # extension of the sharing rule: same history, the reader's own mask
    B, H, d, n, W = 1, 2, 8, 30, 7
    rng = np.random.default_rng(15)
    mixed = _stack([(FULL, 0, 0), (SLIDING, W, 0)], B, H, H, d)
    own = _stack([(SLIDING, W, 0)], B, H, H, d)
    for _ in range(n):
        k = rng.standard_normal((B, H, d)); v = rng.standard_normal((B, H, d))
        mixed.append(0, k, v); own.append(0, k, v)
        q = rng.standard_normal((B, H, d))
        np.testing.assert_array_equal(mixed.decode(1, q), own.decode(0, q))
    with pytest.raises(ValueError):
        _stack([(SLIDING, W, 0), (FULL, 0, 0)])  # a full layer cannot read a ring


def test_chunked_prefill_equals_one_shot_and_equals_appends():
    # Section 1: earlier tokens are unaffected by later ones, so feeding a prompt in chunks changes nothing
    B, Hq, Hkv, d, S, W = 2, 4, 2, 8, 23, 6
    rng = np.random.default_rng(16)
    q = rng.standard_normal((B, S, Hq, d))
    k = rng.standard_normal((B, S, Hkv, d)); v = rng.standard_normal((B, S, Hkv, d))
    layers = [(FULL, 0, 0), (SLIDING, W, 1), (SLIDING, W, 1)]
    whole = _stack(layers, B, Hq, Hkv, d)
    ref = [whole.prefill(0, q, k, v), whole.prefill(1, q, k, v), whole.prefill(2, q, None, None)]
    parts = _stack(layers, B, Hq, Hkv, d)
    got = [[], [], []]
    for (a, b) in ((0, 5), (5, 6), (6, 17), (17, 23)):
        got[0].append(parts.prefill(0, q[:, a:b], k[:, a:b], v[:, a:b]))
        got[1].append(parts.prefill(1, q[:, a:b], k[:, a:b], v[:, a:b]))
        got[2].append(parts.prefill(2, q[:, a:b], None, None))
    for li in range(3):
        np.testing.assert_array_equal(np.concatenate(got[li], axis=1), ref[li])
    # and a decode step after the chunks sees the same history
    qd = rng.standard_normal((B, Hq, d))
    for li in range(3):
        np.testing.assert_array_equal(parts.decode(li, qd), whole.decode(li, qd))


def test_ragged_prefill_equals_token_by_token_decode_and_brute_force():
    # chunks of different lengths per sequence: every row must equal the decode step after that many appends on a
    # batch-of-one stack (decode is pinned by the closed forms above), and a sliding row must equal the plain
    # definition written out over the last W positions
    Hq, Hkv, d, W = 4, 2, 8, 5
    layers = [(FULL, 0, 0), (SLIDING, W, 1), (SLIDING, W, 1)]
    rng = np.random.default_rng(21)
    first_lens, second_lens = [7, 0, 3], [2, 9, 0]
    B = len(first_lens)
    ragged = _stack(layers, B, Hq, Hkv, d)
    singles = [_stack(layers, 1, Hq, Hkv, d) for _ in range(B)]
    hist = [[np.zeros((0, Hkv, d)), np.zeros((0, Hkv, d))] for _ in range(B)]  # K, V of the sliding cache
    for lens in (first_lens, second_lens):
        T = sum(lens)
        q = rng.standard_normal((T, Hq, d))
        kv = {li: (rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d))) for li in (0, 1)}
        out = {0: ragged.prefill_ragged(0, q, kv[0][0], kv[0][1], lens),
               1: ragged.prefill_ragged(1, q, kv[1][0], kv[1][1], lens),
               2: ragged.prefill_ragged(2, q, None, None, lens)}
        row = 0
        for b in range(B):
            for i in range(lens[b]):
                for li in (0, 1):
                    singles[b].append(li, kv[li][0][row][None], kv[li][1][row][None])
                for li in (0, 1, 2):
                    np.testing.assert_allclose(out[li][row], singles[b].decode(li, q[row][None])[0], rtol=0, atol=1e-12)
                hist[b][0] = np.concatenate([hist[b][0], kv[1][0][row][None]])
                hist[b][1] = np.concatenate([hist[b][1], kv[1][1][row][None]])
                K, V = hist[b][0][-W:], hist[b][1][-W:]
                for j in range(Hq):
                    s = K[:, j // (Hq // Hkv)] @ q[row, j] / math.sqrt(d)
                    w = np.exp(s - s.max())
                    np.testing.assert_allclose(out[2][row, j], (w[:, None] * V[:, j // (Hq // Hkv)]).sum(0) / w.sum(),
                                               rtol=0, atol=1e-12)
                row += 1
    assert [ragged.seq_len(0, b) for b in range(B)] == [9, 9, 3]
    with pytest.raises(ValueError):
        ragged.prefill_ragged(0, np.zeros((3, Hq, d)), np.zeros((3, Hkv, d)), np.zeros((3, Hkv, d)), [1, 1])


def test_released_sequence_behaves_like_a_fresh_one():
    Hq, Hkv, d, W = 4, 2, 8, 3
    layers = [(FULL, 0, 0), (SLIDING, W, 1)]
    rng = np.random.default_rng(31)
    a = _stack(layers, 2, Hq, Hkv, d)
    k = rng.standard_normal((9, Hkv, d)); v = rng.standard_normal((9, Hkv, d))
    for li in (0, 1):
        a.load(li, k, v, [5, 4])
    a.release_sequence(0)
    assert [a.seq_len(li, 0) for li in (0, 1)] == [0, 0] and [a.seq_len(li, 1) for li in (0, 1)] == [4, 4]
    # sequence 0 takes a new request of 2 tokens; sequence 1 sits the call out
    k2 = rng.standard_normal((2, Hkv, d)); v2 = rng.standard_normal((2, Hkv, d))
    q2 = rng.standard_normal((2, Hq, d))
    fresh = _stack(layers, 1, Hq, Hkv, d)
    for li in (0, 1):
        got = a.prefill_ragged(li, q2, k2, v2, [2, 0])
        ref = fresh.prefill_ragged(li, q2, k2, v2, [2])
        np.testing.assert_array_equal(got, ref)
    # sequence 1 kept its history
    q = rng.standard_normal((2, Hq, d))
    solo = _stack(layers, 1, Hq, Hkv, d)
    for li in (0, 1):
        solo.load(li, k[5:], v[5:], [4])
        np.testing.assert_array_equal(a.decode(li, q, rows=[(1, j) for j in range(Hq)])[1], solo.decode(li, q[1:2])[0])


def test_idle_sequences_are_passed_over():
    """A released sequence is idle: decode-step tokens pass over it, its decode rows are zero, its batch mates see
    nothing of it, and a new prompt in its slot gives exactly what a fresh stack gives."""
    Hq, Hkv, d, W = 4, 2, 8, 3
    layers = [(FULL, 0, 0), (SLIDING, W, 1), (SLIDING, W, 1)]
    rng = np.random.default_rng(77)
    a = _stack(layers, 3, Hq, Hkv, d)
    solo = _stack(layers, 1, Hq, Hkv, d)     # sequence 2 alone
    k = rng.standard_normal((12, Hkv, d)); v = rng.standard_normal((12, Hkv, d))
    for li in (0, 1):
        a.load(li, k, v, [5, 4, 3])
        solo.load(li, k[9:], v[9:], [3])
    a.release_sequence(1)
    assert all(a.is_idle(li, 1) for li in range(3)) and not a.is_idle(0, 0)
    for step in range(4):
        k1 = rng.standard_normal((3, Hkv, d)); v1 = rng.standard_normal((3, Hkv, d))
        q1 = rng.standard_normal((3, Hq, d))
        for li in (0, 1):
            a.append(li, k1, v1)
            solo.append(li, k1[2:], v1[2:])
        for li in range(3):
            out = a.decode(li, q1)
            assert np.all(out[1] == 0.0)
            np.testing.assert_array_equal(out[2], solo.decode(li, q1[2:])[0])
        assert [a.seq_len(li, 1) for li in (0, 1)] == [0, 0]
        assert a.seq_len(0, 0) == 5 + step + 1
    # a new request in the idle slot: two prompt tokens, the others sit the call out
    k2 = rng.standard_normal((2, Hkv, d)); v2 = rng.standard_normal((2, Hkv, d)); q2 = rng.standard_normal((2, Hq, d))
    fresh = _stack(layers, 1, Hq, Hkv, d)
    for li in range(3):
        wr = li != 2
        got = a.prefill_ragged(li, q2, k2 if wr else None, v2 if wr else None, [0, 2, 0])
        ref = fresh.prefill_ragged(li, q2, k2 if wr else None, v2 if wr else None, [2])
        np.testing.assert_array_equal(got, ref)
        assert not a.is_idle(li, 1)
    k1 = rng.standard_normal((3, Hkv, d)); v1 = rng.standard_normal((3, Hkv, d)); q1 = rng.standard_normal((3, Hq, d))
    for li in (0, 1):
        a.append(li, k1, v1)
        fresh.append(li, k1[1:2], v1[1:2])
    for li in range(3):
        np.testing.assert_array_equal(a.decode(li, q1)[1], fresh.decode(li, q1[1:2])[0])


# ----------------------------------------------------- random request traffic against a list-of-tokens model
def _sdpa_row(q_row, K, V, scale):
    """One output row through torch's fp64 CPU scaled_dot_product_attention (a library routine, not the oracle's sum)."""
    qt = torch.from_numpy(np.ascontiguousarray(q_row)).reshape(1, 1, 1, -1)
    kt = torch.from_numpy(np.ascontiguousarray(K)).reshape(1, 1, K.shape[0], -1)
    vt = torch.from_numpy(np.ascontiguousarray(V)).reshape(1, 1, V.shape[0], -1)
    return torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=scale).reshape(-1).numpy()


@pytest.mark.parametrize("seed", range(12))
def test_random_request_traffic_matches_a_list_of_tokens_model(seed):
    """Random stacks and random sequences of calls (appends, ragged prompt chunks, releases, decodes): every output
    row equals library attention over the tokens a plain per-(cache, sequence) list says the row can see."""
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.integers(1, 3)); G = int(rng.integers(1, 4)); Hq = Hkv * G; d = 4; B = int(rng.integers(1, 4))
    n_caches = int(rng.integers(1, 4))
    kinds = [(int(rng.integers(0, 2)), int(rng.integers(1, 6))) for _ in range(n_caches)]   # per cache: kind, window
    layers, seen = [], set()
    for _ in range(int(rng.integers(n_caches, n_caches + 4))):
        c = int(rng.integers(0, n_caches)) if len(seen) == n_caches else len(seen)
        kind, W = kinds[c]
        if c in seen and kind == FULL and rng.random() < 0.3:
            layers.append((SLIDING, int(rng.integers(1, 6)), c))       # sliding reader of a full cache
        else:
            layers.append((kind, W if kind == SLIDING else 0, c))
        seen.add(c)
    st = _stack(layers, B, Hq, Hkv, d)
    writer = {}
    for li, (_, _, c) in enumerate(layers):
        writer.setdefault(c, li)
    toks = {c: [[] for _ in range(B)] for c in range(n_caches)}       # the model: (k, v) rows per cache and sequence
    idle = {c: [False] * B for c in range(n_caches)}

    def expect(li, b, j, q_row, pos):
        kind, W, c = layers[li]
        lo = max(0, pos - W + 1) if kind == SLIDING else 0
        rows = toks[c][b][lo:pos + 1]
        K = np.stack([r[0][j // G] for r in rows]); V = np.stack([r[1][j // G] for r in rows])
        return _sdpa_row(q_row, K, V, 1.0 / math.sqrt(d))

    for _ in range(25):
        op = rng.choice(["append", "chunk", "release", "decode"], p=[0.35, 0.3, 0.1, 0.25])
        if op == "append":
            for c, li in writer.items():
                k = rng.standard_normal((B, Hkv, d)); v = rng.standard_normal((B, Hkv, d))
                st.append(li, k, v)
                for b in range(B):
                    if not idle[c][b]:
                        toks[c][b].append((k[b], v[b]))
        elif op == "chunk":
            lens = [int(x) for x in rng.integers(0, 4, size=B)]
            if sum(lens) == 0:
                continue
            T = sum(lens); first = np.concatenate([[0], np.cumsum(lens)])
            kv = {c: (rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d))) for c in writer}
            for li, (_, _, c) in enumerate(layers):
                q = rng.standard_normal((T, Hq, d))
                is_w = writer[c] == li
                if is_w:
                    for b in range(B):
                        if lens[b]:
                            idle[c][b] = False
                        toks[c][b].extend((kv[c][0][t], kv[c][1][t]) for t in range(first[b], first[b + 1]))
                out = st.prefill_ragged(li, q, kv[c][0] if is_w else None, kv[c][1] if is_w else None, lens)
                for b in range(B):
                    n = len(toks[c][b])
                    for i in range(lens[b]):
                        j = int(rng.integers(0, Hq))
                        np.testing.assert_allclose(out[first[b] + i, j], expect(li, b, j, q[first[b] + i, j], n - lens[b] + i),
                                                   atol=1e-12)
        elif op == "release":
            b = int(rng.integers(0, B))
            st.release_sequence(b)
            for c in toks:
                toks[c][b] = []
                idle[c][b] = True
        else:
            for li, (_, _, c) in enumerate(layers):
                if any(len(toks[c][b]) == 0 and not idle[c][b] for b in range(B)):
                    continue   # an empty (not idle) sequence: decode is an error there
                q = rng.standard_normal((B, Hq, d))
                out = st.decode(li, q)
                for b in range(B):
                    for j in range(Hq):
                        if idle[c][b]:
                            assert np.all(out[b, j] == 0.0)
                        else:
                            np.testing.assert_allclose(out[b, j], expect(li, b, j, q[b, j], len(toks[c][b]) - 1), atol=1e-12)
    for c, li in writer.items():
        assert [st.seq_len(li, b) for b in range(B)] == [len(toks[c][b]) for b in range(B)]
