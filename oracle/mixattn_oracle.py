"""CPU fp64 oracle for MixAttention attention over KV caches.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the GPU
library is checked against.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does, and this module
imports nothing from the product package.

What it follows (arXiv 2409.15012):

* Section 1: a causal layer attends to every token in its context; the keys and
  values of earlier tokens are cached ("standard" / full attention).
* Section 3, "Sliding Window Attention Layers": with window size s the query
  attends to the last s keys only, so a cache of the past s tokens suffices.
  Reading taken here: the window is exactly W keys *including* the query's own
  token, i.e. positions max(0, i-W+1) .. i.
* Section 3, "KV cache reuse": a layer may read the cache computed by an
  earlier layer; the first (lowest-index) layer of a sharing group writes it.
  Readers have their writer's kind and window; as an extension a sliding layer
  may read a standard layer's cache and then sees its last `window` positions.
* Section 3, last paragraph: grouped-query attention, query head j reads KV
  head j // (Hq // Hkv).

The method is exact softmax attention under a mask, so the oracle is that
definition written out: every cache is an unbounded, position-indexed history
(no ring buffer, no chunks, no tiling) and each output row is computed on its
own from scores -> max -> exp -> weighted mean.  `numpy.dot` is the only
library primitive used as a step.

Ring-slot bookkeeping (`ring_slot`, `ring_view`) is the integer side: position p
of a sliding cache lives in slot p mod W, a full cache keeps position p in
slot p.

Nothing in this file is "parity unpinned": see tests/test_oracle_pins.py.
"""

from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

FULL = 0
SLIDING = 1


@dataclass(frozen=True)
class LayerSpec:
    """One layer of the stack: kind, window (ignored for FULL) and cache id."""

    kind: int
    window: int
    cache_id: int


def ring_slot(kind: int, window: int, pos: int) -> int:
    """Slot that holds absolute position `pos` (Section 3: keep the past s tokens)."""
    if pos < 0:
        raise ValueError("negative position")
    if kind == FULL:
        return pos
    if window < 1:
        raise ValueError("window must be >= 1")
    return pos % window


def ring_view(kind: int, window: int, n: int) -> List[int]:
    """For a cache holding n tokens: list over valid slots of the position stored there.

    A full cache has n valid slots with slot s <- position s.  A ring of W slots has
    min(n, W) valid slots; slot s holds the largest position p < n with p = s (mod W).
    """
    if kind == FULL:
        return list(range(n))
    out = []
    for s in range(min(n, window)):
        p = s + ((n - 1 - s) // window) * window
        out.append(p)
    return out


def attend_row(q_row: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """softmax(scale * K q) weighted mean of V for ONE query row.

    q_row [d], K [m, d], V [m, d] in fp64, m >= 1.  Steps, in order: scores,
    their maximum, exponentials of the differences, normalised weighted sum.
    """
    if K.shape[0] < 1:
        raise ValueError("a query must attend to at least one key")
    s = scale * np.dot(K, q_row)
    m = np.max(s)
    w = np.exp(s - m)
    return np.dot(w, V) / np.sum(w)


class OracleStack:
    """Position-indexed fp64 reference for a MixAttention layer stack.

    layers      per-layer LayerSpec
    batch       number of sequences (each keeps its own length)
    duplicate   if True every layer keeps a private copy of the history it reads
                (the "no sharing" arrangement used to check that sharing changes
                nothing); reader layers are then fed through `append`/`prefill`
                with the writer's k, v by the caller.
    """

    def __init__(
        self,
        layers: Sequence[LayerSpec],
        batch: int,
        n_q_heads: int,
        n_kv_heads: int,
        head_dim: int,
        scale: Optional[float] = None,
        duplicate: bool = False,
    ):
        if n_q_heads % n_kv_heads != 0:
            raise ValueError("query heads must be a multiple of KV heads")
        self.layers = list(layers)
        self.B = batch
        self.Hq = n_q_heads
        self.Hkv = n_kv_heads
        self.G = n_q_heads // n_kv_heads
        self.d = head_dim
        self.scale = (1.0 / math.sqrt(head_dim)) if not scale else float(scale)
        self.duplicate = duplicate
        # writer(c) = lowest layer index using cache c
        self.writer = {}
        for li, sp in enumerate(self.layers):
            if sp.kind not in (FULL, SLIDING):
                raise ValueError("bad kind")
            if sp.kind == SLIDING and sp.window < 1:
                raise ValueError("window must be >= 1")
            if sp.cache_id not in self.writer:
                self.writer[sp.cache_id] = li
            else:
                w = self.layers[self.writer[sp.cache_id]]
                same = (w.kind, w.window if w.kind == SLIDING else 0) == (
                    sp.kind, sp.window if sp.kind == SLIDING else 0)
                windowed_reader = w.kind == FULL and sp.kind == SLIDING  # last `window` positions of a full cache
                if not (same or windowed_reader):
                    raise ValueError("sharers of a cache need the writer's kind and window "
                                     "(or be sliding readers of a full cache)")
        # history store key: cache id (shared) or layer index (duplicate mode)
        self._K = {}
        self._V = {}
        keys = range(len(self.layers)) if duplicate else self.writer.keys()
        for key in keys:
            self._K[key] = [np.zeros((0, self.Hkv, self.d)) for _ in range(batch)]
            self._V[key] = [np.zeros((0, self.Hkv, self.d)) for _ in range(batch)]
        # (store key, b) pairs of released sequences: idle until a prompt chunk or a bulk load gives them tokens
        self._idle = set()

    # ---------------------------------------------------------------- helpers
    def _store_key(self, layer: int):
        return layer if self.duplicate else self.layers[layer].cache_id

    def is_writer(self, layer: int) -> bool:
        return self.writer[self.layers[layer].cache_id] == layer

    def seq_len(self, layer: int, b: int) -> int:
        return self._K[self._store_key(layer)][b].shape[0]

    def is_idle(self, layer: int, b: int) -> bool:
        """Released and not yet given a new prompt, in the cache `layer` reads."""
        return (self._store_key(layer), b) in self._idle

    def history(self, layer: int, b: int) -> Tuple[np.ndarray, np.ndarray]:
        """(K, V) [n_b, Hkv, d] in absolute-position order for the cache `layer` reads."""
        key = self._store_key(layer)
        return self._K[key][b], self._V[key][b]

    def _check_may_write(self, layer: int):
        if not self.duplicate and not self.is_writer(layer):
            raise ValueError("layer %d reads a shared cache and appends nothing" % layer)

    def _attend(self, layer: int, b: int, q_row: np.ndarray, j: int, i: int,
                K: np.ndarray, V: np.ndarray) -> np.ndarray:
        """Output for query head j of sequence b sitting at absolute position i."""
        sp = self.layers[layer]
        h = j // self.G
        lo = max(0, i - sp.window + 1) if sp.kind == SLIDING else 0
        return attend_row(q_row, K[lo:i + 1, h, :], V[lo:i + 1, h, :], self.scale)

    # -------------------------------------------------------------------- API
    def append(self, layer: int, k: np.ndarray, v: np.ndarray):
        """One new token per sequence: k, v [B, Hkv, d]."""
        self._check_may_write(layer)
        k = np.asarray(k, dtype=np.float64).reshape(self.B, 1, self.Hkv, self.d)
        v = np.asarray(v, dtype=np.float64).reshape(self.B, 1, self.Hkv, self.d)
        key = self._store_key(layer)
        for b in range(self.B):
            if (key, b) in self._idle:
                continue  # an idle slot of the batch takes no decode-step token: its row of k, v is ignored
            self._K[key][b] = np.concatenate([self._K[key][b], k[b]], axis=0)
            self._V[key][b] = np.concatenate([self._V[key][b], v[b]], axis=0)

    def load(self, layer: int, k_packed: np.ndarray, v_packed: np.ndarray, seq_lens: Sequence[int]):
        """Bulk append without attention: packed [sum(seq_lens), Hkv, d], sequence after sequence."""
        self._check_may_write(layer)
        k_packed = np.asarray(k_packed, dtype=np.float64)
        v_packed = np.asarray(v_packed, dtype=np.float64)
        if len(seq_lens) != self.B or k_packed.shape[0] != int(sum(seq_lens)):
            raise ValueError("seq_lens does not match the packed tensor")
        key = self._store_key(layer)
        off = 0
        for b in range(self.B):
            n = int(seq_lens[b])
            if n > 0:
                self._idle.discard((key, b))
            self._K[key][b] = np.concatenate([self._K[key][b], k_packed[off:off + n]], axis=0)
            self._V[key][b] = np.concatenate([self._V[key][b], v_packed[off:off + n]], axis=0)
            off += n

    def release_sequence(self, b: int):
        """Sequence b gives up its slot of the batch: every cache forgets it and it is idle (appends pass over it,
        decode returns zeros for it) until a prompt chunk or a bulk load starts a new request in the slot."""
        if not 0 <= b < self.B:
            raise ValueError("no such sequence")
        for key in self._K:
            self._K[key][b] = np.zeros((0, self.Hkv, self.d))
            self._V[key][b] = np.zeros((0, self.Hkv, self.d))
            self._idle.add((key, b))

    def decode(self, layer: int, q: np.ndarray, rows: Optional[Sequence[Tuple[int, int]]] = None) -> np.ndarray:
        """q [B, Hq, d] -> out [B, Hq, d]; the query of sequence b sits at position n_b - 1
        (the group's writer has already appended this step's token).

        rows: optional list of (b, j) pairs; only those rows are computed, others are NaN.
        """
        q = np.asarray(q, dtype=np.float64).reshape(self.B, self.Hq, self.d)
        out = np.full((self.B, self.Hq, self.d), np.nan)
        todo = rows if rows is not None else [(b, j) for b in range(self.B) for j in range(self.Hq)]
        for (b, j) in todo:
            if self.is_idle(layer, b):
                out[b, j] = 0.0
                continue
            K, V = self.history(layer, b)
            n = K.shape[0]
            if n < 1:
                raise ValueError("decode on an empty cache")
            out[b, j] = self._attend(layer, b, q[b, j], j, n - 1, K, V)
        return out

    def prefill(self, layer: int, q: np.ndarray, k: Optional[np.ndarray], v: Optional[np.ndarray],
                rows: Optional[Sequence[Tuple[int, int, int]]] = None) -> np.ndarray:
        """Prompt attention for S new tokens per sequence.  q [B, S, Hq, d]; k, v [B, S, Hkv, d].

        The S tokens follow whatever the cache already holds (Section 1: the representation of
        earlier tokens does not depend on later ones, so a prompt may arrive in chunks): with
        n_b tokens held before the call, query row i of sequence b sits at position n_b + i.
        A writer layer (or any layer in duplicate mode) is given its own k, v and stores them
        first; a reader layer of a shared cache passes k = v = None and attends over the
        history its writer stored (which already includes this chunk).
        rows: optional list of (b, i, j) to compute.
        """
        q = np.asarray(q, dtype=np.float64)
        B, S = q.shape[0], q.shape[1]
        if B != self.B:
            raise ValueError("batch mismatch")
        writes = self.duplicate or self.is_writer(layer)
        if writes:
            if k is None or v is None:
                raise ValueError("writer layer needs k and v")
            first = [self.seq_len(layer, b) for b in range(B)]
            k = np.asarray(k, dtype=np.float64).reshape(B, S, self.Hkv, self.d)
            v = np.asarray(v, dtype=np.float64).reshape(B, S, self.Hkv, self.d)
            key = self._store_key(layer)
            for b in range(B):
                self._idle.discard((key, b))
                self._K[key][b] = np.concatenate([self._K[key][b], k[b]], axis=0)
                self._V[key][b] = np.concatenate([self._V[key][b], v[b]], axis=0)
        else:
            if any(self.seq_len(layer, b) < S for b in range(B)):
                raise ValueError("reader prefill needs the writer's chunk in the cache")
            first = [self.seq_len(layer, b) - S for b in range(B)]
        out = np.full((B, S, self.Hq, self.d), np.nan)
        todo = rows if rows is not None else [
            (b, i, j) for b in range(B) for i in range(S) for j in range(self.Hq)]
        for (b, i, j) in todo:
            K, V = self.history(layer, b)
            out[b, i, j] = self._attend(layer, b, q[b, i, j], j, first[b] + i, K, V)
        return out

    def prefill_ragged(self, layer: int, q: np.ndarray, k: Optional[np.ndarray], v: Optional[np.ndarray],
                       seq_lens: Sequence[int]) -> np.ndarray:
        """prefill() with a chunk length of its own per sequence (Section 4 serves requests of mixed
        lengths).  q [T, Hq, d], k, v [T, Hkv, d] packed by sequence, T = sum(seq_lens); a
        sequence with length 0 takes no part.  Row i of sequence b sits at position n_b + i."""
        q = np.asarray(q, dtype=np.float64)
        lens = [int(x) for x in seq_lens]
        if len(lens) != self.B or any(x < 0 for x in lens) or q.shape[0] != sum(lens):
            raise ValueError("seq_lens do not match the batch or the packed rows")
        first = np.concatenate([[0], np.cumsum(lens)]).astype(int)
        writes = self.duplicate or self.is_writer(layer)
        if writes:
            if k is None or v is None:
                raise ValueError("writer layer needs k and v")
            k = np.asarray(k, dtype=np.float64).reshape(-1, self.Hkv, self.d)
            v = np.asarray(v, dtype=np.float64).reshape(-1, self.Hkv, self.d)
            start = [self.seq_len(layer, b) for b in range(self.B)]
            key = self._store_key(layer)
            for b in range(self.B):
                if lens[b] > 0:
                    self._idle.discard((key, b))
                self._K[key][b] = np.concatenate([self._K[key][b], k[first[b]:first[b + 1]]], axis=0)
                self._V[key][b] = np.concatenate([self._V[key][b], v[first[b]:first[b + 1]]], axis=0)
        else:
            if any(self.seq_len(layer, b) < lens[b] for b in range(self.B)):
                raise ValueError("reader prefill needs the writer's chunk in the cache")
            start = [self.seq_len(layer, b) - lens[b] for b in range(self.B)]
        out = np.full((q.shape[0], self.Hq, self.d), np.nan)
        for b in range(self.B):
            K, V = self.history(layer, b)
            for i in range(lens[b]):
                for j in range(self.Hq):
                    out[first[b] + i, j] = self._attend(layer, b, q[first[b] + i, j], j, start[b] + i, K, V)
        return out

    def cache_view(self, layer: int, b: int) -> List[Tuple[int, int]]:
        """[(slot, position)] for every valid slot of the cache `layer` reads, sequence b."""
        sp = self.layers[self.writer[self.layers[layer].cache_id]]  # the writer's kind decides the storage
        n = self.seq_len(layer, b)
        return list(enumerate(ring_view(sp.kind, sp.window, n)))


def kv_bytes_per_token(n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """K+V bytes one token occupies in one cache."""
    return 2 * n_kv_heads * head_dim * elem_bytes


def resident_kv_tokens(layers: Sequence[LayerSpec], seq_lens: Sequence[int]) -> int:
    """Tokens held over all caches (Section 3: sliding caches hold min(n, s); a shared cache counts once)."""
    seen = {}
    for sp in layers:
        if sp.cache_id in seen:
            continue
        seen[sp.cache_id] = sum((n if sp.kind == FULL else min(n, sp.window)) for n in seq_lens)
    return sum(seen.values())


def step_read_tokens(layers: Sequence[LayerSpec], seq_lens: Sequence[int]) -> int:
    """Tokens whose K and V a decode step reads, summed over every layer (sharers re-read)."""
    return sum(sum((n if sp.kind == FULL else min(n, sp.window)) for n in seq_lens) for sp in layers)
