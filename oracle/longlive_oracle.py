"""CPU oracle for short-window attention with a frame sink over a rolling KV cache.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
the HIP library must compute.  Only tests, the smoke check and the bench's
``cpu_baseline`` leg may import it.  It shares no code with the HIP path and
imports nothing from the product package.

What it follows (paper sections):
  * Sec. 3.3 "Short-window Attention": a chunk's queries attend only to a fixed
    temporal window of recent frames.
  * Sec. 3.3 "Frame Sink": the first frames of the video stay in the KV cache
    for ever and are part of every attention's keys and values; the rest of the
    cache is a short rolling window.
  * Sec. 3.3 "Consistency between Training and Inference": resident set is
    sink + last W frames of the preceding context + the current clip.
  * Sec. 3.1 "KV Recache" and Sec. 3.3 last sentence: rebuild the cache from
    the recent generated frames (re-prefill under the chunk-causal mask).
  * Appendix Alg. 2 "Interactive Inference": denoise passes use the chunk's own
    K/V but only the final clean pass leaves K/V in the cache.
  * Appendix "Implementation": chunk = 3 latent frames, window = 9, sink = 3.

The method is exact attention over a restricted key set, so the oracle is the
definition written out: it keeps every frame ever committed in a dict (it never
evicts), selects the key frames by rule, concatenates them explicitly and
computes softmax(q k^T / sqrt(D)) v in float64.  No intermediate rounding.

Readings where the paper is silent (all parameters, all restated in the design
notes): the window counts past non-sink frames, the current chunk comes on top;
scale is 1/sqrt(D); 3D rotary embedding is the factorised (frame, row, column)
form with adjacent-element pairs described at ``rope_pair_split``.

Pins (tests/test_oracle_pins.py): brute force loops, plain chunk-causal
attention through a library masked softmax, row sums, closed-form key-set
probe, eviction poisoning, key-order invariance, streaming == prefill,
cross-config equality, constant resident size, rotary closed forms; the re-prefill's
outputs (sink kept or rebuilt, short last chunks) against one masked softmax over all
retained tokens; ``error_metrics`` against hand-computed values.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np


@dataclasses.dataclass(frozen=True)
class OracleConfig:
    layers: int
    heads: int
    head_dim: int
    grid_h: int
    grid_w: int
    chunk_frames: int      # C
    sink_frames: int       # S
    window_frames: int     # W (past, non-sink frames)
    theta: float = 10000.0

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64; exact."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# 3D rotary embedding (the paper does not define one; this is the reading).
# --------------------------------------------------------------------------
def rope_pair_split(head_dim: int) -> tuple[int, int, int]:
    """Number of (re, im) pairs given to the frame, row and column axes.

    Rows and columns each get 2*floor(D/6) dims, the frame axis the rest;
    order inside the head vector: frame pairs, then row pairs, then column
    pairs.  D = 128 -> 22 | 21 | 21 pairs, D = 64 -> 12 | 10 | 10.
    """
    d_hw = 2 * (head_dim // 6)
    d_t = head_dim - 2 * d_hw
    return d_t // 2, d_hw // 2, d_hw // 2


def rope_angles(cfg: OracleConfig, f: int, y: int, x: int) -> np.ndarray:
    """Angle of each of the D/2 pairs for a token at frame f, row y, column x.

    Pair i of an axis group that owns d_a dims turns by position * theta^(-2i/d_a).
    Frame positions are absolute latent-frame indices.
    """
    n_t, n_h, n_w = rope_pair_split(cfg.head_dim)
    out = np.empty(cfg.head_dim // 2, dtype=np.float64)
    j = 0
    for n_pairs, pos in ((n_t, f), (n_h, y), (n_w, x)):
        d_a = 2 * n_pairs
        for i in range(n_pairs):
            out[j] = float(pos) * cfg.theta ** (-2.0 * i / d_a)
            j += 1
    return out


def rope_frequencies(cfg: OracleConfig) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """theta^(-2i/d_a) for the pairs of the frame, row and column axes."""
    return tuple(cfg.theta ** (-2.0 * np.arange(n, dtype=np.float64) / (2 * n)) if n else np.zeros(0)
                 for n in rope_pair_split(cfg.head_dim))


def rope_rotate(cfg: OracleConfig, x: np.ndarray, frame_start: int) -> np.ndarray:
    """Rotate x [n*P, H, D] (float64); tokens are frame-major, row-major in a frame.

    Pair (x[2i], x[2i+1]) is one complex number re + i*im, multiplied by
    exp(i*angle): re' = re*cos - im*sin, im' = re*sin + im*cos, with the angle
    of ``rope_angles`` (position times frequency, per axis).
    """
    P = cfg.tokens_per_frame
    n_tok = x.shape[0]
    assert n_tok % P == 0
    t = np.arange(n_tok)
    f = (frame_start + t // P).astype(np.float64)
    y = ((t % P) // cfg.grid_w).astype(np.float64)
    xx = ((t % P) % cfg.grid_w).astype(np.float64)
    w_t, w_h, w_w = rope_frequencies(cfg)
    ang = np.concatenate([f[:, None] * w_t[None, :], y[:, None] * w_h[None, :], xx[:, None] * w_w[None, :]], axis=1)
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    re = x[..., 0::2]
    im = x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = re * c - im * s
    out[..., 1::2] = re * s + im * c
    return out


# --------------------------------------------------------------------------
# Key-set rule (Sec. 3.3).
# --------------------------------------------------------------------------
def key_frames(cfg: OracleConfig, f0: int, n: int, existing) -> list[int]:
    """Frames whose K/V the chunk [f0, f0+n) attends to, ascending, as a set.

    sink frames [0, S)  U  the last W non-sink frames before f0  U  the chunk
    itself, limited to frames that exist.
    """
    S, W = cfg.sink_frames, cfg.window_frames
    want = set(range(0, S))
    want |= set(range(max(S, f0 - W), f0))
    want |= set(range(f0, f0 + n))
    return sorted(f for f in want if f in existing)


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, rows=None) -> np.ndarray:
    """softmax(q K^T / sqrt(D)) V per head.  q [Nq,H,D], K,V [Nk,H,D] float64.

    ``rows`` optionally restricts the computation to some query rows (each
    query's softmax is independent of the others).
    """
    if rows is not None:
        q = q[np.asarray(rows)]
    Nq, H, D = q.shape
    out = np.empty((Nq, H, D), dtype=np.float64)
    scale = 1.0 / math.sqrt(D)
    for h in range(H):
        sc = (q[:, h, :] @ K[:, h, :].T) * scale
        sc -= sc.max(axis=1, keepdims=True)
        pm = np.exp(sc)
        pm /= pm.sum(axis=1, keepdims=True)
        out[:, h, :] = pm @ V[:, h, :]
    return out


class _Layer:
    def __init__(self):
        self.committed: dict[int, tuple[np.ndarray, np.ndarray]] = {}
        self.staged = None  # (f0, n, q_rot, {frame: (K', V)})


class Oracle:
    """Streaming state for all layers; never evicts, selects by rule."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self.layer = [_Layer() for _ in range(cfg.layers)]

    # -- Alg. 2: every pass of chunk i stages its K/V; the last one stays ----
    def append(self, layer: int, frame_start: int, q_bits, k_bits, v_bits) -> np.ndarray:
        """Stage chunk [frame_start, frame_start+n).  Returns rotated q (float64).

        Same frame_start as the staged chunk: replace it (a further denoise
        pass).  frame_start == staged start + staged length: the staged chunk
        becomes permanent and the new one is staged.  Anything else: error.
        """
        cfg, L = self.cfg, self.layer[layer]
        P = cfg.tokens_per_frame
        q = bf16_bits_to_f64(q_bits)
        k = bf16_bits_to_f64(k_bits)
        v = bf16_bits_to_f64(v_bits)
        assert q.shape == k.shape == v.shape and q.shape[0] % P == 0
        n = q.shape[0] // P
        if L.staged is None:
            nxt = (max(L.committed) + 1) if L.committed else 0
            if frame_start != nxt:
                raise ValueError(f"expected frame_start {nxt}, got {frame_start}")
        else:
            s0, sn = L.staged[0], L.staged[1]
            if frame_start == s0:
                pass
            elif frame_start == s0 + sn:
                L.committed.update(L.staged[3])
            else:
                raise ValueError("frame_start neither repeats nor follows the staged chunk")
        return self._stage(layer, frame_start, q, k, v)

    def _stage(self, layer: int, frame_start: int, q, k, v) -> np.ndarray:
        """Rotate q and k at their (frame, row, column) positions and hold the chunk as staged."""
        cfg, L = self.cfg, self.layer[layer]
        P = cfg.tokens_per_frame
        n = q.shape[0] // P
        q_rot = rope_rotate(cfg, q, frame_start)
        k_rot = rope_rotate(cfg, k, frame_start)
        frames = {frame_start + i: (k_rot[i * P:(i + 1) * P], v[i * P:(i + 1) * P]) for i in range(n)}
        L.staged = (frame_start, n, q_rot, frames)
        return q_rot

    def _store(self, layer: int) -> dict:
        L = self.layer[layer]
        store = dict(L.committed)
        if L.staged is not None:
            store.update(L.staged[3])
        return store

    def live_frames(self, layer: int) -> list[int]:
        """Key frames of the staged chunk (what a bounded cache must still hold)."""
        L = self.layer[layer]
        if L.staged is None:
            raise ValueError("no staged chunk")
        return key_frames(self.cfg, L.staged[0], L.staged[1], self._store(layer))

    def gather_keys(self, layer: int, order=None):
        """Explicit concatenation of K', V over the key frames (ascending unless ``order``)."""
        store = self._store(layer)
        F = self.live_frames(layer)
        if order is not None:
            assert sorted(order) == F
            F = list(order)
        K = np.concatenate([store[f][0] for f in F], axis=0)
        V = np.concatenate([store[f][1] for f in F], axis=0)
        return K, V

    def attn(self, layer: int, rows=None, order=None) -> np.ndarray:
        """Attention of the staged chunk's rotated queries over its key frames."""
        K, V = self.gather_keys(layer, order)
        return attention(self.layer[layer].staged[2], K, V, rows)

    def frame_kv(self, layer: int, frame: int):
        """(K' float64, V float64) of a stored frame, each [P, H, D]."""
        return self._store(layer)[frame]

    # -- KV-recache: re-prefill from the retained frames ---------------------
    def recache_chunks(self, include_sink: bool, win_start: int, n_win: int):
        """[(frame_start, n_frames)] in order: the sink cut into chunks of C, then the window."""
        C, S = self.cfg.chunk_frames, self.cfg.sink_frames
        out = []
        if include_sink:
            out += [(a, min(C, S - a)) for a in range(0, S, C)]
        out += [(win_start + a, min(C, n_win - a)) for a in range(0, n_win, C)]
        return out

    def recache_prefill(self, layer: int, include_sink: bool, win_start: int, n_win: int,
                        q_bits, k_bits, v_bits, rows_per_chunk=None) -> np.ndarray:
        """Rebuild the layer from frames sink (if include_sink) + [win_start, win_start+n_win).

        q,k,v: [(S? + n_win)*P, H, D] in that frame order.  Every non-sink frame
        previously held is dropped; with include_sink false the sink frames
        already held stay as they are.  Then the chunks are streamed in order
        (append + attention each), which is the chunk-causal masked prefill.
        Returns the attention output for all query tokens, float64.
        """
        cfg, L = self.cfg, self.layer[layer]
        P, S = cfg.tokens_per_frame, cfg.sink_frames
        if S > 0 and win_start < S:
            raise ValueError("window overlaps the sink")
        keep = {} if include_sink else {f: kv for f, kv in self._store(layer).items() if f < S}
        if not include_sink and S > 0 and len(keep) != S:
            raise ValueError("sink frames not held")
        L.committed = keep
        L.staged = None
        outs = []
        tok = 0
        for (a, n) in self.recache_chunks(include_sink, win_start, n_win):
            sl = slice(tok, tok + n * P)
            if L.staged is not None:          # the chunk before this one is clean: it stays
                L.committed.update(L.staged[3])
            self._stage(layer, a, bf16_bits_to_f64(q_bits[sl]), bf16_bits_to_f64(k_bits[sl]),
                        bf16_bits_to_f64(v_bits[sl]))
            outs.append(self.attn(layer, rows_per_chunk))
            tok += n * P
        return np.concatenate(outs, axis=0)


def error_metrics(got: np.ndarray, want: np.ndarray) -> tuple[float, float]:
    """(max abs error, relative L2 error) over the whole tensor."""
    d = got.astype(np.float64) - want
    return float(np.abs(d).max()), float(np.linalg.norm(d.ravel()) / np.linalg.norm(want.ravel()))
