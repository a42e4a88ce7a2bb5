"""CPU oracle for the variant in which the sink keeps a fixed rotary distance to the window.

TEST INFRASTRUCTURE ONLY, like ``longlive_oracle`` (which it extends).

The paper keeps the first frames as a sink for videos of any length (Sec. 3.3 "Frame Sink"; Appendix, ultra-long
videos of 240 s) and says nothing about the positions the rotary embedding gives them.  With absolute frame positions
the rotary distance between a query and the sink grows with the video without bound, beyond anything seen in
training.  This variant is this build's own reading of how to bound it; it changes nothing else:

    Delta(f0) = max(0, f0 - W - S)          f0 = first frame of the query chunk
    score(query at frame fq, key at frame fk):
        fk >= S (window, chunk):  rotary distance fq - fk                     (as before)
        fk <  S (sink):           rotary distance (fq - Delta(f0)) - fk

i.e. seen from the queries, the sink frames sit at positions 0 .. S-1 and the oldest window frame at position S,
however long the video is; only the frame axis of the rotary embedding is concerned, rows and columns keep their
positions.  While the window still touches the sink (f0 <= W + S) Delta is 0 and nothing differs from the plain
rule.  The oracle writes the definition out: the sink keys are taken as stored (rotated at their own frames), the
queries are rotated a second time from their unrotated values at frame positions reduced by Delta, the two blocks of
scores are concatenated and go through one softmax.

Pins (tests/test_oracle_pins.py): equality with the plain oracle while Delta = 0, brute-force loops with explicit
angles, and the property the variant exists for: outputs do not depend on where in the video the window lies.
"""
from __future__ import annotations

import math

import numpy as np

from .longlive_oracle import Oracle, OracleConfig, rope_rotate


class SinkRelativeOracle(Oracle):
    def __init__(self, cfg: OracleConfig):
        super().__init__(cfg)
        self._raw_q = [None] * cfg.layers

    def delta(self, f0: int) -> int:
        return max(0, f0 - self.cfg.window_frames - self.cfg.sink_frames)

    def _stage(self, layer: int, frame_start: int, q, k, v) -> np.ndarray:
        self._raw_q[layer] = q
        return super()._stage(layer, frame_start, q, k, v)

    def attn(self, layer: int, rows=None, order=None) -> np.ndarray:
        assert order is None
        cfg, L = self.cfg, self.layer[layer]
        f0, n, q_rot, _ = L.staged
        store = self._store(layer)
        frames = self.live_frames(layer)
        sink = [f for f in frames if f < cfg.sink_frames]
        rest = [f for f in frames if f >= cfg.sink_frames]
        q_sink = rope_rotate(cfg, self._raw_q[layer], f0 - self.delta(f0))
        if rows is not None:
            q_rot, q_sink = q_rot[np.asarray(rows)], q_sink[np.asarray(rows)]
        Nq, H, D = q_rot.shape
        K_s = np.concatenate([store[f][0] for f in sink]) if sink else np.zeros((0, H, D))
        K_r = np.concatenate([store[f][0] for f in rest]) if rest else np.zeros((0, H, D))
        V = np.concatenate([store[f][1] for f in sink + rest])
        out = np.empty((Nq, H, D), dtype=np.float64)
        scale = 1.0 / math.sqrt(D)
        for h in range(H):
            sc = np.concatenate([q_sink[:, h, :] @ K_s[:, h, :].T, q_rot[:, h, :] @ K_r[:, h, :].T], axis=1) * scale
            sc -= sc.max(axis=1, keepdims=True)
            pm = np.exp(sc)
            pm /= pm.sum(axis=1, keepdims=True)
            out[:, h, :] = pm @ V[:, h, :]
        return out
