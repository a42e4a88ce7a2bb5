"""CPU oracle for the train-time rule: attention of a supervised clip over sink + detached window + the clip itself,
and its gradients with respect to the clip's own q, k and v.

TEST INFRASTRUCTURE ONLY.  Plain fp64 numpy; only tests, the smoke check and the bench's ``cpu_baseline`` leg may
import it.  It shares no code with the HIP path and imports nothing from the product package.

What it follows: Sec. 3.2 (streaming long tuning: the frames generated so far are detached and act as a constant
causal context, gradients are computed for the current clip only) and Sec. 3.3 "Consistency between Training and
Inference": per training step the resident keys and values are (i) the last W frames of the preceding context,
without gradients, (ii) the T frames of the supervised clip, with gradients, and (iii) the S sink frames; the same
short window and sink as at inference.  Alg. 1 generates the clip chunk by chunk, so the clip's chunks follow the
inference rule one after the other: a chunk starting at frame f0 attends to the sink, to the last W non-sink frames
before f0 (context frames or earlier frames of the clip) and to itself.

The forward is that rule written out with the key-set function of the inference oracle.  The backward is the
derivative of exactly that forward: for one chunk with keys K', values V and rotated queries q',
    Z = q' K'^T / sqrt(D),  P = softmax(Z),  out = P V,
    dV = P^T dOut,  dP = dOut V^T,  dZ = P * (dP - rowsum(P * dP)),  dq' = dZ K' / sqrt(D),  dK' = dZ^T q' / sqrt(D),
summed over the chunks a key takes part in, and carried back through the rotary embedding (a rotation per pair, so
the transpose is the rotation by the opposite angle).  Only rows of the clip's own frames are returned; context and
(unless they belong to the clip) sink frames are constants.

Readings: the window counts frames before the chunk regardless of whether they are context or clip frames; the first
clip of a video (no context yet) contains the sink frames itself and they then receive gradients like any clip frame.

Pins (tests/test_oracle_pins.py): central finite differences of the forward in random directions, a library's
reverse-mode differentiation of a masked attention written with library ops, zero gradient to anything outside the
key set (window eviction inside a long clip), equality of a first clip's forward with the inference oracle
streamed from frame 0, and the sampled form of the backward against the full one.
"""
from __future__ import annotations

import math

import numpy as np

from oracle.longlive_oracle import OracleConfig, key_frames, rope_angles, rope_rotate


def _unrotate_grad(cfg: OracleConfig, g: np.ndarray, frame_start: int) -> np.ndarray:
    """Gradient w.r.t. x of a loss whose gradient w.r.t. rope_rotate(x) is g: the rotation by the opposite angle.
    Done by rotating forward and reflecting: R(-a) g = conj(R(a) conj(g)) for each (re, im) pair."""
    c = g.copy()
    c[..., 1::2] *= -1.0
    r = rope_rotate(cfg, c, frame_start)
    r[..., 1::2] *= -1.0
    return r


class ClipOracle:
    """One layer, one training step.  ``forward`` keeps what ``backward`` needs."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self._saved = None

    def clip_chunks(self, clip_start: int, n_clip: int):
        """(f0, n) of the clip's chunks: C frames each, a shorter last one if n_clip is no multiple of C."""
        C = self.cfg.chunk_frames
        return [(f, min(C, clip_start + n_clip - f)) for f in range(clip_start, clip_start + n_clip, C)]

    def frames(self, ctx_start: int, n_ctx: int, n_clip: int):
        """All resident frames, ascending: sink, context, clip (a sink frame inside the clip is listed once)."""
        S = self.cfg.sink_frames
        clip_start = ctx_start + n_ctx
        have = set(range(ctx_start, clip_start + n_clip))
        if ctx_start >= S:
            have |= set(range(S))
        return sorted(have)

    def forward(self, ctx_start: int, n_ctx: int, n_clip: int, q: np.ndarray, k: np.ndarray, v: np.ndarray):
        """q [n_clip*P, H, D]: the clip's queries.  k, v [n_frames*P, H, D]: keys and values of ``frames(...)`` in that
        order (all float64, unrotated).  Returns out [n_clip*P, H, D]."""
        cfg, P = self.cfg, self.cfg.tokens_per_frame
        clip_start = ctx_start + n_ctx
        fr = self.frames(ctx_start, n_ctx, n_clip)
        assert ctx_start >= cfg.sink_frames or ctx_start == 0, "context must not cut into the sink"
        assert k.shape[0] == len(fr) * P and v.shape == k.shape and q.shape[0] == n_clip * P
        pos = {f: i for i, f in enumerate(fr)}
        k_rot = np.concatenate([rope_rotate(cfg, k[pos[f] * P:(pos[f] + 1) * P], f) for f in fr])
        q_rot = rope_rotate(cfg, q, clip_start)
        out = np.empty_like(q_rot)
        scale = 1.0 / math.sqrt(cfg.head_dim)
        steps = []
        for f0, n in self.clip_chunks(clip_start, n_clip):
            keys = key_frames(cfg, f0, n, [f for f in fr if f < f0 + n])
            kidx = np.concatenate([np.arange(pos[f] * P, (pos[f] + 1) * P) for f in keys])
            rows = slice((f0 - clip_start) * P, (f0 - clip_start + n) * P)
            for h in range(cfg.heads):
                out[rows, h, :] = self._softmax(q_rot[rows, h, :], k_rot[kidx, h, :], scale) @ v[kidx, h, :]
            steps.append((rows, kidx))
        self._saved = (ctx_start, n_ctx, n_clip, fr, pos, q_rot, k_rot, v, steps)
        return out

    @staticmethod
    def _softmax(qh: np.ndarray, kh: np.ndarray, scale: float) -> np.ndarray:
        z = (qh @ kh.T) * scale
        z -= z.max(axis=1, keepdims=True)
        e = np.exp(z)
        return e / e.sum(axis=1, keepdims=True)

    def backward(self, dout: np.ndarray):
        """dout [n_clip*P, H, D] -> (dq, dk, dv), each [n_clip*P, H, D]: gradients of sum(out * dout) with respect to
        the clip's own unrotated q, k and v."""
        cfg, P = self.cfg, self.cfg.tokens_per_frame
        ctx_start, n_ctx, n_clip, fr, pos, q_rot, k_rot, v, steps = self._saved
        clip_start = ctx_start + n_ctx
        scale = 1.0 / math.sqrt(cfg.head_dim)
        dq_rot = np.zeros_like(q_rot)
        dk_rot = np.zeros_like(k_rot)
        dv_all = np.zeros_like(v)
        for rows, kidx in steps:
            for h in range(cfg.heads):
                p = self._softmax(q_rot[rows, h, :], k_rot[kidx, h, :], scale)      # the forward's weights again
                do = dout[rows, h, :]
                dv_all[kidx, h, :] += p.T @ do
                dp = do @ v[kidx, h, :].T
                dz = p * (dp - (p * dp).sum(axis=1, keepdims=True))
                dq_rot[rows, h, :] = (dz @ k_rot[kidx, h, :]) * scale
                dk_rot[kidx, h, :] += (dz.T @ q_rot[rows, h, :]) * scale
        first = pos[clip_start] * P
        assert fr[pos[clip_start]:] == list(range(clip_start, clip_start + n_clip))      # the clip is the tail
        dq = _unrotate_grad(cfg, dq_rot, clip_start)
        dk = _unrotate_grad(cfg, dk_rot[first:], clip_start)
        return dq, dk, dv_all[first:]

    def backward_sample(self, dout: np.ndarray, q_rows, key_rows):
        """The same gradients for a sample only: rows ``q_rows`` of dq and rows ``key_rows`` of dk and dv (indices into
        the clip's tokens), all heads of the tensors given to ``forward``.  Same formulas; only the chunks that hold a
        sampled query or see a sampled key are visited.  For shapes at which the full backward would take minutes."""
        cfg, P = self.cfg, self.cfg.tokens_per_frame
        ctx_start, n_ctx, n_clip, fr, pos, q_rot, k_rot, v, steps = self._saved
        clip_start = ctx_start + n_ctx
        first = pos[clip_start] * P
        scale = 1.0 / math.sqrt(cfg.head_dim)
        q_rows, key_rows = np.asarray(q_rows, dtype=np.int64), np.asarray(key_rows, dtype=np.int64)
        dq_rot = np.zeros((q_rows.size,) + q_rot.shape[1:])
        dk_rot = np.zeros((key_rows.size,) + q_rot.shape[1:])
        dv = np.zeros_like(dk_rot)
        for rows, kidx in steps:
            in_chunk = np.nonzero((q_rows >= rows.start) & (q_rows < rows.stop))[0]
            where = {int(t): i for i, t in enumerate(kidx)}
            seen = [(n, where[first + int(j)]) for n, j in enumerate(key_rows) if first + int(j) in where]
            if in_chunk.size == 0 and not seen:
                continue
            for h in range(cfg.heads):
                if seen:                                     # every query of the chunk contributes to a key it sees
                    p = self._softmax(q_rot[rows, h, :], k_rot[kidx, h, :], scale)
                    do = dout[rows, h, :]
                    dp = do @ v[kidx, h, :].T
                    dz = p * (dp - (p * dp).sum(axis=1, keepdims=True))
                    for n, col in seen:
                        dv[n, h, :] += p[:, col] @ do
                        dk_rot[n, h, :] += (dz[:, col] @ q_rot[rows, h, :]) * scale
                if in_chunk.size:
                    r = q_rows[in_chunk]
                    p = self._softmax(q_rot[r, h, :], k_rot[kidx, h, :], scale)
                    dp = dout[r, h, :] @ v[kidx, h, :].T
                    dz = p * (dp - (p * dp).sum(axis=1, keepdims=True))
                    dq_rot[in_chunk, h, :] = (dz @ k_rot[kidx, h, :]) * scale
        # back through the rotary turn, token by token
        def unrotate(g, tokens):
            out = np.empty_like(g)
            for n, t in enumerate(tokens):
                f, y, x = clip_start + int(t) // P, (int(t) % P) // cfg.grid_w, (int(t) % P) % cfg.grid_w
                a = rope_angles(cfg, f, y, x)
                c, sn = np.cos(a)[None, :], np.sin(a)[None, :]
                re, im = g[n, :, 0::2], g[n, :, 1::2]
                out[n, :, 0::2] = re * c + im * sn            # the rotation by -a
                out[n, :, 1::2] = im * c - re * sn
            return out
        return unrotate(dq_rot, q_rows), unrotate(dk_rot, key_rows), dv

