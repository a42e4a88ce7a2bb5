"""Brute-force loops for tiny inputs: the pin that holds the numpy oracle in place.

TEST INFRASTRUCTURE ONLY.  Pure Python, one scalar at a time, written as a
single masked softmax over EVERY token ever produced: a (query, key) pair
counts iff the key's frame is a sink frame or lies in the query chunk's window
or chunk (Sec. 3.3 of the paper, "Frame Sink" and "Short-window Attention").
The rotary step uses complex multiplication instead of the cos/sin form.
Nothing here is shared with ``longlive_oracle`` except Python itself.
"""
from __future__ import annotations

import cmath
import math


def _bf16(bits: int) -> float:
    import struct
    return struct.unpack("<f", struct.pack("<I", (int(bits) & 0xFFFF) << 16))[0]


def pair_angle(head_dim: int, pair: int, f: int, y: int, x: int, theta: float) -> float:
    d_hw = 2 * (head_dim // 6)
    d_t = head_dim - 2 * d_hw
    if pair < d_t // 2:
        return f * theta ** (-(2.0 * pair) / d_t)
    pair -= d_t // 2
    if pair < d_hw // 2:
        return y * theta ** (-(2.0 * pair) / d_hw)
    pair -= d_hw // 2
    return x * theta ** (-(2.0 * pair) / d_hw)


def rotate_vec(vec, head_dim, f, y, x, theta):
    out = [0.0] * head_dim
    for i in range(head_dim // 2):
        z = complex(vec[2 * i], vec[2 * i + 1]) * cmath.exp(1j * pair_angle(head_dim, i, f, y, x, theta))
        out[2 * i], out[2 * i + 1] = z.real, z.imag
    return out


def stream_attention(chunks, heads, head_dim, grid_h, grid_w, C, S, W, theta=10000.0, sink_relative=False):
    """chunks: list of (q_bits, k_bits, v_bits), each an [n*P, H, D] nested array
    of bf16 bit patterns, appended in order from frame 0.  Returns, per chunk, the
    attention output [n*P][H][D] as nested lists of floats.

    sink_relative: for keys of sink frames the query is rotated as if its frame index were smaller by
    max(0, f0 - W - S), f0 being the first frame of its chunk (the sink keeps a fixed rotary distance to the window).
    """
    P = grid_h * grid_w
    all_k, all_v, all_frame = [], [], []   # one entry per token ever produced
    outs = []
    f0 = 0
    for (qb, kb, vb) in chunks:
        n_tok = len(qb)
        n = n_tok // P
        q_rot, q_sink = [], []
        shift = max(0, f0 - W - S) if sink_relative else 0
        for t in range(n_tok):
            f = f0 + t // P
            y, x = divmod(t % P, grid_w)
            q_rot.append([rotate_vec([_bf16(b) for b in qb[t][h]], head_dim, f, y, x, theta) for h in range(heads)])
            q_sink.append([rotate_vec([_bf16(b) for b in qb[t][h]], head_dim, f - shift, y, x, theta) for h in range(heads)])
            all_k.append([rotate_vec([_bf16(b) for b in kb[t][h]], head_dim, f, y, x, theta) for h in range(heads)])
            all_v.append([[_bf16(b) for b in vb[t][h]] for h in range(heads)])
            all_frame.append(f)
        out = [[[0.0] * head_dim for _ in range(heads)] for _ in range(n_tok)]
        for t in range(n_tok):
            for h in range(heads):
                logits = []
                for j in range(len(all_k)):
                    g = all_frame[j]
                    visible = (g < S) or (f0 - W <= g < f0 + n)
                    if not visible:
                        logits.append(None)
                        continue
                    qv = q_sink[t][h] if g < S else q_rot[t][h]
                    dot = 0.0
                    for d in range(head_dim):
                        dot += qv[d] * all_k[j][h][d]
                    logits.append(dot / math.sqrt(head_dim))
                m = max(l for l in logits if l is not None)
                den = sum(math.exp(l - m) for l in logits if l is not None)
                for j, l in enumerate(logits):
                    if l is None:
                        continue
                    w = math.exp(l - m) / den
                    for d in range(head_dim):
                        out[t][h][d] += w * all_v[j][h][d]
        outs.append(out)
        f0 += n
    return outs
