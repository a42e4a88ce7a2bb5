"""CPU oracle for the 8-bit (E4M3) variant of the rolling KV cache.

TEST INFRASTRUCTURE ONLY, like ``longlive_oracle`` (which it extends): only tests, the
smoke check and the bench's ``cpu_baseline`` leg may import it; it shares no code with
the HIP path.

What it states.  The paper quantises the model's weights to 8 bits after training and
reports that quality holds (Appendix, "Quantization" table: INT8 inference).  Carrying
that idea to the attention operands is this build's extension, not the paper's: rotated
keys, values and rotated queries are stored as 8-bit floating point numbers, everything
else (the key-set rule of Sec. 3.3, stage/commit of Alg. 2, the recache prefill of
Sec. 3.1) is unchanged.  Definition, for one head, with two integer exponents a and b
chosen when the cache is made:

    K8 = e4m3(K' * 2^-a)          K' = rotated key
    V8 = e4m3(V  * 2^-b)
    Q8 = e4m3(q' * c * 2^a)       q' = rotated query, c = log2(e) / sqrt(D)
    t  = Q8 . K8                  (score in the log2 domain; exact products, exact sum)
    O  = 2^b * sum_j 2^(t_j - max t) V8_j / sum_j 2^(t_j - max t)

e4m3(x) is the nearest value of the OCP 8-bit floating point format E4M3 (1 sign bit,
4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinities, largest finite
value 448), ties to the even mantissa, after |x| has been clamped to 448.  A floating
point format keeps its relative precision over 2^-6 .. 448, so one power-of-two scale
per cache (exact to apply) replaces the per-frame scales an integer format would need.
The softmax weights themselves are NOT rounded here: the HIP kernel rounds them to E4M3
before its second product, and the parity tolerance carries that (stated where the test
sets it).

Pins (tests/test_oracle_pins.py): the code table against a library's E4M3 type, the
rounding against the same library's conversion (random values, every midpoint, the
subnormal range), closed forms of the format (largest value, spacing, error bound),
brute-force search on tiny inputs, reduction to the unquantised oracle on inputs that
the format holds exactly, and the error of the quantised attention against the exact
one within the bound the format implies.
"""
from __future__ import annotations

import math

import numpy as np

from .longlive_oracle import Oracle, OracleConfig, bf16_bits_to_f64, rope_rotate

E4M3_MAX = 448.0


def e4m3_table() -> np.ndarray:
    """Value of each of the 256 codes (float64; NaN for the two NaN codes 0x7F and 0xFF).

    Code = s eeee mmm.  eeee = 0: (-1)^s * mmm/8 * 2^-6.  Otherwise (-1)^s * (1 + mmm/8) * 2^(eeee-7),
    except eeee = 1111 with mmm = 111, which is NaN (the format has no infinities).
    """
    out = np.empty(256, dtype=np.float64)
    for code in range(256):
        s = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            out[code] = math.nan
        elif e == 0:
            out[code] = s * (m / 8.0) * 2.0 ** -6
        else:
            out[code] = s * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


_POS = e4m3_table()[:0x7F]          # codes 0x00 .. 0x7E: 0 .. 448, ascending


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Codes (uint8) of the E4M3 values nearest to x; ties to the even code; |x| clamped to 448."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")          # first table value >= a
    hi = np.minimum(hi, len(_POS) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo = a - _POS[lo]
    d_hi = _POS[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))     # consecutive codes alternate mantissa parity
    code = np.where(take_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | np.uint8(0x80), code).astype(np.uint8)


def e4m3_round(x: np.ndarray) -> np.ndarray:
    """The E4M3 value nearest to x (float64), as ``e4m3_encode`` chooses it."""
    return e4m3_table()[e4m3_encode(x)]


def attention_log2(q8: np.ndarray, K8: np.ndarray, V8: np.ndarray, rows=None) -> np.ndarray:
    """sum_j 2^(t_j - max) V8_j / sum_j 2^(t_j - max), t = q8 . K8 per head; all float64."""
    if rows is not None:
        q8 = q8[np.asarray(rows)]
    Nq, H, D = q8.shape
    out = np.empty((Nq, H, D), dtype=np.float64)
    for h in range(H):
        t = q8[:, h, :] @ K8[:, h, :].T
        t -= t.max(axis=1, keepdims=True)
        w = np.exp2(t)
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ V8[:, h, :]
    return out


class Fp8Oracle(Oracle):
    """The streaming oracle with K', V and q' held as E4M3 values (see the module text)."""

    def __init__(self, cfg: OracleConfig, k_exp: int = 0, v_exp: int = 0):
        super().__init__(cfg)
        self.k_exp, self.v_exp = int(k_exp), int(v_exp)

    def _stage(self, layer: int, frame_start: int, q, k, v) -> np.ndarray:
        cfg, L = self.cfg, self.layer[layer]
        P = cfg.tokens_per_frame
        n = q.shape[0] // P
        c = math.log2(math.e) / math.sqrt(cfg.head_dim)
        q8 = e4m3_round(rope_rotate(cfg, q, frame_start) * (c * 2.0 ** self.k_exp))
        k8 = e4m3_round(rope_rotate(cfg, k, frame_start) * 2.0 ** -self.k_exp)
        v8 = e4m3_round(v * 2.0 ** -self.v_exp)
        frames = {frame_start + i: (k8[i * P:(i + 1) * P], v8[i * P:(i + 1) * P]) for i in range(n)}
        L.staged = (frame_start, n, q8, frames)
        return q8

    def attn(self, layer: int, rows=None, order=None) -> np.ndarray:
        K8, V8 = self.gather_keys(layer, order)
        return attention_log2(self.layer[layer].staged[2], K8, V8, rows) * 2.0 ** self.v_exp
