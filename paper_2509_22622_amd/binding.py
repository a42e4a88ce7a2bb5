"""ctypes binding of the C-ABI in ``include/longlive.h``: argument marshalling only.

Every step of the hot path runs in the HIP library.  There is no fallback: if the
library is missing or a call fails, an exception is raised.  torch is used for
device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblonglive.so")
_lib = None

LL_OK, LL_ERR_INVALID_ARG, LL_ERR_STATE, LL_ERR_BUFFER_TOO_SMALL, LL_ERR_UNSUPPORTED, LL_ERR_HIP = range(6)
STATUS_NAMES = {0: "LL_OK", 1: "LL_ERR_INVALID_ARG", 2: "LL_ERR_STATE", 3: "LL_ERR_BUFFER_TOO_SMALL",
                4: "LL_ERR_UNSUPPORTED", 5: "LL_ERR_HIP"}

# name -> (restype, argtypes); mirrors include/longlive.h
_vp, _i, _i64, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
SIGNATURES = {
    "ll_cache_bytes": (_sz, [_i] * 7),
    "ll_cache_create": (_i, [_i] * 9 + [C.c_float, _vp, _sz, C.POINTER(_vp)]),
    "ll_cache_bytes_fp8": (_sz, [_i] * 7),
    "ll_cache_create_fp8": (_i, [_i] * 9 + [C.c_float, _i, _i, _vp, _sz, C.POINTER(_vp)]),
    "ll_cache_destroy": (_i, [_vp]),
    "ll_cache_reset": (_i, [_vp, _i]),
    "ll_chunk_append": (_i, [_vp, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp]),
    "ll_sink_window_attn": (_i, [_vp, _i, _vp, _vp, _vp]),
    "ll_sink_window_attn_unrotated": (_i, [_vp, _i, _vp, _vp, _vp]),
    "ll_recache_prefill": (_i, [_vp, _i, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp]),
    "ll_recache_prefill_static": (_i, [_vp, _i, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp]),
    "ll_cache_live_frames": (_i, [_vp, _i, C.POINTER(_i64), _i, C.POINTER(_i)]),
    "ll_cache_slot_of_frame": (_i, [_vp, _i, _i64, C.POINTER(_i64)]),
    "ll_cache_live_ranges": (_i, [_vp, _i, C.POINTER(_i64), _i, C.POINTER(_i)]),
    "ll_cache_read_frame": (_i, [_vp, _i, _i64, _vp, _vp, _vp]),
    "ll_cache_set_sink_relative": (_i, [_vp, _i]),
    "ll_prompt_bytes": (_sz, [_i] * 4),
    "ll_prompt_create": (_i, [_i] * 4 + [_vp, _sz, C.POINTER(_vp)]),
    "ll_prompt_destroy": (_i, [_vp]),
    "ll_prompt_recache": (_i, [_vp, _i, _vp, _vp, _i, _vp]),
    "ll_prompt_tokens": (_i, [_vp, _i, C.POINTER(_i)]),
    "ll_cross_attn": (_i, [_vp, _i, _vp, _i, _vp, _vp]),
    "ll_cross_attn_out": (_i, [_vp, _i, _vp, _i, _vp, _vp, _vp, _vp]),
    "ll_out_proj_pack_weight": (_i, [_i, _i, _vp, _vp, _vp]),
    "ll_cross_attn_out_workspace_bytes": (C.c_size_t, [_i, _i, _i]),
    "ll_clip_bytes": (_sz, [_i] * 7),
    "ll_clip_create": (_i, [_i] * 9 + [C.c_float, _vp, _sz, C.POINTER(_vp)]),
    "ll_clip_destroy": (_i, [_vp]),
    "ll_clip_forward": (_i, [_vp, _i64, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "ll_clip_backward": (_i, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "ll_clip_chunk_key_ranges": (_i, [_vp, _i, C.POINTER(_i64), _i, C.POINTER(_i)]),
    "ll_set_attn_variant": (_i, [_i]),
    "ll_attn_variant_name": (C.c_char_p, [_i]),
    "ll_probe_mfma_rate": (_i, [C.c_void_p, C.c_size_t, _i, _i, _i, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]),
    "ll_probe_mfma_mix": (_i, [C.c_void_p, C.c_size_t, _i, _i, _i, _i, _i, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]),
    "ll_status_string": (C.c_char_p, [_i]),
    "ll_last_error": (C.c_char_p, []),
}


class LongLiveError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def lib() -> C.CDLL:
    """Load liblonglive.so (built by ``paper_2509_22622_amd.build``); raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2509_22622_amd.build`")
        # torch first: it ships its own copy of the HIP runtime, and the library must bind to the copy that owns
        # the process's device memory and streams.  Loaded the other way round, the process holds two runtimes and
        # the library's own one finds no device.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != LL_OK:
        raise LongLiveError(status, lib().ll_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def cache_bytes(layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames, kv_format="bf16") -> int:
    fn = lib().ll_cache_bytes_fp8 if kv_format == "fp8_e4m3" else lib().ll_cache_bytes
    return fn(layers, heads, head_dim, tokens_per_frame, sink_frames, window_frames, chunk_frames)


def set_attn_variant(variant: int) -> None:
    _check(lib().ll_set_attn_variant(variant))


def probe_mfma_rate(workgroups: int = 256, iters: int = 20000, random_operands: bool = True):
    """(TFLOP/s, core clock in GHz) of a pure 32x32x16 bf16 MFMA stream on the current device."""
    import torch
    scratch = torch.empty(workgroups * 2048 + 16, dtype=torch.uint8, device="cuda")
    tflops, ghz = C.c_double(), C.c_double()
    _check(lib().ll_probe_mfma_rate(C.c_void_p(scratch.data_ptr()), scratch.numel(), workgroups, iters,
                                    int(random_operands), C.byref(tflops), C.byref(ghz), _stream()))
    return tflops.value, ghz.value


PROBE_COMPANIONS = {0: "none", 1: "v_add_f32", 2: "v_exp_f32", 3: "v_cvt_pk_bf16_f32", 4: "v_dot2c_f32_bf16",
                    5: "v_max3_f32", 6: "ds_read_b128", 7: "16x16x32 MFMAs, no companion"}
PROBE_FP8_KINDS = {8: "fp8 32x32x64 MFMAs alone", 9: "+ the 8-bit kernel's vector and LDS work per MFMA",
                   10: "+ its vector work only (4 exp2, 4 add, 2 cvt, 2 max3)", 11: "+ its LDS reads only (2 x 16 B)"}


def probe_mfma_mix(companion: int, per_mfma: int = 1, workgroups: int = 256, iters: int = 20000, random_operands: bool = True):
    """(MFMA TFLOP/s, core clock in GHz) with `per_mfma` companion instructions behind every MFMA (see the header)."""
    import torch
    scratch = torch.empty(workgroups * 2048 + 16, dtype=torch.uint8, device="cuda")
    tflops, ghz = C.c_double(), C.c_double()
    _check(lib().ll_probe_mfma_mix(C.c_void_p(scratch.data_ptr()), scratch.numel(), workgroups, iters, int(random_operands),
                                   companion, per_mfma, C.byref(tflops), C.byref(ghz), _stream()))
    return tflops.value, ghz.value


def attn_variant_names() -> dict:
    out, v = {}, 1
    while True:
        n = lib().ll_attn_variant_name(v)
        if n is None:
            return out
        out[v] = n.decode()
        v += 1


class Cache:
    """Handle on ``layers`` rolling KV caches.  ``device=None`` makes an index-only handle.

    ``kv_format="fp8_e4m3"`` makes the 8-bit cache (``ll_cache_create_fp8``): q_out of ``chunk_append`` and the
    tensors of ``read_frame`` are then uint8 (E4M3 codes) of the same shape; everything else stays bfloat16.
    """

    def __init__(self, layers, heads, head_dim, grid_h, grid_w, chunk_frames, sink_frames, window_frames,
                 rope_theta=10000.0, device="cuda", kv_format="bf16", k_exp=0, v_exp=0):
        if kv_format not in ("bf16", "fp8_e4m3"):
            raise ValueError(f"kv_format {kv_format!r}")
        self.kv_format = kv_format
        self.layers, self.heads, self.head_dim = layers, heads, head_dim
        self.grid_h, self.grid_w = grid_h, grid_w
        self.P = grid_h * grid_w
        self.C, self.S, self.W = chunk_frames, sink_frames, window_frames
        self._h = C.c_void_p()
        self.buffer = None
        nbytes = cache_bytes(layers, heads, head_dim, self.P, sink_frames, window_frames, chunk_frames, kv_format)
        if device is not None:
            import torch
            if nbytes == 0:
                raise LongLiveError(1, "invalid shape")
            self.buffer = torch.empty(nbytes, dtype=torch.uint8, device=device)
            ptr, size = C.c_void_p(self.buffer.data_ptr()), nbytes
        else:
            ptr, size = None, 0
        if kv_format == "fp8_e4m3":
            _check(lib().ll_cache_create_fp8(layers, heads, head_dim, self.P, sink_frames, window_frames, chunk_frames,
                                             grid_h, grid_w, rope_theta, k_exp, v_exp, ptr, size, C.byref(self._h)))
        else:
            _check(lib().ll_cache_create(layers, heads, head_dim, self.P, sink_frames, window_frames, chunk_frames,
                                         grid_h, grid_w, rope_theta, ptr, size, C.byref(self._h)))

    def close(self):
        if self._h:
            lib().ll_cache_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_sink_relative(self, on: bool) -> None:
        """Sink at a fixed rotary distance from the window (see ``ll_cache_set_sink_relative``)."""
        _check(lib().ll_cache_set_sink_relative(self._h, int(bool(on))))

    def reset(self, layer=-1):
        _check(lib().ll_cache_reset(self._h, layer))

    def chunk_append(self, layer, frame_start, n_frames, q=None, k=None, v=None, q_out=None):
        """q and q_out None with k, v given: keys and values only (the queries go to sink_window_attn_unrotated)."""
        stream = _stream() if k is not None else None
        _check(lib().ll_chunk_append(self._h, layer, frame_start, n_frames, _ptr(q), _ptr(k), _ptr(v), _ptr(q_out), stream))

    def sink_window_attn(self, layer, q_roped, out):
        _check(lib().ll_sink_window_attn(self._h, layer, _ptr(q_roped), _ptr(out), _stream()))

    def sink_window_attn_unrotated(self, layer, q, out):
        """The same attention from the chunk's unrotated, unscaled queries (the kernel turns them on load)."""
        _check(lib().ll_sink_window_attn_unrotated(self._h, layer, _ptr(q), _ptr(out), _stream()))

    def recache_prefill(self, layer, include_sink, win_start, n_win, q=None, k=None, v=None, out=None):
        stream = _stream() if q is not None else None
        _check(lib().ll_recache_prefill(self._h, layer, int(include_sink), win_start, n_win, _ptr(q), _ptr(k), _ptr(v),
                                        _ptr(out), stream))

    def recache_prefill_static(self, layer, include_sink, win_start, n_win, q=None, k=None, v=None, out=None):
        stream = _stream() if q is not None else None
        _check(lib().ll_recache_prefill_static(self._h, layer, int(include_sink), win_start, n_win, _ptr(q), _ptr(k),
                                               _ptr(v), _ptr(out), stream))

    def live_frames(self, layer):
        cap = self.S + self.W + self.C + 1
        buf, n = (C.c_int64 * cap)(), C.c_int()
        _check(lib().ll_cache_live_frames(self._h, layer, buf, cap, C.byref(n)))
        return list(buf[: n.value])

    def slot_of_frame(self, layer, frame):
        s = C.c_int64()
        _check(lib().ll_cache_slot_of_frame(self._h, layer, frame, C.byref(s)))
        return s.value

    def live_ranges(self, layer):
        buf, n = (C.c_int64 * 16)(), C.c_int()
        _check(lib().ll_cache_live_ranges(self._h, layer, buf, 8, C.byref(n)))
        return [(buf[2 * i], buf[2 * i + 1]) for i in range(n.value)]

    def read_frame(self, layer, frame, k_out, v_out):
        _check(lib().ll_cache_read_frame(self._h, layer, frame, _ptr(k_out), _ptr(v_out), _stream()))


class Prompt:
    """Handle on the per-layer keys and values of the active prompt (``ll_prompt_*``, ``ll_cross_attn``).
    ``device=None`` makes an index-only handle."""

    def __init__(self, layers, heads, head_dim, max_tokens, device="cuda"):
        self.layers, self.heads, self.head_dim, self.max_tokens = layers, heads, head_dim, max_tokens
        self._h = C.c_void_p()
        self.buffer = None
        nbytes = lib().ll_prompt_bytes(layers, heads, head_dim, max_tokens)
        if device is not None:
            import torch
            if nbytes == 0:
                raise LongLiveError(1, "invalid shape")
            self.buffer = torch.empty(nbytes, dtype=torch.uint8, device=device)
            ptr, size = C.c_void_p(self.buffer.data_ptr()), nbytes
        else:
            ptr, size = None, 0
        _check(lib().ll_prompt_create(layers, heads, head_dim, max_tokens, ptr, size, C.byref(self._h)))

    def close(self):
        if self._h:
            lib().ll_prompt_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def recache(self, layer, k, v, n_tokens=None):
        """Replace the layer's prompt keys and values: k, v bf16 [n_tokens, H, D] on the device."""
        if n_tokens is None:
            n_tokens = k.shape[0]
        if self.buffer is not None:
            _check(lib().ll_prompt_recache(self._h, layer, _ptr(k), _ptr(v), n_tokens, _stream()))
        else:
            _check(lib().ll_prompt_recache(self._h, layer, None, None, n_tokens, None))

    def tokens(self, layer) -> int:
        n = C.c_int()
        _check(lib().ll_prompt_tokens(self._h, layer, C.byref(n)))
        return n.value

    def cross_attn(self, layer, q, out, n_q=None):
        """out = softmax(q k^T / sqrt(D)) v over the layer's prompt; q, out bf16 [n_q, H, D] on the device."""
        if n_q is None:
            n_q = q.shape[0]
        if self.buffer is not None:
            _check(lib().ll_cross_attn(self._h, layer, _ptr(q), n_q, _ptr(out), _stream()))
        else:
            _check(lib().ll_cross_attn(self._h, layer, None, n_q, None, None))

    def pack_out_weight(self, w_out, w_packed):
        """The layer's output weight (bf16 [H*D, H*D], [output feature][input feature]) in the projection's order."""
        _check(lib().ll_out_proj_pack_weight(self.heads, self.head_dim, _ptr(w_out), _ptr(w_packed), _stream()))

    def cross_attn_out_workspace_bytes(self, n_q) -> int:
        return lib().ll_cross_attn_out_workspace_bytes(self.heads, self.head_dim, n_q)

    def cross_attn_out(self, layer, q=None, w_packed=None, workspace=None, y=None, n_q=None):
        """Cross-attention followed by the output projection y = concat_heads(attention output) w_out^T; w_packed from
        pack_out_weight, workspace of cross_attn_out_workspace_bytes(n_q) bytes."""
        if q is not None:
            n_q = q.shape[0]
            _check(lib().ll_cross_attn_out(self._h, layer, _ptr(q), n_q, _ptr(w_packed), _ptr(workspace), _ptr(y), _stream()))
        else:
            _check(lib().ll_cross_attn_out(self._h, layer, None, n_q, None, None, None, None))


class Clip:
    """Handle on one layer's training step: attention of a supervised clip over sink + detached window + itself
    (``ll_clip_forward``) and its gradients (``ll_clip_backward``).  ``device=None`` makes an index-only handle."""

    def __init__(self, heads, head_dim, grid_h, grid_w, chunk_frames, sink_frames, window_frames, clip_frames,
                 rope_theta=10000.0, device="cuda"):
        self.heads, self.head_dim, self.P = heads, head_dim, grid_h * grid_w
        self._h = C.c_void_p()
        self.buffer = None
        nbytes = lib().ll_clip_bytes(heads, head_dim, self.P, sink_frames, window_frames, clip_frames, chunk_frames)
        if device is not None:
            import torch
            if nbytes == 0:
                raise LongLiveError(1, "invalid shape")
            self.buffer = torch.empty(nbytes, dtype=torch.uint8, device=device)
            ptr, size = C.c_void_p(self.buffer.data_ptr()), nbytes
        else:
            ptr, size = None, 0
        _check(lib().ll_clip_create(heads, head_dim, self.P, sink_frames, window_frames, clip_frames, chunk_frames,
                                    grid_h, grid_w, rope_theta, ptr, size, C.byref(self._h)))

    def close(self):
        if self._h:
            lib().ll_clip_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def forward(self, ctx_start, n_ctx, n_clip, q=None, k=None, v=None, out=None):
        stream = _stream() if self.buffer is not None else None
        _check(lib().ll_clip_forward(self._h, ctx_start, n_ctx, n_clip, _ptr(q), _ptr(k), _ptr(v), _ptr(out), stream))

    def chunk_key_ranges(self, chunk):
        """Key set of one chunk of the last forward: [(begin, end)] token-slot ranges into the resident frames."""
        buf, n = (C.c_int64 * 4)(), C.c_int()
        _check(lib().ll_clip_chunk_key_ranges(self._h, chunk, buf, 2, C.byref(n)))
        return [(buf[2 * i], buf[2 * i + 1]) for i in range(n.value)]

    def backward(self, dout=None, dq=None, dk=None, dv=None):
        stream = _stream() if self.buffer is not None else None
        _check(lib().ll_clip_backward(self._h, _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), stream))
