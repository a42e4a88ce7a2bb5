"""Host bookkeeping of the library (index-only handles, no GPU) against the oracle's key-set rule.

Integers must agree exactly: live frames, the slot map, and the merged slot ranges.
"""
import random
import re
import shutil
import subprocess

import ctypes as C
import os

import numpy as np
import pytest

from oracle.longlive_oracle import OracleConfig, key_frames
from paper_2509_22622_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _check_ranges(cache, cfg, frames):
    P, S, R = cfg.tokens_per_frame, cfg.sink_frames, cfg.window_frames + cfg.chunk_frames
    slots = []
    for f in frames:
        want = f * P if f < S else (S + (f - S) % R) * P       # canonical map
        assert cache.slot_of_frame(0, f) == want
        slots.append(want)
    assert len(set(slots)) == len(slots)                       # live frames never share a slot
    ranges = cache.live_ranges(0)
    assert 1 <= len(ranges) <= 3
    covered = set()
    prev_end = -1
    for (a, b) in ranges:
        assert a < b and a > prev_end                          # ascending, disjoint, not touching
        prev_end = b
        assert a % P == 0 and b % P == 0
        covered |= set(range(a // P, b // P))
    assert covered == {s // P for s in slots}


@pytest.mark.parametrize("seed", range(40))
def test_streaming_live_sets_match_oracle(seed):
    rnd = random.Random(seed)
    Cc = rnd.choice([1, 2, 3, 4])
    S = rnd.choice([0, 1, 2, 3, 4, 6])
    W = rnd.choice([0, 1, 2, 3, 5, 6, 9, 21])
    cfg = OracleConfig(1, 1, 64, 1, rnd.choice([1, 3, 8]), Cc, S, W)
    cache = B.Cache(1, 1, 64, cfg.grid_h, cfg.grid_w, Cc, S, W, device=None)
    existing, f0 = set(), 0
    for step in range(rnd.choice([5, 30, 70])):
        n = Cc if rnd.random() < 0.8 else rnd.randint(1, Cc)
        for rep in range(rnd.choice([1, 1, 3])):              # repeated passes overwrite the staged chunk
            m = n if rep else rnd.randint(n, Cc)              # an earlier pass may have been longer
            existing -= set(range(f0, f0 + Cc))
            existing |= set(range(f0, f0 + (n if rep else m)))
            cache.chunk_append(0, f0, n if rep else m)
            cur = n if rep else m
        want = key_frames(cfg, f0, cur, existing)
        assert cache.live_frames(0) == want
        _check_ranges(cache, cfg, want)
        f0 += cur
    cache.close()


@pytest.mark.parametrize("S,W,Cc", [(3, 9, 3), (3, 6, 3), (0, 21, 3), (2, 5, 3), (4, 3, 2)])
def test_long_rollout_resident_size_is_constant(S, W, Cc):
    cfg = OracleConfig(1, 1, 64, 2, 2, Cc, S, W)
    cache = B.Cache(1, 1, 64, 2, 2, Cc, S, W, device=None)
    existing = set()
    for i in range(320):                                       # 240 s of video
        f0 = i * Cc
        existing |= set(range(f0, f0 + Cc))
        cache.chunk_append(0, f0, Cc)
        got = cache.live_frames(0)
        assert got == key_frames(cfg, f0, Cc, existing)
        if f0 >= S + W:
            assert len(got) == S + W + Cc
            assert sum(b - a for a, b in cache.live_ranges(0)) == (S + W + Cc) * cfg.tokens_per_frame
    cache.close()


@pytest.mark.parametrize("seed", range(20))
def test_recache_bookkeeping(seed):
    rnd = random.Random(1000 + seed)
    Cc = rnd.choice([2, 3])
    S = rnd.choice([0, 2, 3])
    W = rnd.choice([3, 6, 9])
    cfg = OracleConfig(1, 1, 64, 1, 2, Cc, S, W)
    cache = B.Cache(1, 1, 64, 1, 2, Cc, S, W, device=None)
    n_pre = rnd.randint(3, 20)
    for i in range(n_pre):
        cache.chunk_append(0, i * Cc, Cc)
    hi = n_pre * Cc
    if hi <= S:
        return
    n_win = min(W + Cc, hi - S)
    n_win = rnd.randint(1, n_win)
    ws = hi - n_win
    include_sink = rnd.random() < 0.5
    cache.recache_prefill(0, include_sink, ws, n_win)
    existing = set(range(S)) | set(range(ws, hi))
    last_f0 = ws + ((n_win - 1) // Cc) * Cc
    assert cache.live_frames(0) == key_frames(cfg, last_f0, hi - last_f0, existing)
    f0 = hi
    for i in range(8):
        existing |= set(range(f0, f0 + Cc))
        cache.chunk_append(0, f0, Cc)
        want = key_frames(cfg, f0, Cc, existing)
        assert cache.live_frames(0) == want
        _check_ranges(cache, cfg, want)
        f0 += Cc
    cache.close()


def test_error_paths():
    L = B.lib()
    assert B.cache_bytes(1, 4, 96, 60, 3, 6, 3) == 0                       # unsupported head_dim
    assert B.cache_bytes(0, 4, 64, 60, 3, 6, 3) == 0
    with pytest.raises(B.LongLiveError) as e:
        B.Cache(1, 4, 96, 6, 10, 3, 3, 6, device=None)
    assert e.value.status == 4
    h = C.c_void_p()
    assert L.ll_cache_create(1, 4, 64, 61, 3, 6, 3, 6, 10, 10000.0, None, 0, C.byref(h)) == 1   # P != grid
    assert L.ll_cache_create(1, 4, 64, 60, 3, 6, 3, 6, 10, 10000.0, None, 16, C.byref(h)) == 1  # null buffer with size
    assert L.ll_cache_create(1, 4, 64, 60, 3, 6, 3, 6, 10, 10000.0, None, 0, None) == 1
    assert b"out is null" in L.ll_last_error()
    c = B.Cache(2, 4, 64, 6, 10, 3, 3, 6, device=None)
    for bad in (lambda: c.chunk_append(2, 0, 3), lambda: c.chunk_append(-1, 0, 3), lambda: c.chunk_append(0, 0, 4),
                lambda: c.chunk_append(0, 0, 0)):
        with pytest.raises(B.LongLiveError) as e:
            bad()
        assert e.value.status == 1
    with pytest.raises(B.LongLiveError) as e:
        c.chunk_append(0, 3, 3)                                            # must start at 0
    assert e.value.status == 2
    with pytest.raises(B.LongLiveError) as e:
        c.live_ranges(5)
    assert e.value.status == 1
    c.chunk_append(0, 0, 3)
    c.chunk_append(0, 0, 3)
    c.chunk_append(0, 3, 3)
    with pytest.raises(B.LongLiveError) as e:
        c.chunk_append(0, 9, 3)                                            # skipped a chunk
    assert e.value.status == 2
    with pytest.raises(B.LongLiveError) as e:
        c.chunk_append(0, 0, 3)                                            # went back
    assert e.value.status == 2
    assert c.live_frames(1) == []                                          # layers are independent
    with pytest.raises(B.LongLiveError) as e:
        c.recache_prefill(1, False, 3, 3)                                  # sink not held
    assert e.value.status == 2
    with pytest.raises(B.LongLiveError) as e:
        c.recache_prefill(0, True, 2, 3)                                   # window overlaps sink
    assert e.value.status == 1
    with pytest.raises(B.LongLiveError) as e:
        c.recache_prefill(0, True, 3, 10)                                  # more than the ring holds
    assert e.value.status == 1
    with pytest.raises(B.LongLiveError) as e:                              # compute needs a device cache
        B._check(L.ll_sink_window_attn(c._h, 0, None, None, None))
    assert e.value.status == 1
    with pytest.raises(B.LongLiveError) as e:                              # and so does the form that turns the queries
        B._check(L.ll_sink_window_attn_unrotated(c._h, 0, None, None, None))
    assert e.value.status == 1
    buf, n = (C.c_int64 * 2)(), C.c_int()
    assert L.ll_cache_live_frames(c._h, 0, buf, 2, C.byref(n)) == 3 and n.value == 6
    c.reset(0)
    c.chunk_append(0, 0, 3)
    assert L.ll_status_string(2) == b"LL_ERR_STATE"
    # ll_cache_read_frame: nothing to write to is an error of the arguments, whatever the handle (a keys-only copy
    # with no key tensor would otherwise store through a null pointer); a misaligned tensor likewise
    assert L.ll_cache_read_frame(c._h, 0, 0, None, None, None) == B.LL_ERR_INVALID_ARG
    assert b"both null" in L.ll_last_error()
    assert L.ll_cache_read_frame(c._h, 0, 0, C.c_void_p(0x1008), None, None) == B.LL_ERR_INVALID_ARG
    assert b"aligned" in L.ll_last_error()
    # a re-prefill of the sink alone: the next chunk can only follow the sink, so any other win_start is refused
    with pytest.raises(B.LongLiveError) as e:
        c.recache_prefill(0, True, 9, 0)
    assert e.value.status == B.LL_ERR_INVALID_ARG
    before = c.live_frames(0)
    c.recache_prefill(0, True, 3, 0)
    assert c.live_frames(0) == [0, 1, 2]
    c.chunk_append(0, 3, 3)
    assert c.live_frames(0) == [0, 1, 2, 3, 4, 5] and before == [0, 1, 2]
    # a refused re-prefill leaves the layer as it was
    with pytest.raises(B.LongLiveError):
        c.recache_prefill(0, True, 3, 10)
    assert c.live_frames(0) == [0, 1, 2, 3, 4, 5]
    c.close()


def test_library_exports_every_declared_symbol():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        hdr = open(os.path.join(ROOT, "include", h)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        found = set(re.findall(r"\b(ll_[a-z_0-9]+)\s*\(", hdr))
        if h == "longlive.h":      # the method's header carries no instruments
            assert {"ll_cache_create", "ll_chunk_append", "ll_sink_window_attn", "ll_recache_prefill"} <= found
            assert not any("probe" in n or "variant" in n for n in found)
        names |= found
    L = B.lib()
    for name in sorted(names):
        assert hasattr(L, name), name
    assert names == set(B.SIGNATURES)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host C compiler")
def test_header_and_library_from_plain_c(tmp_path):
    """include/longlive.h compiles as pedantic C99, links against the built library with C linkage, and the
    index-only handle works from C (tests/c_abi_check.c)."""
    here = os.path.dirname(os.path.abspath(__file__))
    libdir = os.path.dirname(B.LIB_PATH)
    exe = tmp_path / "c_abi_check"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-o", str(exe), os.path.join(here, "c_abi_check.c"),
                    "-L", libdir, "-l:" + os.path.basename(B.LIB_PATH), "-Wl,-rpath," + libdir], check=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0 and "c abi ok" in run.stdout, f"exit {run.returncode}: {run.stdout}{run.stderr}"


def test_fp8_and_sink_relative_handles_share_the_bookkeeping():
    """Index-only handles of the 8-bit cache and of the sink-relative mode keep exactly the plain handle's books
    (the variants change what is stored or how scores are taken, never which frames are live or where they sit)."""
    rng = random.Random(77)
    for _ in range(10):
        S, W, Cc = rng.randint(0, 4), rng.randint(0, 7), rng.randint(1, 4)
        gh, gw = rng.randint(2, 6), rng.randint(2, 9)
        make = lambda **kw: B.Cache(1, 2, 64, gh, gw, Cc, S, W, device=None, **kw)
        a, b, c = make(), make(kv_format="fp8_e4m3", k_exp=1, v_exp=-2), make()
        c.set_sink_relative(True)
        f0 = 0
        for i in range(12):
            n = rng.randint(1, Cc)
            for h in (a, b, c):
                h.chunk_append(0, f0, n)
            assert a.live_frames(0) == b.live_frames(0) == c.live_frames(0)
            assert a.live_ranges(0) == b.live_ranges(0) == c.live_ranges(0)
            if rng.random() < 0.3:                                  # a re-pass of the same chunk
                for h in (a, b, c):
                    h.chunk_append(0, f0, n)
            f0 += n
        assert B.cache_bytes(1, 2, 64, gh * gw, S, W, Cc, "fp8_e4m3") < B.cache_bytes(1, 2, 64, gh * gw, S, W, Cc) + (S + W + Cc) * gh * gw * 2 * 64 + 1
        for h in (a, b, c):
            h.close()
    with pytest.raises(B.LongLiveError) as e:
        B.Cache(1, 2, 64, 2, 2, 1, 1, 1, device=None, kv_format="fp8_e4m3", k_exp=17)
    assert e.value.status == B.LL_ERR_INVALID_ARG
    h8 = B.Cache(1, 2, 64, 2, 2, 1, 1, 1, device=None, kv_format="fp8_e4m3")
    with pytest.raises(B.LongLiveError) as e:
        h8.set_sink_relative(True)
    assert e.value.status == B.LL_ERR_UNSUPPORTED
    h8.close()


def test_prompt_handle_bookkeeping_and_errors():
    """The prompt side's host logic on an index-only handle: sizes, argument checks, call order."""
    L = B.lib()
    assert L.ll_prompt_bytes(30, 12, 128, 512) >= 30 * 12 * 2 * 512 * 128 * 2
    for bad in ((0, 12, 128, 512), (1, 0, 128, 512), (1, 12, 96, 512), (1, 12, 128, 0), (1, 12, 128, 65537)):
        assert L.ll_prompt_bytes(*bad) == 0, bad
    with pytest.raises(B.LongLiveError) as e:
        B.Prompt(1, 12, 96, 512, device=None)
    assert e.value.status == 4
    h = C.c_void_p()
    assert L.ll_prompt_create(1, 2, 64, 77, None, 16, C.byref(h)) == 1          # null buffer with a size
    assert L.ll_prompt_create(1, 2, 64, 77, None, 0, None) == 1
    p = B.Prompt(3, 2, 64, 77, device=None)
    assert [p.tokens(l) for l in range(3)] == [0, 0, 0]
    with pytest.raises(B.LongLiveError) as e:
        p.cross_attn(1, None, None, n_q=10)                                     # no prompt yet
    assert e.value.status == 2
    for bad in (lambda: p.recache(3, None, None, 5), lambda: p.recache(-1, None, None, 5),
                lambda: p.recache(0, None, None, 0), lambda: p.recache(0, None, None, 78),
                lambda: p.tokens(3)):
        with pytest.raises(B.LongLiveError) as e:
            bad()
        assert e.value.status == 1
    p.recache(1, None, None, 77)
    p.recache(1, None, None, 40)                                                # the switch: shorter prompt
    assert [p.tokens(l) for l in range(3)] == [0, 40, 0]                        # layers are independent
    p.cross_attn(1, None, None, n_q=4680)
    for n_q in (0, -3, (1 << 24) + 1):
        with pytest.raises(B.LongLiveError) as e:
            p.cross_attn(1, None, None, n_q=n_q)
        assert e.value.status == 1
    with pytest.raises(B.LongLiveError) as e:
        p.cross_attn(0, None, None, n_q=10)
    assert e.value.status == 2
    one = C.c_int(1)                                                            # any non-null pointer: refused before use
    with pytest.raises(B.LongLiveError) as e:
        B._check(L.ll_prompt_recache(p._h, 0, C.cast(C.pointer(one), C.c_void_p), None, 5, None))
    assert e.value.status == 1
    # the call with the output projection keeps the same books and makes the same checks
    p.cross_attn_out(1, n_q=3000)
    with pytest.raises(B.LongLiveError) as e:
        p.cross_attn_out(1, n_q=0)
    assert e.value.status == B.LL_ERR_INVALID_ARG
    with pytest.raises(B.LongLiveError) as e:
        p.cross_attn_out(0, n_q=10)                                             # no prompt in layer 0
    assert e.value.status == B.LL_ERR_STATE
    with pytest.raises(B.LongLiveError) as e:                                   # an index-only handle takes no tensors
        B._check(L.ll_cross_attn_out(p._h, 1, None, 10, C.cast(C.pointer(one), C.c_void_p), None, None, None))
    assert e.value.status == B.LL_ERR_INVALID_ARG
    # the workspace of the hand-over between the two kernels: rows rounded up to 16, all heads, bf16
    assert p.cross_attn_out_workspace_bytes(1) == 16 * p.heads * p.head_dim * 2
    assert p.cross_attn_out_workspace_bytes(4680) == 4688 * p.heads * p.head_dim * 2
    assert p.cross_attn_out_workspace_bytes(0) == 0 and L.ll_cross_attn_out_workspace_bytes(3, 96, 100) == 0
    for heads, head_dim, w, wp in ((0, 128, one, one), (3, 96, one, one), (3, 128, None, one), (3, 128, one, None)):
        ptr = lambda x: C.cast(C.pointer(x), C.c_void_p) if x is not None else None
        assert L.ll_out_proj_pack_weight(heads, head_dim, ptr(w), ptr(wp), None) == B.LL_ERR_INVALID_ARG
    p.close()


def test_clip_handle_bookkeeping_and_errors():
    """The train-time handle's host logic on an index-only handle: sizes, argument checks, call order."""
    L = B.lib()
    assert L.ll_clip_bytes(12, 128, 1560, 3, 9, 21, 3) > 21 * 1560 * 12 * 128 * 2
    for bad in ((0, 128, 60, 3, 6, 9, 3), (4, 96, 60, 3, 6, 9, 3), (4, 64, 0, 3, 6, 9, 3), (4, 64, 60, -1, 6, 9, 3),
                (4, 64, 60, 3, 6, 0, 3), (4, 64, 60, 3, 6, 9, 0)):
        assert L.ll_clip_bytes(*bad) == 0, bad
    with pytest.raises(B.LongLiveError) as e:
        B.Clip(4, 96, 6, 10, 3, 3, 6, 9, device=None)
    assert e.value.status == 4
    h = C.c_void_p()
    assert L.ll_clip_create(4, 64, 61, 3, 6, 9, 3, 6, 10, 10000.0, None, 0, C.byref(h)) == 1     # P != grid
    assert L.ll_clip_create(4, 64, 60, 3, 6, 9, 3, 6, 10, 10000.0, None, 16, C.byref(h)) == 1    # null buffer with a size
    c = B.Clip(4, 64, 6, 10, 3, 3, 6, 9, device=None)
    with pytest.raises(B.LongLiveError) as e:
        c.backward()                                                              # nothing to differentiate yet
    assert e.value.status == 2
    for bad in (lambda: c.forward(9, 6, 10), lambda: c.forward(9, 6, 0), lambda: c.forward(9, 7, 9),
                lambda: c.forward(-1, 0, 3), lambda: c.forward(2, 1, 3),          # context cuts into the sink
                lambda: c.forward(0, 2, 3)):                                      # a context that would hold the sink
        with pytest.raises(B.LongLiveError) as e:
            bad()
        assert e.value.status == 1
    with pytest.raises(B.LongLiveError) as e:
        c.backward()                                                              # a refused forward leaves no state
    assert e.value.status == 2
    c.forward(9, 6, 9)
    c.backward()
    c.forward(0, 0, 7)                                                            # a video's first clip
    c.backward()
    c.forward(3, 0, 4)                                                            # right after the sink, no context
    c.backward()
    c.close()


@pytest.mark.parametrize("seed", range(6))
def test_clip_key_sets_match_oracle(seed):
    """The train-time handle's key ranges (host logic, index-only) against the oracle's key-set rule over the list
    of resident frames, for random geometries, first clips and later ones."""
    from oracle.clip_backward import ClipOracle
    from oracle.longlive_oracle import OracleConfig, key_frames
    rng = np.random.Generator(np.random.Philox(key=700 + seed))
    for trial in range(30):
        gh, gw = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        Cc, S, W, T = int(rng.integers(1, 5)), int(rng.integers(0, 5)), int(rng.integers(0, 9)), int(rng.integers(1, 12))
        n_clip = int(rng.integers(1, T + 1))
        if trial % 3 == 0:
            ctx_start, n_ctx = 0, 0
        else:
            n_ctx, ctx_start = int(rng.integers(0, W + 1)), S + int(rng.integers(0, 30))
        cfg = OracleConfig(1, 1, 64, gh, gw, Cc, S, W)
        P = gh * gw
        o = ClipOracle(cfg)
        frames = o.frames(ctx_start, n_ctx, n_clip)
        pos = {f: i for i, f in enumerate(frames)}
        clip = B.Clip(1, 64, gh, gw, Cc, S, W, T, device=None)
        clip.forward(ctx_start, n_ctx, n_clip)
        clip_start = ctx_start + n_ctx
        for ci, (f0, n) in enumerate(o.clip_chunks(clip_start, n_clip)):
            want = set()
            for f in key_frames(cfg, f0, n, [g for g in frames if g < f0 + n]):
                want |= set(range(pos[f] * P, (pos[f] + 1) * P))
            ranges = clip.chunk_key_ranges(ci)
            assert 1 <= len(ranges) <= 2 and all(a < b for a, b in ranges)
            assert all(ranges[i][1] < ranges[i + 1][0] for i in range(len(ranges) - 1))      # disjoint, not touching
            got = set()
            for a, b in ranges:
                got |= set(range(a, b))
            assert got == want, (gh, gw, Cc, S, W, T, ctx_start, n_ctx, n_clip, ci)
        with pytest.raises(B.LongLiveError):
            clip.chunk_key_ranges(len(o.clip_chunks(clip_start, n_clip)))
        clip.close()


HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ROCM_CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(ROCM_CLANG)), reason="no ROCm toolchain")
def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    """The library's host code (every api*.cpp and the cache index) built with AddressSanitizer and
    UndefinedBehaviorSanitizer on the host pass only, the kernel launchers replaced by stand-ins
    (tests/host_stubs.cpp), driven from C over index-only handles (tests/host_sanitize_driver.c): random streams of
    appends, re-prefills, resets and introspection calls, the prompt and the train-time handles.  Any report of
    either sanitizer ends the driver with a non-zero status."""
    csrc = os.path.join(ROOT, "paper_2509_22622_amd", "csrc")
    here = os.path.join(ROOT, "tests")
    lib = tmp_path / "libll_san.so"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    srcs = [os.path.join(csrc, f) for f in ("api.cpp", "api_prompt.cpp", "api_clip.cpp", "api_diag.cpp", "cache_index.cpp")]
    build = subprocess.run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", *san,
                            "-Wno-unused-command-line-argument", *srcs, os.path.join(here, "host_stubs.cpp"), "-o", str(lib)],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    exe = tmp_path / "host_walk"
    link = subprocess.run([ROCM_CLANG, "-std=c99", "-pedantic", "-Wall", "-Werror", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-o", str(exe), os.path.join(here, "host_sanitize_driver.c"),
                           "-L", str(tmp_path), "-l:libll_san.so", "-Wl,-rpath," + str(tmp_path)], capture_output=True, text=True)
    assert link.returncode == 0, link.stderr[-3000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1"})
    assert run.returncode == 0 and "host walk ok" in run.stdout, f"exit {run.returncode}\n{run.stdout[-2000:]}\n{run.stderr[-4000:]}"
