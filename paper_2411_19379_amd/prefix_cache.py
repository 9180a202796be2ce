"""ctypes binding of the host-side prefix-cache library (`include/prefix_cache.h`): argument marshalling only.

    cache = PrefixCache(n_attn=4, n_ssm=24, n_mlp=28, d_model=4096, d_state=128, capacity_bytes=..., alpha=1.0)
    look = cache.begin(input_tokens, now)        # look.hit_len, look.hit_handle, look.checkpoint_pos
    ... prefill tokens[look.hit_len:] from state look.hit_handle, checkpoint at look.checkpoint_pos, decode ...
    evicted, rejected = cache.finish(all_tokens, look, branch_handle, final_handle, now)
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libprefix_cache.so")
_lib = None

PC_OK, PC_ERR_INVALID_ARG, PC_ERR_BAD_REQUEST, PC_ERR_BUFFER_TOO_SMALL = 0, -1, -2, -3


class PcConfig(ctypes.Structure):
    _fields_ = [("n_attn_layers", ctypes.c_int32), ("n_ssm_layers", ctypes.c_int32), ("n_mlp_layers", ctypes.c_int32),
                ("d_model", ctypes.c_int32), ("d_state", ctypes.c_int32), ("conv_state_bytes", ctypes.c_int64),
                ("capacity_bytes", ctypes.c_int64), ("alpha", ctypes.c_double)]


class PcLookup(ctypes.Structure):
    _fields_ = [("hit_len", ctypes.c_int32), ("checkpoint_pos", ctypes.c_int32), ("hit_handle", ctypes.c_int64)]


class PcStats(ctypes.Structure):
    _fields_ = [("used_bytes", ctypes.c_int64), ("kv_tokens", ctypes.c_int64), ("n_states", ctypes.c_int64),
                ("n_nodes", ctypes.c_int64)]


class PrefixCacheError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"prefix cache error {code}: {msg}")
        self.code = code


def load_library():
    """Load libprefix_cache.so; fails loudly if it has not been built (python -m paper_2411_19379_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is not built: run `python -m paper_2411_19379_amd.build`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32p, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        lib.pc_create.restype = ctypes.c_int
        lib.pc_create.argtypes = [ctypes.POINTER(PcConfig), ctypes.POINTER(vp)]
        lib.pc_destroy.restype = None
        lib.pc_destroy.argtypes = [vp]
        lib.pc_clone.restype = ctypes.c_int
        lib.pc_clone.argtypes = [vp, ctypes.POINTER(vp)]
        lib.pc_begin.restype = ctypes.c_int
        lib.pc_begin.argtypes = [vp, i32p, ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(PcLookup)]
        lib.pc_abort.restype = ctypes.c_int
        lib.pc_abort.argtypes = [vp, i32p, ctypes.c_int32]
        lib.pc_finish.restype = ctypes.c_int
        lib.pc_finish.argtypes = [vp, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                  ctypes.c_int64, ctypes.c_int64, i32p, i32p]
        lib.pc_released.restype = ctypes.c_int
        lib.pc_released.argtypes = [vp, i64p, ctypes.c_int32]
        lib.pc_stats.restype = ctypes.c_int
        lib.pc_stats.argtypes = [vp, ctypes.POINTER(PcStats)]
        lib.pc_set_alpha.restype = ctypes.c_int
        lib.pc_set_alpha.argtypes = [vp, ctypes.c_double]
        lib.pc_set_capacity.restype = ctypes.c_int
        lib.pc_set_capacity.argtypes = [vp, ctypes.c_int64]
        lib.pc_prefill_flops.restype = ctypes.c_double
        lib.pc_prefill_flops.argtypes = [ctypes.POINTER(PcConfig), ctypes.c_int64]
        lib.pc_node_score.restype = ctypes.c_int
        lib.pc_node_score.argtypes = [vp, i32p, ctypes.c_int32, ctypes.POINTER(ctypes.c_double)]
        lib.pc_last_error.restype = ctypes.c_char_p
        lib.pc_last_error.argtypes = []
        _lib = lib
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise PrefixCacheError(rc, load_library().pc_last_error().decode())
    return rc


def _tokens(tokens: Sequence[int]):
    a = np.ascontiguousarray(tokens, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


class PrefixCache:
    def __init__(self, n_attn: int, n_ssm: int, n_mlp: int, d_model: int, d_state: int, capacity_bytes: int,
                 alpha: float, conv_state_bytes: int = 0, _handle=None):
        self.config = PcConfig(n_attn, n_ssm, n_mlp, d_model, d_state, conv_state_bytes, capacity_bytes, alpha)
        if _handle is None:
            h = ctypes.c_void_p()
            _check(load_library().pc_create(ctypes.byref(self.config), ctypes.byref(h)))
            _handle = h
        self.handle = _handle

    def close(self):
        if getattr(self, "handle", None):
            load_library().pc_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def clone(self) -> "PrefixCache":
        h = ctypes.c_void_p()
        _check(load_library().pc_clone(self.handle, ctypes.byref(h)))
        c = self.config
        return PrefixCache(c.n_attn_layers, c.n_ssm_layers, c.n_mlp_layers, c.d_model, c.d_state, c.capacity_bytes,
                           c.alpha, c.conv_state_bytes, _handle=h)

    def begin(self, tokens: Sequence[int], now: int) -> PcLookup:
        a, p = _tokens(tokens)
        out = PcLookup()
        _check(load_library().pc_begin(self.handle, p, len(a), now, ctypes.byref(out)))
        return out

    def abort(self, tokens: Sequence[int], look: PcLookup) -> None:
        """Give back the pin of a request that will not reach finish()."""
        a, p = _tokens(tokens[: look.hit_len] if look.hit_len else [0])
        _check(load_library().pc_abort(self.handle, p, look.hit_len))

    def finish(self, tokens: Sequence[int], look: PcLookup, branch_handle: Optional[int], final_handle: int,
               now: int) -> Tuple[List[int], List[int]]:
        """Returns (evicted handles in eviction order, rejected handles); the caller frees both."""
        a, p = _tokens(tokens)
        ne, nr = ctypes.c_int32(), ctypes.c_int32()
        lib = load_library()
        _check(lib.pc_finish(self.handle, p, len(a), look.hit_len, look.checkpoint_pos,
                             -1 if branch_handle is None else branch_handle, final_handle, now,
                             ctypes.byref(ne), ctypes.byref(nr)))
        k = ne.value + nr.value
        buf = (ctypes.c_int64 * max(k, 1))()
        got = _check(lib.pc_released(self.handle, buf, k))
        vals = [int(buf[i]) for i in range(got)]
        return vals[: ne.value], vals[ne.value:]

    def stats(self) -> PcStats:
        s = PcStats()
        _check(load_library().pc_stats(self.handle, ctypes.byref(s)))
        return s

    def set_alpha(self, alpha: float) -> None:
        _check(load_library().pc_set_alpha(self.handle, alpha))
        self.config.alpha = alpha

    def set_capacity(self, capacity_bytes: int) -> None:
        _check(load_library().pc_set_capacity(self.handle, capacity_bytes))
        self.config.capacity_bytes = capacity_bytes

    def prefill_flops(self, L: int) -> float:
        return float(load_library().pc_prefill_flops(ctypes.byref(self.config), L))

    def node_score(self, tokens: Sequence[int]) -> float:
        a, p = _tokens(tokens)
        s = ctypes.c_double()
        _check(load_library().pc_node_score(self.handle, p, len(a), ctypes.byref(s)))
        return s.value


def replay(cache: PrefixCache, trace, handles_from: int = 1):
    """Run a trace of (input tokens, output tokens) pairs through the cache; returns the per-request decisions
    (hit_len, checkpoint_pos, evicted, rejected) and the token hit rate (tokens that skipped prefill over all input
    tokens, Section 5.1)."""
    h = handles_from
    log = []
    hit_tokens = in_tokens = 0
    for now, (inp, outp) in enumerate(trace, start=1):
        look = cache.begin(inp, now)
        full = list(inp) + list(outp)
        bh = None
        if look.checkpoint_pos:
            bh, h = h, h + 1
        fh, h = h, h + 1
        ev, rej = cache.finish(full, look, bh, fh, now)
        log.append((look.hit_len, look.checkpoint_pos, tuple(ev), tuple(rej)))
        hit_tokens += look.hit_len
        in_tokens += len(inp)
    return log, (hit_tokens / in_tokens if in_tokens else 0.0)


class AdaptiveCache:
    """A PrefixCache whose alpha is set retrospectively (Section 4.2, "Managing the balance"): alpha stays 0 (LRU)
    until the first eviction; then a snapshot of the tree is taken and the following requests are recorded while
    LRU goes on; once `bootstrap_multiplier` times as many requests as preceded the first eviction have been seen,
    every alpha of the grid replays the recorded requests from the snapshot, and the one with the highest token hit
    rate is adopted (ties: the smallest).  The replays run on clones, one thread each."""

    def __init__(self, cache: PrefixCache, alphas: Sequence[float] = (0.0, 0.25, 0.5, 1.0, 2.0, 4.0),
                 bootstrap_multiplier: int = 5, workers: Optional[int] = None):
        self.cache = cache
        self.cache.set_alpha(0.0)
        self.alphas = tuple(alphas)
        self.multiplier = bootstrap_multiplier
        self.workers = workers
        self.seen = 0
        self.seen_before_first_eviction = None
        self.snapshot: Optional[PrefixCache] = None
        self.window: list = []          # (input tokens, all tokens, now)
        self.tuned = False
        self.rates: dict = {}
        self._inputs: dict = {}

    def begin(self, tokens: Sequence[int], now: int) -> PcLookup:
        look = self.cache.begin(tokens, now)
        self._inputs[id(look)] = list(tokens)
        return look

    def finish(self, tokens: Sequence[int], look: PcLookup, branch_handle: Optional[int], final_handle: int,
               now: int) -> Tuple[List[int], List[int]]:
        inp = self._inputs.pop(id(look), None)
        ev, rej = self.cache.finish(tokens, look, branch_handle, final_handle, now)
        self.seen += 1
        if self.snapshot is not None and not self.tuned and inp is not None:
            self.window.append((inp, list(tokens), now))
            if len(self.window) >= self.multiplier * max(self.seen_before_first_eviction, 1):
                self._tune()
        if ev and self.snapshot is None and not self.tuned:
            self.seen_before_first_eviction = self.seen
            self.snapshot = self.cache.clone()
        return ev, rej

    def _replay_window(self, alpha: float) -> float:
        c = self.snapshot.clone()
        try:
            c.set_alpha(alpha)
            hit = total = 0
            h = 1 << 40  # handles of the replay never reach a real pool
            for inp, full, now in self.window:
                look = c.begin(inp, now)
                bh = None
                if look.checkpoint_pos:
                    bh, h = h, h + 1
                c.finish(full, look, bh, h, now)
                h += 1
                hit += look.hit_len
                total += len(inp)
            return hit / total if total else 0.0
        finally:
            c.close()

    def _tune(self) -> None:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=self.workers or min(len(self.alphas), os.cpu_count() or 1)) as ex:
            rates = list(ex.map(self._replay_window, self.alphas))
        self.rates = dict(zip(self.alphas, rates))
        best = max(rates)
        self.cache.set_alpha(min(a for a, r in self.rates.items() if r == best))
        self.tuned = True
        self.snapshot.close()
        self.snapshot = None
        self.window = []
