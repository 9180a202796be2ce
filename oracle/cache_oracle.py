"""Oracle of the prefix-cache policy for hybrid models: judicious admission by speculative insertion and
FLOP-aware eviction (Sections 4.1 to 4.3, Eq. 1 and 2, Table 1 of the appendix).

TEST INFRASTRUCTURE ONLY, like the rest of this package.  It shares no code with the C++ radix tree and is written
the slow, obvious way: there is no tree at all.  The cache is two plain collections,

    KV      the set of all token prefixes (tuples) whose last token's KVs are cached
    STATES  prefix -> cached SSM state (handle, last access time)

and everything the paper states in terms of the radix tree is derived from them each time it is needed (an index
from a prefix to its next tokens keeps that affordable).  A prefix q in KV is a *node* of the radix tree exactly
if it holds a state, or is the end of a cached path (no extension of it is in KV), or branches (two or more
different next tokens); its children are counted by the distinct next tokens, and its parent is its longest proper
prefix that is a node (the root is the empty prefix).

Policy, with the passage each step follows:

* Lookup (Section 2.2, Section 3): SSM states cannot be rolled back, so a request can only resume from a prefix
  that holds a state.  The hit is the longest such prefix of the input, at most n - 1 tokens long so that the last
  input token is still computed.  Only the hit node's timestamp is refreshed (Section 4.3, item 2).
* Admission (Section 4.1): before prefill the input is inserted speculatively.  If that would create a new
  intermediate node, i.e. the input leaves the cached paths, or ends, in the middle of an edge, the state at that
  depth is to be checkpointed during prefill.  The state after the last decoded token is cached in any case.  At
  most two states per sequence.
* Eviction (Section 4.2, 4.3 item 1): while the cache is over capacity, among the nodes with at most one child the
  one with the lowest S(n) = recency(n) + alpha * flop_efficiency(n) goes; both terms are min-max normalised over
  the state-holding nodes; flop efficiency is the FLOPs saved relative to the parent over the bytes of the node's
  own KVs and state (Eq. 1, Table 1).  A leaf is removed with its KVs; an intermediate node gives up its state and
  its KVs pass to its child.  The states of the request being inserted are exempt in its own round.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple


@dataclass(frozen=True)
class ModelCost:
    """Layer counts and sizes of Table 1 (FP16: 2 bytes per parameter)."""
    n_attn: int
    n_ssm: int
    n_mlp: int
    d_model: int   # D
    d_state: int   # N
    conv_state_bytes: int = 0  # per SSM layer (Appendix A.1); Table 1 leaves it out

    def flops(self, L: int) -> float:
        """Prefill FLOPs of a sequence of length L over all layers (Table 1, first row)."""
        D, N = float(self.d_model), float(self.d_state)
        Lf = float(L)
        attn = 8.0 * Lf * D * D + 4.0 * Lf * Lf * D
        mlp = 16.0 * Lf * D * D
        ssm = 12.0 * Lf * D * D + 16.0 * Lf * D * N + 10.0 * Lf
        return self.n_attn * attn + self.n_mlp * mlp + self.n_ssm * ssm

    @property
    def kv_bytes_per_token(self) -> int:
        return self.n_attn * 4 * self.d_model

    @property
    def ssm_bytes_per_state(self) -> int:
        return self.n_ssm * (2 * self.d_model * self.d_state + self.conv_state_bytes)


@dataclass
class _State:
    handle: int
    last_access: int
    pins: int = 0


class CacheOracle:
    def __init__(self, model: ModelCost, capacity_bytes: int, alpha: float):
        self.model = model
        self.capacity = int(capacity_bytes)
        self.alpha = float(alpha)
        self.kv = set()                       # prefixes (tuples of ints), never the empty one
        self.nxt: Dict[tuple, set] = {}       # prefix -> the next tokens t with prefix + (t,) in KV (an index of KV)
        self.states: Dict[tuple, _State] = {}

    # ------------------------------------------------------------------ derived structure
    def used_bytes(self) -> int:
        return len(self.kv) * self.model.kv_bytes_per_token + len(self.states) * self.model.ssm_bytes_per_state

    def _kv_add(self, p: tuple) -> None:
        if p not in self.kv:
            self.kv.add(p)
            self.nxt.setdefault(p[:-1], set()).add(p[-1])

    def _kv_discard(self, p: tuple) -> None:
        if p in self.kv:
            self.kv.discard(p)
            self.nxt[p[:-1]].discard(p[-1])

    def _next_tokens(self, q: tuple) -> set:
        return self.nxt.get(q, set())

    def _is_node(self, q: tuple) -> bool:
        if len(q) == 0:
            return True
        if q not in self.kv:
            return False
        return q in self.states or len(self._next_tokens(q)) != 1

    def _parent_depth(self, q: tuple) -> int:
        for d in range(len(q) - 1, 0, -1):
            if self._is_node(q[:d]):
                return d
        return 0

    def nodes(self) -> List[tuple]:
        return sorted(q for q in self.kv if self._is_node(q))

    # ------------------------------------------------------------------ requests
    def begin(self, tokens: Sequence[int], now: int) -> Tuple[int, Optional[int], int]:
        """Returns (hit_len, handle of the state to resume from or None, depth to checkpoint during prefill or 0)."""
        toks = tuple(int(t) for t in tokens)
        n = len(toks)
        hit = 0
        for d in range(1, n):            # at most n - 1
            if toks[:d] in self.states:
                hit = d
        handle = None
        if hit:
            st = self.states[toks[:hit]]
            st.last_access = now
            st.pins += 1
            handle = st.handle
        # speculative insertion: how far do the cached paths follow the input?
        lcp = 0
        while lcp < n and toks[:lcp + 1] in self.kv:
            lcp += 1
        ckpt = 0
        if lcp >= 1 and not self._is_node(toks[:lcp]) and lcp > hit:
            ckpt = lcp                   # the input leaves (or ends in) the middle of an edge
        return hit, handle, ckpt

    def finish(self, tokens: Sequence[int], hit_len: int, branch_pos: int, branch_handle: Optional[int],
               final_handle: int, now: int):
        """Insert the whole sequence (input and output), attach its states, evict.  Returns (evicted handles in
        eviction order, handles not admitted because a state was already cached there)."""
        toks = tuple(int(t) for t in tokens)
        m = len(toks)
        if hit_len:
            self.states[toks[:hit_len]].pins -= 1
        for d in range(1, m + 1):
            self._kv_add(toks[:d])
        rejected = []
        own = []
        for pos, h in ((branch_pos, branch_handle), (m, final_handle)):
            if h is None or pos <= 0:
                continue
            q = toks[:pos]
            if q in self.states:
                self.states[q].last_access = now
                rejected.append(h)
            else:
                self.states[q] = _State(h, now)
            own.append(q)
        evicted = []
        while self.used_bytes() > self.capacity:
            victim = self._pick_victim(exempt=own)
            if victim is None:
                break
            evicted.append(self.states[victim].handle)
            self._evict(victim)
        return evicted, rejected

    # ------------------------------------------------------------------ eviction
    def _flop_efficiency(self, q: tuple) -> float:
        pd = self._parent_depth(q)
        saved = self.model.flops(len(q)) - self.model.flops(pd)
        mem = (len(q) - pd) * self.model.kv_bytes_per_token + self.model.ssm_bytes_per_state
        return saved / float(mem)

    def scores(self) -> Dict[tuple, float]:
        """S(n) of Eq. 2 for every state-holding node."""
        holders = sorted(self.states)
        if not holders:
            return {}
        ts = {q: float(self.states[q].last_access) for q in holders}
        fe = {q: self._flop_efficiency(q) for q in holders}

        def norm(v):
            lo, hi = min(v.values()), max(v.values())
            return {q: ((x - lo) / (hi - lo) if hi > lo else 0.0) for q, x in v.items()}

        r, f = norm(ts), norm(fe)
        return {q: r[q] + self.alpha * f[q] for q in holders}

    def _pick_victim(self, exempt) -> Optional[tuple]:
        s = self.scores()
        best = None
        for q in sorted(s):
            if q in exempt or self.states[q].pins > 0 or len(self._next_tokens(q)) > 1:
                continue
            key = (s[q], self.states[q].last_access, len(q), q)
            if best is None or key < best[0]:
                best = (key, q)
        return None if best is None else best[1]

    def _evict(self, q: tuple) -> None:
        children = self._next_tokens(q)
        del self.states[q]
        if children:
            return                       # intermediate node: its KVs pass to the child
        # leaf: its own KVs go, i.e. the tokens below its parent node
        pd = self._parent_depth(q)
        for d in range(pd + 1, len(q) + 1):
            self._kv_discard(q[:d])


def replay(oracle: CacheOracle, trace, handles_from: int = 1):
    """Run a trace of (input tokens, output tokens) pairs; returns per-request (hit_len, ckpt) and the token hit
    rate (Section 5.1, "Metrics": tokens that skipped prefill over all input tokens)."""
    h = handles_from
    log = []
    hit_tokens = in_tokens = 0
    for now, (inp, outp) in enumerate(trace, start=1):
        hit, _, ck = oracle.begin(inp, now)
        full = list(inp) + list(outp)
        bh = None
        if ck:
            bh, h = h, h + 1
        fh, h = h, h + 1
        ev, rej = oracle.finish(full, hit, ck, bh, fh, now)
        log.append((hit, ck, tuple(ev), tuple(rej)))
        hit_tokens += hit
        in_tokens += len(inp)
    return log, (hit_tokens / in_tokens if in_tokens else 0.0)


def tune_alpha_oracle(model: ModelCost, capacity: int, trace, alphas, multiplier: int):
    """The retrospective choice of alpha (Section 4.2, "Managing the balance") the slow way: run LRU until the first
    eviction, copy the cache, keep running LRU while recording multiplier x (requests before the first eviction)
    requests, then replay that window from the copy under every alpha and keep the best token hit rate (ties: the
    smallest alpha).  Returns (alpha, rates by alpha, index of the request after which it was chosen) or
    (None, {}, None) if the trace ends before."""
    import copy

    live = CacheOracle(model, capacity, 0.0)
    snap = None
    window = []
    first = None
    h = 1
    for idx, (inp, outp) in enumerate(trace):
        now = idx + 1
        hit, _, ck = live.begin(inp, now)
        full = list(inp) + list(outp)
        bh = None
        if ck:
            bh, h = h, h + 1
        fh, h = h, h + 1
        ev, _ = live.finish(full, hit, ck, bh, fh, now)
        if snap is not None:
            window.append((list(inp), full, now))
            if len(window) >= multiplier * max(first, 1):
                rates = {}
                for a in alphas:
                    c = copy.deepcopy(snap)
                    c.alpha = float(a)
                    hits = total = 0
                    hh = 1 << 40
                    for winp, wfull, wnow in window:
                        whit, _, wck = c.begin(winp, wnow)
                        wb = None
                        if wck:
                            wb, hh = hh, hh + 1
                        c.finish(wfull, whit, wck, wb, hh, wnow)
                        hh += 1
                        hits += whit
                        total += len(winp)
                    rates[a] = hits / total if total else 0.0
                best = max(rates.values())
                return min(a for a, r in rates.items() if r == best), rates, idx
        if ev and snap is None:
            first = idx + 1
            snap = copy.deepcopy(live)
    return None, {}, None
