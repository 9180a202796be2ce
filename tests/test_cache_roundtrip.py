"""End to end on the CPU: the prefix cache drives a serving loop whose "engine" is the scan oracle.  Every request
resumes from the state the cache names, checkpoints where the cache asks, and must produce the outputs of a prefill
from scratch: the handles, hit lengths and checkpoint positions the cache hands out mean what they say (prefix reuse
is exact, Section 5.1, "Metrics").  Evicted and rejected handles are freed from the pool, and a freed handle is
never named again."""
import numpy as np

from oracle import ssm_prefill_oracle
from paper_2411_19379_amd import prefix_cache as pc
from workloads.traces import make_trace

H, P, N, G, VOCAB = 2, 4, 8, 1, 50


def embed(tokens, table):
    """Per-token inputs of the layer, looked up by token id: equal token prefixes give equal inputs."""
    idx = np.asarray(tokens, dtype=np.int64)
    return table["x"][idx], table["dt"][idx], table["B"][idx], table["C"][idx]


def test_requests_resumed_from_cached_states_equal_prefills_from_scratch():
    rs = np.random.RandomState(0)
    table = dict(x=rs.randn(VOCAB, H, P).astype(np.float32),
                 dt=np.exp(rs.uniform(np.log(1e-3), np.log(1e-1), size=(VOCAB, H))).astype(np.float32),
                 B=(rs.randn(VOCAB, G, N) / np.sqrt(N)).astype(np.float32),
                 C=(rs.randn(VOCAB, G, N) / np.sqrt(N)).astype(np.float32))
    A = -np.exp(rs.uniform(0, np.log(16.0), size=H)).astype(np.float32)
    D = rs.randn(H).astype(np.float32)
    trace = make_trace(3, n_sessions=10, n_prompts=2, prompt_len=(8, 20), turns=(1, 4), user_len=(2, 8),
                       out_len=(1, 6), vocab=VOCAB)
    model = dict(n_attn=1, n_ssm=2, n_mlp=1, d_model=64, d_state=N)
    probe = pc.PrefixCache(capacity_bytes=10 ** 15, alpha=1.0, **model)
    pc.replay(probe, trace)
    cache = pc.PrefixCache(capacity_bytes=int(probe.stats().used_bytes * 0.35), alpha=1.0, **model)

    pool = {}      # handle -> (state [H,P,N] float64, number of tokens it stands for)
    freed = set()
    next_handle = 1
    hits = ckpts = 0
    for now, (inp, outp) in enumerate(trace, 1):
        full = inp + outp
        look = cache.begin(inp, now)
        assert look.hit_len < len(inp)
        init = None
        if look.hit_len:
            assert look.hit_handle in pool and look.hit_handle not in freed
            state, length = pool[look.hit_handle]
            assert length == look.hit_len
            init = [state]
            hits += 1
        # the engine prefills (and "decodes") only what the cache did not cover
        x, dt, B, C = embed(full[look.hit_len:], table)
        positions = []
        if look.checkpoint_pos:
            assert look.hit_len < look.checkpoint_pos <= len(inp)
            positions.append(look.checkpoint_pos - look.hit_len)
            ckpts += 1
        if not positions or positions[-1] != len(full) - look.hit_len:
            positions.append(len(full) - look.hit_len)
        y, states = ssm_prefill_oracle(x, dt, A, B, C, D, [0, len(full) - look.hit_len], init, [positions])
        # the same sequence from scratch
        xf, dtf, Bf, Cf = embed(full, table)
        y_ref, _ = ssm_prefill_oracle(xf, dtf, A, Bf, Cf, D, [0, len(full)], None, [[len(full)]])
        assert np.max(np.abs(y - y_ref[look.hit_len:])) <= 1e-12 * max(1.0, np.max(np.abs(y_ref)))
        # hand the new states to the cache
        branch = None
        if look.checkpoint_pos:
            branch, next_handle = next_handle, next_handle + 1
            pool[branch] = (states[0], look.checkpoint_pos)
        final, next_handle = next_handle, next_handle + 1
        pool[final] = (states[-1], len(full))
        evicted, rejected = cache.finish(full, look, branch, final, now)
        for h in evicted + rejected:
            assert h in pool and h not in freed
            freed.add(h)
            del pool[h]
        assert len(pool) == cache.stats().n_states
    assert hits >= 10 and ckpts >= 1 and len(freed) >= 5
