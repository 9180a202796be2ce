"""Pins of the cache-policy oracle (`oracle/cache_oracle.py`) against what the paper prints and states: the FLOP
efficiencies of Table 1 (appendix), the reuse scenarios of Section 4.1 ("Tradeoffs"), the admission bound of two
states per sequence, LRU as the alpha = 0 limit of Eq. 2, and the eviction rules of Section 4.3."""
import numpy as np
import pytest

from oracle.cache_oracle import CacheOracle, ModelCost, replay

M7B = ModelCost(n_attn=4, n_ssm=24, n_mlp=28, d_model=4096, d_state=128)  # Section 5.1, "Models"
BIG = 10 ** 15


def test_table1_flops_saved_per_byte():
    """Last two rows of Table 1: attention L + 2D (L + 8192 for the 7B model), SSM L (6D/N + 8 + 5/DN) (200 L)."""
    for L in (1, 100, 4096, 100000):
        attn = ModelCost(1, 0, 0, 4096, 128)
        ssm = ModelCost(0, 1, 0, 4096, 128)
        assert attn.flops(L) / (attn.kv_bytes_per_token * L) == pytest.approx(L + 8192, rel=1e-12)
        assert ssm.flops(L) / ssm.ssm_bytes_per_state == pytest.approx(L * (6 * 4096 / 128 + 8 + 5 / (4096 * 128)),
                                                                      rel=1e-12)
        assert ssm.flops(L) / ssm.ssm_bytes_per_state == pytest.approx(200 * L, rel=1e-6)
    # state sizes of Table 1: 4 L D bytes of KVs per attention layer, 2 D N per SSM layer
    assert ModelCost(1, 0, 0, 4096, 128).kv_bytes_per_token == 4 * 4096
    assert ModelCost(0, 1, 0, 4096, 128).ssm_bytes_per_state == 2 * 4096 * 128
    # an SSM state is N/2 = 64 times the KVs of one token (caption of Table 1)
    assert ModelCost(0, 1, 0, 4096, 128).ssm_bytes_per_state == 64 * ModelCost(1, 0, 0, 4096, 128).kv_bytes_per_token


def test_purely_input_prefix_is_reused_from_its_third_occurrence():
    """Section 4.1, "Tradeoffs": the second occurrence identifies the shared prefix and checkpoints it, the third
    one hits it."""
    c = CacheOracle(M7B, BIG, 1.0)
    system = list(range(1000, 1040))
    assert c.begin(system + [1, 2, 3], 1) == (0, None, 0)
    c.finish(system + [1, 2, 3] + [50, 51], 0, 0, None, 100, 1)
    hit, h, ck = c.begin(system + [4, 5, 6], 2)
    assert (hit, h, ck) == (0, None, 40)               # branch point found by speculative insertion
    c.finish(system + [4, 5, 6] + [60], hit, ck, 200, 201, 2)
    assert c.begin(system + [7, 8], 3) == (40, 200, 0)  # third occurrence resumes from the checkpointed state


def test_input_and_output_prefix_is_reused_at_once():
    """Section 4.1: the state after the last decoded token is cached in any case, so the next round of the same
    conversation hits at the full length of the previous round."""
    c = CacheOracle(M7B, BIG, 1.0)
    turn1_in, turn1_out = [1, 2, 3, 4, 5], [6, 7, 8]
    hit, _, ck = c.begin(turn1_in, 1)
    c.finish(turn1_in + turn1_out, hit, ck, None, 10, 1)
    turn2_in = turn1_in + turn1_out + [9, 10]
    assert c.begin(turn2_in, 2) == (8, 10, 0)


def test_a_hit_needs_a_state_and_leaves_the_last_token_to_compute():
    c = CacheOracle(M7B, BIG, 1.0)
    seq = list(range(20))
    c.finish(seq, 0, 0, None, 1, 1)
    # KVs of all 20 tokens are cached, but the only state sits at 20: a 12-token prefix cannot resume from it
    assert c.begin(seq[:12], 2)[0] == 0
    # the same 20 tokens again: the state at 20 is not usable either, the last token must still be computed
    assert c.begin(seq, 3)[0] == 0
    # one token more and it is
    assert c.begin(seq + [99], 4)[:2] == (20, 1)


def test_at_most_two_states_per_sequence_and_exact_accounting():
    rs = np.random.RandomState(0)
    c = CacheOracle(M7B, BIG, 1.0)
    trace = []
    shared = [list(rs.randint(0, 50, size=30)) for _ in range(3)]
    for _ in range(40):
        inp = shared[rs.randint(3)][: rs.randint(5, 31)] + list(rs.randint(0, 50, size=rs.randint(1, 10)))
        trace.append((inp, list(rs.randint(0, 50, size=rs.randint(1, 6)))))
    before = 0
    for now, (inp, outp) in enumerate(trace, 1):
        hit, _, ck = c.begin(inp, now)
        c.finish(inp + outp, hit, ck, 1000 + now if ck else None, 2000 + now, now)
        assert len(c.states) - before <= 2
        before = len(c.states)
        assert c.used_bytes() == len(c.kv) * M7B.kv_bytes_per_token + len(c.states) * M7B.ssm_bytes_per_state
        # every state sits on a cached path, every path end holds a state
        assert all(q in c.kv for q in c.states)
        assert all(q in c.states for q in c.kv if not c._next_tokens(q))


def test_alpha_zero_is_lru_over_nodes_with_at_most_one_child():
    """Eq. 2 with alpha = 0 falls back to LRU (Section 4.2, "Managing the balance"); nodes with several children are
    not evicted while they have them (Section 4.3, item 1)."""
    kv, st = M7B.kv_bytes_per_token, M7B.ssm_bytes_per_state
    c = CacheOracle(M7B, BIG, 0.0)
    a, b = [1] * 10 + [2] * 5, [1] * 10 + [3] * 5
    c.finish(a, 0, 0, None, 11, 1)
    hit, _, ck = c.begin(b, 2)
    assert ck == 10
    c.finish(b, hit, ck, 21, 22, 2)           # branch node [1]*10 (state 21), leaves a (11) and b (22)
    c.begin([1] * 10 + [9], 3)                # touches the branch node only: its recency is now the best
    c.capacity = c.used_bytes()
    d = [7] * 4
    ev, _ = c.finish(d, 0, 0, None, 31, 4)    # needs 4 tokens + 1 state: the oldest leaf goes (5 tokens + 1 state)
    assert ev == [11]
    # now the branch node has one child: it is a candidate, but the more recent leaf b is older than its touch
    c.capacity = c.used_bytes() - 1
    ev, _ = c.finish([7] * 4, 0, 0, None, 32, 5)   # nothing new is stored (state already there), one eviction needed
    assert ev == [22]


def test_intermediate_eviction_keeps_kvs_and_leaf_eviction_frees_them():
    """Section 4.3, item 1: an evicted intermediate node releases its state and its KVs are absorbed by its child."""
    c = CacheOracle(M7B, BIG, 0.0)
    c.finish([1, 2, 3, 4, 5, 6], 0, 0, None, 1, 5)
    hit, _, ck = c.begin([1, 2, 3], 6)        # input ends in the middle of the edge: checkpoint at 3
    assert (hit, ck) == (0, 3)
    c.finish([1, 2, 3, 4, 5, 6], hit, ck, 2, 3, 1)   # same continuation: state 3 is a duplicate at depth 6
    assert sorted(len(q) for q in c.states) == [3, 6]
    kv_before = len(c.kv)
    c.capacity = c.used_bytes() - 1
    ev, _ = c.finish([1, 2, 3, 4, 5, 6], 0, 0, None, 9, 7)   # over by one byte: lowest recency is the node at 3
    assert ev == [2] and len(c.kv) == kv_before and sorted(len(q) for q in c.states) == [6]
    c.capacity = 0
    ev, _ = c.finish([8], 0, 0, None, 10, 8)                # everything but the request's own state must go
    assert ev == [1] and c.kv == {(8,)}


def test_flop_aware_eviction_prefers_to_keep_long_sequences():
    """Section 4.2: with alpha > 0 a long prefix (many FLOPs saved per byte of its fixed-size state) outlives a
    slightly more recent short one; with alpha = 0 recency alone decides."""
    def run(alpha):
        c = CacheOracle(M7B, BIG, alpha)
        c.finish(list(range(1, 2001)), 0, 0, None, 1, 1)          # long, older
        c.finish(list(range(5000, 5020)), 0, 0, None, 2, 2)       # short, newer
        c.capacity = c.used_bytes()
        ev, _ = c.finish(list(range(9000, 9010)), 0, 0, None, 3, 3)
        return ev
    assert run(0.0)[0] == 1      # LRU evicts the long old one first
    assert run(2.0)[0] == 2      # FLOP-aware evicts the short one


def test_token_hit_rate_of_a_replayed_trace():
    """Section 5.1, "Metrics": tokens that skipped prefill over all input tokens."""
    c = CacheOracle(M7B, BIG, 1.0)
    trace = [([1, 2, 3, 4], [5]), ([1, 2, 3, 4, 5, 6, 7], [8]), ([1, 2, 3, 4, 5, 6, 7, 8, 9], [10])]
    log, rate = replay(c, trace)
    assert [r[0] for r in log] == [0, 5, 8]
    assert rate == pytest.approx(13 / 20)


def test_flop_efficiency_grows_faster_with_more_ssm_layers():
    """Section 4.2, figure on FLOP efficiency of 7B models: FLOPs saved per byte of all states (Eq. 1) grows with
    the sequence length, and the more SSM layers the model has the steeper; for attention-only it is near-constant
    relative to its size (L + 2D plus the MLP share)."""
    models = {"transformer": ModelCost(32, 0, 32, 4096, 128), "hybrid": ModelCost(4, 24, 28, 4096, 128),
              "mamba": ModelCost(0, 64, 0, 4096, 128)}

    def eff(m, L):
        return m.flops(L) / (m.kv_bytes_per_token * L + (m.ssm_bytes_per_state if m.n_ssm else 0))

    slopes = {k: (eff(m, 32768) - eff(m, 1024)) / (32768 - 1024) for k, m in models.items()}
    assert slopes["mamba"] > slopes["hybrid"] > slopes["transformer"] > 0
    # attention-only: L + 2D from the attention layers plus 4D from the MLPs, i.e. it only doubles over 16K tokens,
    # while the SSM-only model's grows in proportion to L
    assert eff(models["transformer"], 16384) / eff(models["transformer"], 1) < 2.1
    assert eff(models["mamba"], 16384) / eff(models["mamba"], 1) == pytest.approx(16384, rel=1e-6)
