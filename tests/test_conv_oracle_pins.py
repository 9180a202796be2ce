"""Pins of the convolution oracle (`oracle/conv_oracle.c`) against things other than itself: a library FIR filter,
torch's SiLU, plain concatenation for the meaning of the cached state, the impulse response, and the prefix-cache
invariant at the paper's (80, 20) split (Section 4.1, two-pass prefill)."""
import numpy as np
import pytest
import torch
from scipy.signal import lfilter

from oracle import conv1d_prefill_oracle


def draw(T, C, K, seed):
    rs = np.random.RandomState(seed)
    x = rs.randn(T, C).astype(np.float32)
    w = (rs.randn(C, K) / np.sqrt(K)).astype(np.float32)
    b = rs.randn(C).astype(np.float32)
    return x, w, b


@pytest.mark.parametrize("K", [1, 2, 4])
def test_matches_library_fir_filter(K):
    """Zero history, identity activation: per channel an FIR filter whose taps are the kernel reversed."""
    x, w, b = draw(50, 5, K, 0)
    out, _ = conv1d_prefill_oracle(x, w, b, [0, 50], silu=False)
    ref = np.stack([lfilter(w[c, ::-1].astype(np.float64), [1.0], x[:, c].astype(np.float64)) + b[c]
                    for c in range(5)], axis=1)
    assert np.max(np.abs(out - ref)) <= 1e-14


def test_silu_is_torch_silu():
    x, w, b = draw(40, 6, 4, 1)
    lin, _ = conv1d_prefill_oracle(x, w, b, [0, 40], silu=False)
    act, _ = conv1d_prefill_oracle(x, w, b, [0, 40], silu=True)
    ref = torch.nn.functional.silu(torch.from_numpy(lin)).numpy()
    assert np.max(np.abs(act - ref)) <= 1e-14


def test_impulse_response_is_the_kernel_and_k1_is_pointwise():
    C, K = 3, 4
    _, w, _ = draw(1, C, K, 2)
    x = np.zeros((8, C), dtype=np.float32)
    x[0] = 1.0
    out, _ = conv1d_prefill_oracle(x, w, None, [0, 8], silu=False)
    for t in range(8):  # token t+1 sees the impulse K-1-t places back
        want = w[:, K - 1 - t] if t < K else np.zeros(C)
        assert np.array_equal(out[t], want.astype(np.float64))
    x1, w1, b1 = draw(9, 4, 1, 3)
    out1, st1 = conv1d_prefill_oracle(x1, w1, b1, [0, 9], None, [[9]], silu=False)
    assert np.array_equal(out1, x1.astype(np.float64) * w1[:, 0].astype(np.float64) + b1.astype(np.float64))
    assert np.array_equal(st1[0][:, 0], x1[8].astype(np.float64))


def test_cached_state_means_the_inputs_that_came_before():
    """Definition by concatenation: with the last K inputs of a history as cached state, the outputs equal those of
    history + sequence run from nothing, and the state taken at p is the last K inputs up to p, oldest first."""
    T, C, K = 30, 4, 4
    x, w, b = draw(T + 10, C, K, 4)
    hist, seq = x[:10], x[10:]
    whole, _ = conv1d_prefill_oracle(x, w, b, [0, T + 10])
    state = np.ascontiguousarray(hist[-K:].T.astype(np.float64))  # [C,K], oldest first
    out, st = conv1d_prefill_oracle(seq, w, b, [0, T], [state], [[1, 2, 3, 17, T]])
    assert np.array_equal(out, whole[10:])
    for k, p in enumerate([1, 2, 3, 17, T]):
        want = x[10 + p - K:10 + p].T.astype(np.float64)  # reaches back into the history for p < K
        assert np.array_equal(st[k], want)
    # without a cached state the history is zeros
    out0, st0 = conv1d_prefill_oracle(seq, w, b, [0, T], None, [[2]])
    pad = np.concatenate([np.zeros((K, C), np.float32), seq])
    ref0, _ = conv1d_prefill_oracle(pad, w, b, [0, T + K])
    assert np.array_equal(out0, ref0[K:])
    assert np.array_equal(st0[0], pad[K + 2 - K:K + 2].T.astype(np.float64))


@pytest.mark.parametrize("split", [(80, 20), (1, 40), (2, 40), (128, 128)])
def test_prefix_cache_invariant(split):
    """scan(prefix + suffix) == scan(suffix, from the state cached after the prefix), outputs and every later state."""
    npre, nsuf = split
    x, w, b = draw(npre + nsuf, 7, 4, 5)
    ck_full = [npre, npre + 1, npre + nsuf // 2, npre + nsuf]
    full, st_full = conv1d_prefill_oracle(x, w, b, [0, npre + nsuf], None, [ck_full])
    suf, st_suf = conv1d_prefill_oracle(x[npre:], w, b, [0, nsuf], [st_full[0]], [[1, nsuf // 2, nsuf]])
    assert np.array_equal(suf, full[npre:])
    assert np.array_equal(st_suf, st_full[1:])


def test_packing_independence_and_off_by_one():
    x, w, b = draw(60, 3, 4, 6)
    cu = [0, 25, 25, 60]
    st_a = np.random.RandomState(7).randn(3, 4)
    out, st = conv1d_prefill_oracle(x, w, b, cu, [st_a, None, None], [[25], [], [10, 35]])
    solo0, s0 = conv1d_prefill_oracle(x[:25], w, b, [0, 25], [st_a], [[25]])
    solo2, s2 = conv1d_prefill_oracle(x[25:], w, b, [0, 35], None, [[10, 35]])
    assert np.array_equal(out[:25], solo0) and np.array_equal(out[25:], solo2)
    assert np.array_equal(st[0], s0[0]) and np.array_equal(st[1:], s2)
    # a state one token off is a different state
    _, near = conv1d_prefill_oracle(x[25:], w, b, [0, 35], None, [[9, 10, 11]])
    assert not np.array_equal(near[0], near[1]) and not np.array_equal(near[1], near[2])


@pytest.mark.parametrize("bad", [[[0]], [[61]], [[5, 5]], [[7, 3]]])
def test_bad_checkpoints_are_rejected(bad):
    x, w, b = draw(60, 2, 4, 8)
    with pytest.raises(ValueError):
        conv1d_prefill_oracle(x, w, b, [0, 60], None, bad)
