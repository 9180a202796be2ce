"""Pins for the CPU oracle: everything here checks `oracle.ssm_prefill_oracle`
against something other than itself (unrolled sums, library matmuls, closed
forms, the prefix-cache invariant).  No GPU needed."""
import math
import os

import numpy as np
import pytest

from oracle import ssm_prefill_oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def draw(T, H, P, N, G, seed, dt_lo=1e-3, dt_hi=1e-1):
    r = np.random.RandomState(seed)
    x = r.randn(T, H, P).astype(np.float32)
    dt = np.exp(r.uniform(math.log(dt_lo), math.log(dt_hi), size=(T, H))).astype(np.float32)
    A = (-np.exp(r.uniform(0.0, math.log(16.0), size=H))).astype(np.float32)
    B = (r.randn(T, G, N) / math.sqrt(N)).astype(np.float32)
    C = (r.randn(T, G, N) / math.sqrt(N)).astype(np.float32)
    D = r.randn(H).astype(np.float32)
    return x, dt, A, B, C, D


def unrolled(x, dt, A, B, C, D, S0, t_eval):
    """Closed form of the recurrence by plain nested loops:
    S_t = e^{A sum_{k<=t} dt_k} S_0 + sum_{j<=t} e^{A sum_{k=j+1..t} dt_k} dt_j x_j B_j^T,
    y_t = C_t . S_t + D x_t.  Every sum is started afresh for each t."""
    T, H, P = x.shape
    G, N = B.shape[1], B.shape[2]
    t = t_eval  # 1-based token count
    S = np.zeros((H, P, N))
    y = np.zeros((H, P))
    for h in range(H):
        g = h // (H // G)
        for p in range(P):
            for n in range(N):
                tot = math.exp(float(A[h]) * math.fsum(float(dt[k, h]) for k in range(t))) * S0[h, p, n]
                terms = []
                for j in range(t):
                    dec = math.exp(float(A[h]) * math.fsum(float(dt[k, h]) for k in range(j + 1, t)))
                    terms.append(dec * float(dt[j, h]) * float(x[j, h, p]) * float(B[j, g, n]))
                S[h, p, n] = tot + math.fsum(terms)
            y[h, p] = math.fsum(float(C[t - 1, g, n]) * S[h, p, n] for n in range(N)) \
                + float(D[h]) * float(x[t - 1, h, p])
    return S, y


@pytest.mark.parametrize("G", [1, 2])
def test_unrolled_closed_form(G):
    T, H, P, N = 19, 4, 3, 5
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=11 + G, dt_hi=0.5)
    S0 = np.random.RandomState(5).randn(H, P, N)
    ck = [3, 8, 19]
    y, st = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], [S0], [ck])
    for k, t in enumerate(ck + [1, 12]):
        S_ref, y_ref = unrolled(x, dt, A, B, C, D, S0, t)
        np.testing.assert_allclose(y[t - 1], y_ref, rtol=1e-12, atol=1e-13)
        if k < len(ck):
            np.testing.assert_allclose(st[k], S_ref, rtol=1e-12, atol=1e-13)


def test_unrolled_varlen_batch_and_slots():
    """Three packed sequences (one empty, one without checkpoints): each must
    equal the unrolled sums of its own tokens, and slots follow CSR order."""
    H, P, N, G = 2, 2, 3, 2
    lens = [7, 0, 5, 9]
    T = sum(lens)
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=3, dt_hi=0.3)
    cu = np.concatenate([[0], np.cumsum(lens)])
    r = np.random.RandomState(9)
    inits = [r.randn(H, P, N), None, None, r.randn(H, P, N)]
    ck = [[2, 7], [], [], [1, 4, 9]]
    y, st = ssm_prefill_oracle(x, dt, A, B, C, D, cu, inits, ck)
    assert st.shape == (5, H, P, N)
    slot = 0
    for s, L in enumerate(lens):
        sl = slice(cu[s], cu[s + 1])
        S0 = inits[s] if inits[s] is not None else np.zeros((H, P, N))
        for t in ck[s]:
            S_ref, _ = unrolled(x[sl], dt[sl], A, B[sl], C[sl], D, S0, t)
            np.testing.assert_allclose(st[slot], S_ref, rtol=1e-12, atol=1e-13)
            slot += 1
        if L:
            _, y_ref = unrolled(x[sl], dt[sl], A, B[sl], C[sl], D, S0, L)
            np.testing.assert_allclose(y[cu[s + 1] - 1], y_ref, rtol=1e-12, atol=1e-13)


def test_A_zero_reduces_to_masked_matmul():
    """A = 0: y = tril(C B^T) (dt*x) + D x and S_T = S_0 + sum_j dt_j x_j B_j^T."""
    T, H, P, N, G = 40, 4, 6, 8, 2
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=21)
    A[:] = 0.0
    S0 = np.random.RandomState(2).randn(H, P, N)
    y, st = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], [S0], [[T]])
    xd, dtd, Bd, Cd = (v.astype(np.float64) for v in (x, dt, B, C))
    for h in range(H):
        g = h // (H // G)
        M = np.tril(Cd[:, g] @ Bd[:, g].T)
        u = dtd[:, h:h + 1] * xd[:, h]
        y_ref = M @ u + Cd[:, g] @ S0[h].T + D[h] * xd[:, h]
        np.testing.assert_allclose(y[:, h], y_ref, rtol=1e-11, atol=1e-12)
        S_ref = S0[h] + u.T @ Bd[:, g]
        np.testing.assert_allclose(st[0, h], S_ref, rtol=1e-11, atol=1e-12)


def test_B_zero_cases():
    T, H, P, N, G = 30, 2, 4, 4, 1
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=8)
    B[:] = 0.0
    # no input coupling and no initial state: the skip path alone, exactly
    y, _ = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T])
    np.testing.assert_array_equal(y, D[None, :, None].astype(np.float64) * x.astype(np.float64))
    # with an initial state: y = e^{A cumsum(dt)} (S_0 C) + D x
    S0 = np.random.RandomState(4).randn(H, P, N)
    y, st = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], [S0], [[T]])
    ell = np.cumsum(dt.astype(np.float64), axis=0) * A[None, :].astype(np.float64)
    for h in range(H):
        y_ref = np.exp(ell[:, h:h + 1]) * (C[:, 0].astype(np.float64) @ S0[h].T) \
            + float(D[h]) * x[:, h].astype(np.float64)
        np.testing.assert_allclose(y[:, h], y_ref, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(st[0, h], math.exp(ell[-1, h]) * S0[h], rtol=1e-12)


def test_dt_zero_freezes_state():
    T, H, P, N, G = 12, 2, 3, 4, 1
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=13)
    dt[:] = 0.0
    S0 = np.random.RandomState(1).randn(H, P, N)
    _, st = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], [S0], [[1, 5, T]])
    for k in range(3):
        np.testing.assert_array_equal(st[k], S0)


def test_geometric_series():
    """Constant dt, x = B = C = 1, D = 0: S_t = dt (1 - a^t)/(1 - a), a = e^{dt A};
    y_t = N S_t."""
    T, H, P, N = 50, 1, 2, 3
    dtv, Av = 0.0625, -2.0
    x = np.ones((T, H, P), np.float32)
    dt = np.full((T, H), dtv, np.float32)
    A = np.full(H, Av, np.float32)
    B = np.ones((T, 1, N), np.float32)
    C = np.ones((T, 1, N), np.float32)
    D = np.zeros(H, np.float32)
    y, st = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], None, [[10, T]])
    a = math.exp(dtv * Av)
    for k, t in enumerate([10, T]):
        np.testing.assert_allclose(st[k], dtv * (1 - a ** t) / (1 - a), rtol=1e-12)
    t = np.arange(1, T + 1)
    np.testing.assert_allclose(y[:, 0, 0], N * dtv * (1 - a ** t) / (1 - a), rtol=1e-12)


def test_memoryless_limit():
    """dt*A -> -inf: the state forgets everything, y_t = dt_t (C_t.B_t) x_t + D x_t."""
    T, H, P, N, G = 16, 2, 3, 4, 2
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=17)
    A[:] = -1.0e6
    y, _ = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T])
    for h in range(H):
        cb = np.sum(C[:, h].astype(np.float64) * B[:, h].astype(np.float64), axis=1)
        xh = x[:, h].astype(np.float64)
        y_ref = (dt[:, h].astype(np.float64) * cb)[:, None] * xh + float(D[h]) * xh
        np.testing.assert_allclose(y[:, h], y_ref, rtol=1e-12, atol=1e-300)


def _paper_example():
    with open(os.path.join(GOLDEN, "position_example.txt")) as f:
        row = [ln for ln in f if ln.strip() and not ln.startswith("#")][0].split()
    return tuple(int(v) for v in row)


@pytest.mark.parametrize("split", ["paper_80_20", "cfg0_128_128"])
def test_prefix_cache_invariant(split):
    """Section 4.1, two-pass prefill: scanning prefix||suffix equals scanning
    the suffix from the prefix's state, in y and in every checkpoint."""
    if split == "paper_80_20":
        total, chunk, want, boundary, rest = _paper_example()
        assert boundary == (want // chunk) * chunk and rest == total - want
        T, cut = total, want
        ck = [boundary, want, total]
    else:
        T, cut = 256, 128
        ck = [128, 256]
    H, P, N, G = 4, 16, 16, 1
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=0)
    y_full, st_full = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], None, [ck])
    k_cut = ck.index(cut)
    later = [p - cut for p in ck if p > cut]
    y_res, st_res = ssm_prefill_oracle(x[cut:], dt[cut:], A, B[cut:], C[cut:], D, [0, T - cut],
                                       [st_full[k_cut]], [later])
    np.testing.assert_allclose(y_res, y_full[cut:], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(st_res, st_full[k_cut + 1:], rtol=1e-12, atol=1e-13)


def test_superposition_and_head_permutation():
    T, H, P, N, G = 24, 4, 3, 4, 2
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=31)
    r = np.random.RandomState(6)
    x2 = r.randn(T, H, P).astype(np.float32)
    S1, S2 = r.randn(H, P, N), r.randn(H, P, N)
    # inputs exactly representable so that x + x2 is the exact sum
    x, x2 = np.round(x * 64) / 64, np.round(x2 * 64) / 64
    ya, sa = ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], [S1], [[T]])
    yb, sb = ssm_prefill_oracle(x2, dt, A, B, C, D, [0, T], [S2], [[T]])
    yc, sc = ssm_prefill_oracle((x + x2).astype(np.float32), dt, A, B, C, D, [0, T], [S1 + S2], [[T]])
    np.testing.assert_allclose(yc, ya + yb, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(sc, sa + sb, rtol=1e-11, atol=1e-12)
    # swapping heads inside each group permutes the outputs the same way
    perm = np.array([1, 0, 3, 2])
    yp, sp = ssm_prefill_oracle(x[:, perm], dt[:, perm], A[perm], B, C, D[perm], [0, T], [S1[perm]], [[T]])
    np.testing.assert_array_equal(yp, ya[:, perm])
    np.testing.assert_array_equal(sp, sa[:, perm])


def test_packing_independence_and_off_by_one():
    H, P, N, G = 2, 4, 4, 1
    lens = [13, 21]
    T = sum(lens)
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=41)
    y, st = ssm_prefill_oracle(x, dt, A, B, C, D, [0, 13, 34], None, [[6, 13], [20, 21]])
    y1, st1 = ssm_prefill_oracle(x[13:], dt[13:], A, B[13:], C[13:], D, [0, 21], None, [[20, 21]])
    np.testing.assert_array_equal(y[13:], y1)
    np.testing.assert_array_equal(st[2:], st1)
    # a checkpoint one token off is a different state, far outside any tolerance
    rel = np.abs(st1[0] - st1[1]).max() / np.abs(st1[1]).max()
    assert rel > 1e-2


def test_rejects_bad_checkpoints():
    T, H, P, N, G = 8, 1, 2, 2, 1
    x, dt, A, B, C, D = draw(T, H, P, N, G, seed=1)
    for bad in ([0], [9], [3, 3], [5, 2]):
        with pytest.raises(ValueError):
            ssm_prefill_oracle(x, dt, A, B, C, D, [0, T], None, [bad])
