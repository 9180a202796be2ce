"""The tile algebra of the GPU kernels, restated with numpy/torch on the CPU and
checked against the token-by-token oracle.

This is not the product path (that runs only in the HIP kernels); it checks the
derivation the kernels rely on, with no GPU: per tile of q tokens,

    Gm[i,j] = (C_i.B_j) e^{l_i-l_j} dt_j  (j <= i),   D added on the diagonal
    y_i     = e^{l_i} (S C_i) + sum_j Gm[i,j] x_j
    S'      = e^{l_q} S + sum_j (e^{l_q-l_j} dt_j x_j) B_j^T

with the decay of Gm formed from two per-token factors around the tile's token
31, e^{l_i-l_31} * e^{l_31-l_j} dt_j, while the tile's total decay is above
2^-100 (one exponential of the difference per entry otherwise; the off-diagonal
32x32 block always takes the two factors, which are both <= 1 there), tiles cut
at checkpoint positions, and (in the reduced-precision mode) rounding exactly
where the matrix-core kernels round: the raw scores, the decay-weighted x and
the copy of S used for S.C to fp16, Gm and y to bf16.  In exact arithmetic the
result equals the recurrence; with the roundings it must stay inside the 2e-2
budget of the bf16 mode with margin."""
import math

import numpy as np
import pytest
import torch

from helpers import rel_err
from oracle import ssm_prefill_oracle


def bf16(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy().astype(np.float64)


def tiles_for(length, ckpts, q):
    cuts = sorted(set(ckpts) | {length})
    out, pos = [], 0
    for c in cuts:
        while pos < c:
            n = min(q, c - pos)
            out.append((pos, n))
            pos += n
    return out


def fp16(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16).astype(np.float64)


def exact(a):
    return np.asarray(a, dtype=np.float64)


def tiled_scan(x, dt, A, B, C, D, S0, ckpts, q, rnd, rnd16=None):
    """One sequence, one group. x [T,H,P], dt [T,H], B,C [T,N]. rnd rounds what the kernel keeps in bf16 (Gm, y),
    rnd16 what it keeps in fp16 (raw scores, decay-weighted x, the copy of S)."""
    rnd16 = rnd16 or rnd
    T, H, P = x.shape
    N = B.shape[1]
    y = np.zeros((T, H, P))
    states = {}
    for h in range(H):
        S = S0[h].astype(np.float64).copy()  # [P,N]
        for (t0, n) in tiles_for(T, ckpts, q):
            sl = slice(t0, t0 + n)
            ell = np.cumsum(dt[sl, h] * A[h])
            Bt, Ct, xt, dtt = B[sl], C[sl], x[sl, h], dt[sl, h]
            CB = rnd16(Ct @ Bt.T)
            c = min(31, n - 1)               # the centre token of the two-factor form
            fast = ell[-1] * math.log2(math.e) > -100.0
            Gm = np.zeros((n, n))
            for i in range(n):
                for j in range(i + 1):
                    if fast or (i >= 32 and j < 32):
                        dec = math.exp(ell[i] - ell[c]) * (math.exp(ell[c] - ell[j]) * dtt[j])
                    else:
                        dec = math.exp(ell[i] - ell[j]) * dtt[j]
                    Gm[i, j] = CB[i, j] * dec
                Gm[i, i] += D[h]
            Y = np.exp(ell)[:, None] * (Ct @ rnd16(S).T) + rnd(Gm) @ xt
            y[sl, h] = rnd(Y)
            w = np.exp(ell[-1] - ell) * dtt
            S = math.exp(ell[-1]) * S + rnd16(w[:, None] * xt).T @ Bt
            if t0 + n in ckpts:
                states[(t0 + n, h)] = S.copy()
    return y, states


@pytest.mark.parametrize("mode,q,tol", [("exact", 64, 1e-9), ("exact", 16, 1e-9), ("bf16", 64, 2e-2)])
def test_tile_algebra_matches_recurrence(mode, q, tol):
    rs = np.random.RandomState(3)
    T, H, P, N = 333, 3, 8, 16
    x = rs.randn(T, H, P)
    dt = np.exp(rs.uniform(math.log(1e-3), math.log(1e-1), size=(T, H)))
    A = -np.exp(rs.uniform(0, math.log(16.0), size=H))
    B = rs.randn(T, N) / math.sqrt(N)
    C = rs.randn(T, N) / math.sqrt(N)
    D = rs.randn(H)
    S0 = rs.randn(H, P, N)
    # the oracle's inputs are fp32 (or bf16) values: make every input representable
    f32 = lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)
    x, dt, A, B, C, D = (f32(v) for v in (x, dt, A, B, C, D))
    if mode == "bf16":
        x, dt, B, C = bf16(x), bf16(dt), bf16(B), bf16(C)
    rnd, rnd16 = (bf16, fp16) if mode == "bf16" else (exact, exact)
    ck = [1, 64, 65, 200, 333]
    y, states = tiled_scan(x, dt, A, B, C, D, S0, ck, q, rnd, rnd16)
    y_ref, st_ref = ssm_prefill_oracle(x, dt, A, B[:, None, :], C[:, None, :], D, [0, T], [S0], [ck])
    e_y = max(rel_err(y, y_ref))
    e_s = 0.0
    for k, p in enumerate(ck):
        got = np.stack([states[(p, h)] for h in range(H)])
        e_s = max(e_s, *rel_err(got, st_ref[k]))
    assert e_y <= tol and e_s <= tol, (e_y, e_s)
    if mode == "bf16":
        # the budget is not consumed by the algebra: y sits at its output rounding plus that of Gm, and the states,
        # fed by fp16 operands only, an order of magnitude below the budget
        assert e_y <= 1e-2 and e_s <= 2e-3, (e_y, e_s)


def test_decay_factorisation_is_safe_for_extreme_rates():
    """dt*A of -50 per token: the tile's total decay is far below 2^-100, so the
    two-factor form is not used on the diagonal blocks, every factor the kernels
    form is <= 1 (or the exponential of a non-positive difference), nothing
    overflows and the result is still the recurrence."""
    rs = np.random.RandomState(5)
    T, H, P, N = 70, 1, 4, 8
    x = rs.randn(T, H, P)
    dt = np.full((T, H), 0.5)
    A = np.array([-100.0])
    B = rs.randn(T, N)
    C = rs.randn(T, N)
    D = np.array([0.3])
    S0 = rs.randn(H, P, N)
    x, B, C, D = (np.asarray(v, dtype=np.float32).astype(np.float64) for v in (x, B, C, D))
    y, st = tiled_scan(x, dt, A, B, C, D, S0, [T], 64, exact)
    y_ref, st_ref = ssm_prefill_oracle(x, dt, A, B[:, None, :], C[:, None, :], D, [0, T], [S0], [[T]])
    assert np.all(np.isfinite(y))
    assert max(rel_err(y, y_ref)) <= 1e-9
    assert max(rel_err(st[(T, 0)][None], st_ref[0])) <= 1e-9


def test_two_factor_decay_stays_inside_the_fp32_range():
    """At the edge of the two-factor form (total decay of the tile 2^-99.9) both factors are normal fp32 numbers and
    their product is the decay to fp32 accuracy for every pair j <= i."""
    n = 64
    dt = np.full(n, 0.5, dtype=np.float32)
    A = np.float32(-99.9 / (n * 0.5) / math.log2(math.e))
    ell2 = (np.cumsum(dt * A, dtype=np.float32) * np.float32(math.log2(math.e))).astype(np.float32)
    assert -100.0 < ell2[-1] < -99.0
    ri = np.exp2(ell2 - ell2[31]).astype(np.float32)
    cf = (np.exp2(ell2[31] - ell2) * dt).astype(np.float32)
    tiny = np.finfo(np.float32).tiny
    assert np.all(np.isfinite(ri)) and np.all(np.isfinite(cf)) and ri.min() >= tiny and cf.min() >= tiny
    i, j = np.tril_indices(n)
    want = np.exp2(ell2[i].astype(np.float64) - ell2[j].astype(np.float64)) * dt[j]
    got = ri[i].astype(np.float64) * cf[j].astype(np.float64)
    assert np.max(np.abs(got - want) / want) < 1e-5
