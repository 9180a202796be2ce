"""The tile algebra of the GPU kernels, restated with numpy/torch on the CPU and
checked against the token-by-token oracle.

This is not the product path (that runs only in the HIP kernels); it checks the
derivation the kernels rely on, with no GPU: per tile of q tokens,

    Gm[i,j] = (C_i.B_j) e^{l_i-l_j} dt_j  (j <= i),   D added on the diagonal
    y_i     = e^{l_i} (S C_i) + sum_j Gm[i,j] x_j
    S'      = e^{l_q} S + sum_j (e^{l_q-l_j} dt_j x_j) B_j^T

with the off-diagonal 32x32 block of Gm factorised as e^{l_i-l_31} e^{l_31-l_j},
tiles cut at checkpoint positions, and (in bf16 mode) rounding exactly where the
MFMA kernel rounds: Gm, the decay-weighted x, the copy of S used for S.C, and y.
In exact arithmetic the result equals the recurrence; with the bf16 roundings it
must stay inside the 2e-2 budget of the bf16 mode with margin."""
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


def tiled_scan(x, dt, A, B, C, D, S0, ckpts, q, rnd):
    """One sequence, one group. x [T,H,P], dt [T,H], B,C [T,N]. rnd rounds MFMA operands."""
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
            CB = Ct @ Bt.T
            Gm = np.zeros((n, n))
            for i in range(n):
                for j in range(i + 1):
                    if i >= 32 and j < 32:  # off-diagonal block: two factors, both <= 1
                        dec = math.exp(ell[i] - ell[31]) * (math.exp(ell[31] - ell[j]) * dtt[j])
                    else:
                        dec = math.exp(ell[i] - ell[j]) * dtt[j]
                    Gm[i, j] = CB[i, j] * dec
                Gm[i, i] += D[h]
            Y = np.exp(ell)[:, None] * (Ct @ rnd(S).T) + rnd(Gm) @ xt
            y[sl, h] = rnd(Y)
            w = np.exp(ell[-1] - ell) * dtt
            S = math.exp(ell[-1]) * S + rnd(w[:, None] * xt).T @ Bt
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
    rnd = bf16 if mode == "bf16" else (lambda a: np.asarray(a, dtype=np.float64))
    ck = [1, 64, 65, 200, 333]
    y, states = tiled_scan(x, dt, A, B, C, D, S0, ck, q, rnd)
    y_ref, st_ref = ssm_prefill_oracle(x, dt, A, B[:, None, :], C[:, None, :], D, [0, T], [S0], [ck])
    e_y = max(rel_err(y, y_ref))
    e_s = 0.0
    for k, p in enumerate(ck):
        got = np.stack([states[(p, h)] for h in range(H)])
        e_s = max(e_s, *rel_err(got, st_ref[k]))
    assert e_y <= tol and e_s <= tol, (e_y, e_s)
    if mode == "bf16":
        # the budget is not consumed by the algebra: a clear margin remains
        assert e_y <= 1e-2 and e_s <= 1.5e-2, (e_y, e_s)


def test_decay_factorisation_is_safe_for_extreme_rates():
    """dt*A of -50 per token: every factor the kernels form is <= 1 (or the
    exponential of a non-positive difference), so nothing overflows and the
    result is still the recurrence."""
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
    y, st = tiled_scan(x, dt, A, B, C, D, S0, [T], 64, lambda a: np.asarray(a, dtype=np.float64))
    y_ref, st_ref = ssm_prefill_oracle(x, dt, A, B[:, None, :], C[:, None, :], D, [0, T], [S0], [[T]])
    assert np.all(np.isfinite(y))
    assert max(rel_err(y, y_ref)) <= 1e-9
    assert max(rel_err(st[(T, 0)][None], st_ref[0])) <= 1e-9
