"""Shared plumbing of the GPU parity tests: run a workload through the HIP
library, run (a head subset of) it through the CPU oracle, compare."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(got: np.ndarray, ref: np.ndarray):
    """Max relative error of a tensor: |g - o| / max(|o|, rms(o)) maximised over
    elements (the floor keeps zero crossings of y from dividing by zero), and
    the normwise ratio max|g - o| / max|o|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    floor = rms if rms > 0 else 1.0
    diff = np.abs(got - ref)
    elem = float(np.max(diff / np.maximum(np.abs(ref), floor)))
    mx = float(np.max(np.abs(ref)))
    return elem, float(np.max(diff) / (mx if mx > 0 else 1.0))


def assert_close(got, ref, tol, what=""):
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite values"
    e, nrm = rel_err(got, ref)
    assert e <= tol and nrm <= tol, f"{what}: max rel err {e:.3e} (normwise {nrm:.3e}) > {tol:g}"
    return e


def head_groups(H: int, G: int, heads: Sequence[int]) -> List[int]:
    return [h // (H // G) for h in heads]


def oracle_on_heads(wl, heads: Optional[Sequence[int]], init_states, inputs=None, cu=None,
                    ckpt_pos=None, want_y=True):
    """Run the oracle on a head subset.  Heads are independent given their
    group's B and C, so the subset is handed over as a problem of its own with
    one group per selected head."""
    from oracle import ssm_prefill_oracle

    s = wl.shape
    inp = inputs if inputs is not None else wl.inputs
    cu = wl.cu_seqlens if cu is None else cu
    ckpt_pos = wl.ckpt_pos if ckpt_pos is None else ckpt_pos
    if heads is None:
        heads = list(range(s.nheads))
    hs = torch.as_tensor(list(heads), device=inp.x.device)
    gs = torch.as_tensor(head_groups(s.nheads, s.ngroups, heads), device=inp.x.device)
    x = inp.x.index_select(1, hs).float().cpu().numpy()
    dt = inp.dt.index_select(1, hs).float().cpu().numpy()
    B = inp.B.index_select(1, gs).float().cpu().numpy()
    C = inp.C.index_select(1, gs).float().cpu().numpy()
    A = wl.A.index_select(0, hs).cpu().numpy()
    D = wl.D.index_select(0, hs).cpu().numpy()
    inits = None
    if init_states is not None:
        inits = []
        for st in init_states:
            if st is None:
                inits.append(None)
            else:
                st = st if isinstance(st, np.ndarray) else st.detach().cpu().numpy()
                inits.append(np.asarray(st)[list(heads)])
    return ssm_prefill_oracle(x, dt, A, B, C, D, cu, inits, ckpt_pos, want_y=want_y)


def gpu_run(wl, init_states, inputs=None, cu=None, ckpt_pos=None, chunk=None, state_dtype="f32"):
    """Run the HIP library on a workload whose tensors live on the GPU.  With a reduced `state_dtype` the initial
    states must already be tensors of that type, and the checkpoints come back in it."""
    import paper_2411_19379_amd as ssm

    s = wl.shape
    inp = inputs if inputs is not None else wl.inputs
    cu = wl.cu_seqlens if cu is None else cu
    ckpt_pos = wl.ckpt_pos if ckpt_pos is None else ckpt_pos
    plan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, chunk or s.chunk, s.io_dtype, cu, ckpt_pos,
                    state_dtype=state_dtype)
    y, st = ssm.prefill(plan, inp.x, inp.dt, wl.A, inp.B, inp.C, wl.D, init_states)
    torch.cuda.synchronize()
    info = plan.info
    plan.close()
    return y, st, info
