"""GPU parity over seeded random batches that land on every branch of the planner: sequences cut into stretches and
left whole, the 32- and the 64-channel scan, chains of carried states, decay rates down to a fiftieth of the usual
ones (where the carried state reaches far into the next stretch), checkpoints at random positions, cached initial
states.  Every head of every case is compared with the oracle."""
import numpy as np
import pytest
import torch

from helpers import gpu_run, rel_err
from test_gpu_configs import oracle_on_heads
from test_gpu_parity import say
from workloads import LayerShape, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_batches_match_the_oracle(seed):
    import paper_2411_19379_amd as ssm

    rs = np.random.RandomState(seed)
    cut = 0
    for it in range(8):
        H = int(rs.choice([2, 4, 8, 16]))
        P = int(rs.choice([64, 128]))
        G = int(rs.choice([g for g in (1, 2, 4) if H % g == 0]))
        chunk = int(rs.choice([64, 128, 256]))
        batch = int(rs.randint(1, 4))
        hi = int(rs.choice([3000, 12000, 20000]))
        lo = int(rs.choice([1, 5000])) if hi > 5000 else 1
        shape = LayerShape(H, P, 128, G, chunk, "bf16")
        wl = make_workload(2, DEV, seed=1000 * seed + it, batch=batch, len_range=(lo, hi), shape=shape)
        for b, L in enumerate(wl.seqlens):  # up to two more checkpoints per request, anywhere
            extra = [int(v) for v in rs.randint(1, L + 1, size=rs.randint(0, 3))] if L > 0 else []
            wl.ckpt_pos[b] = sorted(set(wl.ckpt_pos[b]) | set(extra))
        wl.A = wl.A * float(rs.choice([1.0, 1.0, 0.1, 0.02]))
        plan = ssm.Plan(H, P, 128, G, chunk, "bf16", wl.cu_seqlens, wl.ckpt_pos)
        stretches = plan.stretches()
        plan.close()
        cut += len(stretches) > batch
        init_np = [None if s is None else s.cpu().numpy() for s in wl.init_state]
        y, st, info = gpu_run(wl, wl.init_state)
        y_ref, st_ref = oracle_on_heads(wl, list(range(H)), init_np)
        e_y = max(rel_err(y.float().cpu().numpy(), y_ref))
        e_s = max([max(rel_err(st[k].cpu().numpy(), st_ref[k])) for k in range(st_ref.shape[0])] or [0.0])
        say(f"    seed {seed}.{it}: H={H} P={P} G={G} requests {wl.seqlens} in stretches of "
            f"{[e - b for b, e, _ in stretches]} tiles, {info.n_workgroups} workgroups: err_y={e_y:.2e} err_state={e_s:.2e}")
        assert torch.isfinite(y.float()).all() and e_y <= 2e-2 and e_s <= 2e-2
    assert cut >= 2, "the seeds are meant to include cut sequences"
