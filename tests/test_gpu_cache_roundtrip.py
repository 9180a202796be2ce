"""The serving loop of test_cache_roundtrip.py with the HIP library as the engine (Section 4.1: a request resumes
from the deepest cached state, checkpoints the branch point the cache asks for and its own last token): states live
in device memory under the handles the prefix cache names, and every request is compared with the oracle's prefill
of the whole sequence from scratch."""
import numpy as np
import pytest
import torch

from helpers import TOL, rel_err
from oracle import ssm_prefill_oracle
from paper_2411_19379_amd import prefix_cache as pc
from workloads.traces import make_trace

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
H, P, N, G, VOCAB = 4, 64, 128, 2, 200


def test_cache_driven_requests_on_the_gpu_match_prefills_from_scratch():
    import paper_2411_19379_amd as ssm
    g = torch.Generator().manual_seed(0)
    bf = torch.bfloat16
    table = dict(x=torch.randn((VOCAB, H, P), generator=g).to(bf),
                 dt=torch.exp(np.log(1e-3) + (np.log(1e-1) - np.log(1e-3)) * torch.rand((VOCAB, H), generator=g)).to(bf),
                 B=(torch.randn((VOCAB, G, N), generator=g) / N ** 0.5).to(bf),
                 C=(torch.randn((VOCAB, G, N), generator=g) / N ** 0.5).to(bf))
    A = -torch.exp(np.log(16.0) * torch.rand((H,), generator=g))
    D = torch.randn((H,), generator=g)
    dev = {k: v.to(DEV) for k, v in table.items()}
    A_d, D_d = A.to(DEV), D.to(DEV)
    trace = make_trace(3, n_sessions=8, n_prompts=2, prompt_len=(40, 150), turns=(1, 4), user_len=(5, 60),
                       out_len=(1, 40), vocab=VOCAB)
    model = dict(n_attn=1, n_ssm=2, n_mlp=1, d_model=H * P // 2, d_state=N)
    probe = pc.PrefixCache(capacity_bytes=10 ** 15, alpha=1.0, **model)
    pc.replay(probe, trace)
    cache = pc.PrefixCache(capacity_bytes=int(probe.stats().used_bytes * 0.35), alpha=1.0, **model)
    pool = {}
    next_handle = 1
    hits = 0
    for now, (inp, outp) in enumerate(trace, 1):
        full = inp + outp
        look = cache.begin(inp, now)
        idx = torch.as_tensor(full[look.hit_len:], device=DEV)
        x, dt, B, C = (dev[k].index_select(0, idx).contiguous() for k in ("x", "dt", "B", "C"))
        n = len(full) - look.hit_len
        positions = [look.checkpoint_pos - look.hit_len] if look.checkpoint_pos else []
        if not positions or positions[-1] != n:
            positions.append(n)
        plan = ssm.Plan(H, P, N, G, 256, "bf16", [0, n], [positions])
        init = [pool[look.hit_handle]] if look.hit_len else None
        hits += bool(look.hit_len)
        y, states = ssm.prefill(plan, x, dt, A_d, B, C, D_d, init)
        torch.cuda.synchronize()
        plan.close()
        cpu_idx = torch.as_tensor(full)
        y_ref, st_ref = ssm_prefill_oracle(table["x"][cpu_idx], table["dt"][cpu_idx], A, table["B"][cpu_idx],
                                           table["C"][cpu_idx], D, [0, len(full)], None, [[len(full)]])
        assert max(rel_err(y.float().cpu().numpy(), y_ref[look.hit_len:])) <= TOL["bf16"]
        assert max(rel_err(states[-1].cpu().numpy(), st_ref[0])) <= TOL["bf16"]
        branch = None
        if look.checkpoint_pos:
            branch, next_handle = next_handle, next_handle + 1
            pool[branch] = states[0].clone()
        final, next_handle = next_handle, next_handle + 1
        pool[final] = states[-1].clone()
        evicted, rejected = cache.finish(full, look, branch, final, now)
        for h in evicted + rejected:
            del pool[h]
    assert hits >= 5
