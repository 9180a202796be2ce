"""GPU parity of batches whose long sequences the plan cuts into stretches: the stretches of a sequence are scanned at
the same time, the later ones from a zero state, and two more kernels carry the states over and add what they
contribute.  Batches with few heads, so that a few thousand tokens are enough; every head is compared with the
oracle, which knows nothing of stretches."""
import pytest
import torch

from helpers import gpu_run
from test_gpu_configs import compare_all_heads
from test_gpu_parity import say
from workloads import LayerShape, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda"
TORCH_ST = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _stretches(wl, state_dtype="f32"):
    import paper_2411_19379_amd as ssm

    s = wl.shape
    plan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, s.io_dtype, wl.cu_seqlens, wl.ckpt_pos,
                    state_dtype=state_dtype)
    st = plan.stretches()
    plan.close()
    return st


@pytest.mark.parametrize("case,shape,batch,lens,a_scale", [
    # 16 streams: the shorter request in two stretches, the longer in four (a chain of carried states); cached
    # states, a checkpoint somewhere inside and one at the end of each request
    ("chain", LayerShape(8, 64, 128, 2, 256, "bf16"), 2, (10300, 20000), 1.0),
    # decay a hundred times slower than usual: the carried state reaches every token of the later stretches
    ("slow_decay", LayerShape(8, 64, 128, 2, 256, "bf16"), 2, (14000, 14000), 0.01),
    # the same with 128 heads and one request: two stretches of more than 96 tiles, so that the last workgroup of the
    # second kernel walks on beyond its own tile
    ("slow_decay_long", LayerShape(128, 64, 128, 8, 256, "bf16"), 1, (14000, 14000), 0.01),
    # headdim 128: two 64-channel slices per head
    ("p128", LayerShape(4, 128, 128, 1, 64, "bf16"), 2, (10300, 10300), 1.0),
])
def test_sequences_cut_into_stretches_match_the_oracle(case, shape, batch, lens, a_scale):
    wl = make_workload(2, DEV, seed=53, batch=batch, len_range=lens, shape=shape)
    wl.A = wl.A * a_scale
    st = _stretches(wl)
    say(f"{case}: H={shape.nheads} P={shape.headdim}, requests of {wl.seqlens} tokens in stretches of "
        f"{[e - b for b, e, _ in st]} tiles, decay x{a_scale}")
    assert len(st) > batch and sum(z for _, _, z in st) == len(st) - batch
    init_np = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    y, states, info = gpu_run(wl, wl.init_state)
    assert info.path == 1 and info.n_stretches == len(st)
    compare_all_heads(wl, y, states, init_np, block=min(shape.nheads, 32))


@pytest.mark.parametrize("state_dtype", ["f16", "bf16"])
def test_stretches_with_reduced_precision_states(state_dtype):
    shape = LayerShape(8, 64, 128, 2, 64, "bf16")
    wl = make_workload(2, DEV, seed=59, batch=3, len_range=(4000, 16000), shape=shape)
    st = _stretches(wl, state_dtype)
    say(f"stretches of {[e - b for b, e, _ in st]} tiles, states in {state_dtype}")
    assert any(z for _, _, z in st)
    dev, ref = [], []
    for s in wl.init_state:
        r = None if s is None else s.to(TORCH_ST[state_dtype]).contiguous()
        dev.append(r)
        ref.append(None if r is None else r.float().cpu().numpy())
    y, states, info = gpu_run(wl, dev, state_dtype=state_dtype)
    compare_all_heads(wl, y, states.float(), ref, tol=2.5e-2 if state_dtype == "bf16" else 2e-2, block=8)
