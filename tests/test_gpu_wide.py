"""GPU parity of the variant of the matrix-core scan whose workgroups own 64 channels of a head.  The plan picks it
when more than 128 (sequence, head, 64-channel slice) streams have work, so these batches are small in tokens but
wide in heads; every head is compared with the oracle."""
import numpy as np
import pytest
import torch

from helpers import gpu_run
from test_gpu_configs import compare_all_heads
from test_gpu_parity import say
from workloads import LayerShape, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda"
TORCH_ST = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _with_empty_sequence(wl):
    wl.seqlens.insert(1, 0)
    wl.cu_seqlens = np.concatenate([[0], np.cumsum(wl.seqlens)]).astype(np.int32)
    wl.ckpt_pos.insert(1, [])
    wl.init_kind.insert(1, "zeros")
    wl.init_state.insert(1, None)
    return wl


@pytest.mark.parametrize("case,shape,batch,want_wgs", [
    # 4 sequences x 64 heads x one 64-channel slice = 256 streams: the 64-channel kernel
    ("p64", LayerShape(64, 64, 128, 4, 256, "bf16"), 4, 4 * 64),
    # headdim 128: two 64-channel slices per head
    ("p128", LayerShape(32, 128, 128, 2, 256, "bf16"), 4, 4 * 32 * 2),
    # 255 streams: the 32-channel kernel would need a second round of workgroups, so still the 64-channel one
    ("p64_255", LayerShape(51, 64, 128, 1, 256, "bf16"), 5, 5 * 51),
    # 125 streams: the 32-channel kernel's 250 workgroups fit one round
    ("p64_narrow", LayerShape(25, 64, 128, 1, 256, "bf16"), 5, 5 * 25 * 2),
])
def test_wide_and_narrow_kernels_match_the_oracle(case, shape, batch, want_wgs):
    say(f"{case}: H={shape.nheads} P={shape.headdim}, {batch} requests of 1..400 tokens, half of them cache hits, "
        f"mid-tile checkpoints")
    wl = make_workload(2, DEV, seed=31, batch=batch, len_range=(1, 400), shape=shape)
    init_np = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    y, st, info = gpu_run(wl, wl.init_state)
    assert info.path == 1 and info.n_workgroups == want_wgs
    compare_all_heads(wl, y, st, init_np, block=shape.nheads)


@pytest.mark.parametrize("state_dtype", ["f16", "bf16"])
def test_wide_kernel_with_an_empty_sequence_and_reduced_precision_states(state_dtype):
    shape = LayerShape(64, 64, 128, 8, 64, "bf16")
    say(f"64-channel kernel: states in {state_dtype}, an empty sequence in the batch, chunk 64")
    wl = _with_empty_sequence(make_workload(2, DEV, seed=41, batch=4, len_range=(60, 300), shape=shape))
    dev, ref = [], []
    for s in wl.init_state:
        r = None if s is None else s.to(TORCH_ST[state_dtype]).contiguous()
        dev.append(r)
        ref.append(None if r is None else r.float().cpu().numpy())
    y, st, info = gpu_run(wl, dev, state_dtype=state_dtype)
    assert info.n_workgroups == 5 * 64  # the empty sequence keeps its workgroups; they exit at once
    compare_all_heads(wl, y, st.float(), ref, tol=2.5e-2 if state_dtype == "bf16" else 2e-2, block=64)
