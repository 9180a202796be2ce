"""GPU parity with cached states kept in fp16 or bf16 (a cache that stores its entries in half the bytes), and at
d_state = 16 (the state width of the first-generation selective SSM layers), which the vector-ALU kernel serves.

The oracle starts from the initial states as the cache holds them (rounded to the storage type), so what is compared
is the scan itself plus one rounding of each checkpoint to the storage type."""
import numpy as np
import pytest
import torch

from helpers import assert_close, gpu_run
from test_gpu_configs import compare_all_heads
from test_gpu_parity import say
from workloads import LayerShape, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda"
TORCH_ST = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
# one rounding to the storage type: 2^-11 (fp16) or 2^-8 (bf16) relative, on top of the scan's own error
STATE_TOL = {"f32": 2e-2, "f16": 2e-2, "bf16": 2.5e-2}

SHAPES = {
    # the matrix-core kernel: the 7B layer's head shape on 8 heads in 2 groups
    "mfma_p64_n128": (LayerShape(8, 64, 128, 2, 256, "bf16"), 1),
    # d_state = 16: served by the fp32 vector-ALU kernel, bf16 storage
    "valu_p64_n16": (LayerShape(32, 64, 16, 1, 256, "bf16"), 0),
}


def _as_cache(wl, state_dtype):
    """The workload's random initial states as a cache of `state_dtype` holds them: the tensors to pass to the
    library, and their values in fp32 for the oracle."""
    dev, ref = [], []
    for s in wl.init_state:
        if s is None:
            dev.append(None)
            ref.append(None)
        else:
            r = s.to(TORCH_ST[state_dtype]).contiguous()
            dev.append(r)
            ref.append(r.float().cpu().numpy())
    return dev, ref


@pytest.mark.parametrize("state_dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("case", sorted(SHAPES))
def test_scan_with_cached_states_in_reduced_precision(case, state_dtype):
    shape, path = SHAPES[case]
    say(f"{case}: states in {state_dtype}; 4 requests, half of them cache hits, mid-tile checkpoints")
    wl = make_workload(2, DEV, seed=23, batch=4, len_range=(70, 900), shape=shape)
    init_dev, init_ref = _as_cache(wl, state_dtype)
    y, st, info = gpu_run(wl, init_dev, state_dtype=state_dtype)
    assert info.path == path and st.dtype == TORCH_ST[state_dtype]
    compare_all_heads(wl, y, st.float(), init_ref, tol=STATE_TOL[state_dtype], block=shape.nheads)


@pytest.mark.parametrize("state_dtype", ["f16", "bf16"])
def test_reduced_precision_checkpoint_is_a_valid_initial_state(state_dtype):
    """A checkpoint slot in the storage type goes back in unchanged as the next call's initial state: prefix then
    suffix equals the oracle on the suffix started from that very (rounded) checkpoint."""
    shape, _ = SHAPES["mfma_p64_n128"]
    say(f"round trip of a {state_dtype} checkpoint")
    wl = make_workload(1, DEV, seed=5, seqlen=700, prefix_len=333, shape=shape)
    cu_p = np.array([0, wl.prefix_len], dtype=np.int32)
    _, st_p, _ = gpu_run(wl, None, inputs=wl.prefix, cu=cu_p, ckpt_pos=[[wl.prefix_len]], state_dtype=state_dtype)
    assert st_p.dtype == TORCH_ST[state_dtype]
    init = st_p[0].contiguous()
    y, st, _ = gpu_run(wl, [init], state_dtype=state_dtype)
    compare_all_heads(wl, y, st.float(), [init.float().cpu().numpy()], tol=STATE_TOL[state_dtype], block=shape.nheads)
    # and the fp32 run from the same values agrees with it to the storage rounding
    y32, st32, _ = gpu_run(wl, [init.float().contiguous()])
    assert_close(st.float().cpu().numpy(), st32.cpu().numpy(), 2.0 ** -8 if state_dtype == "bf16" else 2.0 ** -10,
                 "checkpoint against the fp32-state run")
    assert torch.equal(y, y32), "y must not depend on the storage type of the checkpoints"
