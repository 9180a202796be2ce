"""GPU parity at the full sizes of the five named configurations, in the launch
configuration the benchmark times.  Every head of every configuration is
compared with the token-by-token oracle (heads are independent given their
group's B and C, so the oracle takes them in blocks to bound host memory);
every checkpoint slot is compared in full."""
import numpy as np
import pytest
import torch

from helpers import TOL, assert_close, gpu_run, oracle_on_heads
from test_gpu_parity import prefix_state, say
from workloads import make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda"


def prefix_init(wl):
    """Initial state of a 'prefix' workload: the oracle's state after the random prefix, scanned from zero, on
    every head.  The library's own prefix scan is checked against it on the way."""
    cu = np.array([0, wl.prefix_len], dtype=np.int32)
    _, st_g, _ = gpu_run(wl, None, inputs=wl.prefix, cu=cu, ckpt_pos=[[wl.prefix_len]])
    st_o = prefix_state(wl, None)  # [H, P, N]
    assert_close(st_g[0].cpu().numpy(), st_o, TOL[wl.shape.io_dtype], "prefix state")
    return torch.as_tensor(st_o).to(DEV).contiguous(), st_o


def compare_all_heads(wl, y, st, init_np, tol=2e-2, block=32):
    """y and every checkpoint slot of every head against the oracle, `block` heads at a time."""
    H = wl.shape.nheads
    e_y = e_s = 0.0
    assert torch.isfinite(y.float()).all(), "y holds non-finite values"
    if st is not None:
        assert torch.isfinite(st).all(), "a checkpoint holds non-finite values"
    for h0 in range(0, H, block):
        heads = list(range(h0, min(H, h0 + block)))
        y_ref, st_ref = oracle_on_heads(wl, heads, init_np)
        e_y = max(e_y, assert_close(y[:, heads].float().cpu().numpy(), y_ref, tol, f"y, heads {h0}.."))
        for k in range(st_ref.shape[0]):
            e_s = max(e_s, assert_close(st[k][heads].cpu().numpy(), st_ref[k], tol,
                                        f"checkpoint slot {k}, heads {h0}.."))
        say(f"    heads {heads[0]}..{heads[-1]}: err_y={e_y:.2e} err_state={e_s:.2e}")
    return e_y, e_s


def test_cfg1_2p7b_2k_prefix_hit():
    say("cfg1: H=80 P=64 N=128 G=1, T=2048 after a 1024-token cached prefix, checkpoint at the last token")
    wl = make_workload(1, DEV)
    init, st_o = prefix_init(wl)
    y, st, info = gpu_run(wl, [init])
    assert info.path == 1
    compare_all_heads(wl, y, st, [st_o], block=80)


def test_cfg2_varlen16():
    say("cfg2: 16 requests U{512..8192}, half cache hits, 2 checkpoints each; all 80 heads")
    wl = make_workload(2, DEV)
    init_np = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    y, st, info = gpu_run(wl, wl.init_state)
    assert info.path == 1 and info.n_ckpt == 32
    compare_all_heads(wl, y, st, init_np, block=40)


def test_cfg3_7b_32k_prefix_hit():
    say("cfg3: H=128 P=64 N=128 G=8, T=32768 after a 16384-token cached prefix; all 128 heads")
    wl = make_workload(3, DEV)
    init, st_o = prefix_init(wl)
    y, st, info = gpu_run(wl, [init])
    assert info.path == 1
    compare_all_heads(wl, y, st, [st_o], block=64)


def test_cfg4_128k_fine_grained_checkpoints():
    say("cfg4: T=131072, a 4 MiB fp32 state every 4096 tokens (32 slots); all 128 heads")
    wl = make_workload(4, DEV)
    y, st, info = gpu_run(wl, None)
    assert info.n_ckpt == 32 and tuple(st.shape) == (32, 128, 64, 128)
    compare_all_heads(wl, y, st, None, block=16)


def test_fp32_mode_at_the_2p7b_layer_shape():
    """fp32 mode (tolerance 1e-4) at P=64, N=128: 8192 state elements per head, 32 per thread of the vector-ALU
    kernel.  8 heads in 2 groups, cached initial states, checkpoints inside and at the ends of tiles."""
    from workloads import LayerShape
    say("fp32 mode: H=8 P=64 N=128 G=2, 3 requests, random initial states, mid-tile checkpoints")
    shape = LayerShape(8, 64, 128, 2, 256, "f32")
    wl = make_workload(2, DEV, seed=17, batch=3, len_range=(100, 600), shape=shape)
    init_np = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    y, st, info = gpu_run(wl, wl.init_state)
    assert info.path == 0
    compare_all_heads(wl, y, st, init_np, tol=1e-4, block=8)


def test_fp32_mode_of_cfg1_at_full_size():
    """The 2.7B-shaped 2K-token configuration with fp32 inputs and outputs (fp32 vector-ALU kernel, all 80 heads,
    cached 1024-token prefix): the 1e-4 tolerance of the fp32 mode at a full layer."""
    from workloads import LayerShape
    say("cfg1 in fp32 mode: H=80 P=64 N=128 G=1, T=2048 after a 1024-token cached prefix; all 80 heads")
    wl = make_workload(1, DEV, shape=LayerShape(80, 64, 128, 1, 256, "f32"))
    init, st_o = prefix_init(wl)
    y, st, info = gpu_run(wl, [init])
    assert info.path == 0
    compare_all_heads(wl, y, st, [st_o], tol=1e-4, block=80)
