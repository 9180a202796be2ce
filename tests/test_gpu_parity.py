"""GPU parity: the HIP library against the CPU oracle, element by element, on
the same seeded inputs, through the C ABI (ctypes binding)."""
import numpy as np
import pytest
import torch

from helpers import TOL, assert_close, gpu_run, oracle_on_heads, rel_err
from workloads import LayerShape, make_workload
from workloads.gen import LayerInputs

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def to_dev(states):
    return None if states is None else [None if s is None else
                                        torch.as_tensor(np.asarray(s, dtype=np.float32)).to(DEV).contiguous()
                                        for s in states]


def check_workload(wl, init_np, heads=None, tol=None, inputs=None, cu=None, ckpt_pos=None, chunk=None,
                   expect_path=None):
    """Run both sides and compare y and every checkpoint.  `init_np` holds
    per-sequence fp32 numpy states (or None); `heads` samples the oracle."""
    tol = tol or TOL[wl.shape.io_dtype]
    y, st, info = gpu_run(wl, to_dev(init_np), inputs=inputs, cu=cu, ckpt_pos=ckpt_pos, chunk=chunk)
    if expect_path is not None:
        assert info.path == expect_path
    y_ref, st_ref = oracle_on_heads(wl, heads, init_np, inputs=inputs, cu=cu, ckpt_pos=ckpt_pos)
    hs = list(range(wl.shape.nheads)) if heads is None else list(heads)
    y_g = y[:, hs].float().cpu().numpy()
    e_y = assert_close(y_g, y_ref, tol, "y")
    e_s = 0.0
    if st_ref.shape[0]:
        st_g = st[:, hs].cpu().numpy()
        assert st.dtype == torch.float32
        for k in range(st_ref.shape[0]):
            e_s = max(e_s, assert_close(st_g[k], st_ref[k], tol, f"checkpoint slot {k}"))
    say(f"    path={info.path} tiles={info.n_tiles} wgs={info.n_workgroups} err_y={e_y:.2e} err_state={e_s:.2e}")
    return y, st


def prefix_state(wl, heads=None):
    """Oracle state after the workload's random prefix, scanned from zero."""
    cu = np.array([0, wl.prefix_len], dtype=np.int32)
    _, st = oracle_on_heads(wl, heads, None, inputs=wl.prefix, cu=cu, ckpt_pos=[[wl.prefix_len]], want_y=False)
    return st[0].astype(np.float32)


# ---------------------------------------------------------------- configuration 0
def test_cfg0_tiny_f32_and_resume():
    say("cfg0: fp32, T=256, checkpoints {128,256}, then resume 129..256 from the 128-state")
    wl = make_workload(0, DEV)
    y, st = check_workload(wl, [None], expect_path=0)
    # resume on the GPU from the GPU's own checkpoint (the cache round trip)
    inp = wl.inputs
    tail = LayerInputs(x=inp.x[128:].contiguous(), dt=inp.dt[128:].contiguous(),
                       B=inp.B[128:].contiguous(), C=inp.C[128:].contiguous())
    y2, st2, _ = gpu_run(wl, [st[0]], inputs=tail, cu=np.array([0, 128], np.int32), ckpt_pos=[[128]])
    assert_close(y2.cpu().numpy(), y[128:].cpu().numpy(), 1e-5, "resumed y vs one-shot y")
    assert_close(st2[0].cpu().numpy(), st[1].cpu().numpy(), 1e-5, "resumed final state")
    # and against the oracle resumed from the oracle's own 128-state
    _, st_o = oracle_on_heads(wl, None, None)
    check_workload(wl, [st_o[0].astype(np.float32)], inputs=tail, cu=np.array([0, 128], np.int32),
                   ckpt_pos=[[128]])


def test_paper_position_example_f32():
    say("100 tokens, chunk 32, states at 64 (chunk boundary), 80 (exact) and 100; then 80+20 two-pass")
    shape = LayerShape(4, 16, 16, 1, 32, "f32")
    wl = make_workload(0, DEV, seed=5, seqlen=100, shape=shape)
    wl.ckpt_pos = [[64, 80, 100]]
    y, st = check_workload(wl, [None])
    inp = wl.inputs
    tail = LayerInputs(x=inp.x[80:].contiguous(), dt=inp.dt[80:].contiguous(),
                       B=inp.B[80:].contiguous(), C=inp.C[80:].contiguous())
    y2, st2, _ = gpu_run(wl, [st[1]], inputs=tail, cu=np.array([0, 20], np.int32), ckpt_pos=[[20]])
    assert_close(y2.cpu().numpy(), y[80:].cpu().numpy(), 1e-5, "second pass y")
    assert_close(st2[0].cpu().numpy(), st[2].cpu().numpy(), 1e-5, "second pass state")


# ---------------------------------------------------------------- small shapes, both paths
@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_valu_odd_shapes_varlen(io):
    say(f"VALU kernel, io={io}: H=6 P=24 N=40 G=3, ragged batch with empty and 1-token sequences")
    shape = LayerShape(6, 24, 40, 3, 64, io)
    wl = make_workload(2, DEV, seed=21, batch=6, len_range=(1, 150), shape=shape)
    lens = list(wl.seqlens)
    lens[1] = 0
    lens[3] = 1
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    inp = wl.inputs
    sub = LayerInputs(x=inp.x[:T].contiguous(), dt=inp.dt[:T].contiguous(),
                      B=inp.B[:T].contiguous(), C=inp.C[:T].contiguous())
    ck = []
    rs = np.random.RandomState(3)
    for L in lens:
        ck.append(sorted(set(int(v) for v in rs.randint(1, L + 1, size=2))) if L else [])
    init = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    check_workload(wl, init, inputs=sub, cu=cu, ckpt_pos=ck, expect_path=0)


def test_mfma_small_single_sequence():
    say("MFMA kernel: H=4 P=64 N=128 G=2, T=333 (ragged tiles), random init, checkpoints {1, 64, 65, 200, 333}")
    shape = LayerShape(4, 64, 128, 2, 256, "bf16")
    wl = make_workload(1, DEV, seed=31, seqlen=333, prefix_len=0, shape=shape)
    wl.ckpt_pos = [[1, 64, 65, 200, 333]]
    g = torch.Generator(device="cpu").manual_seed(4)
    init = [torch.randn((4, 64, 128), generator=g).numpy()]
    check_workload(wl, init, expect_path=1)
    check_workload(wl, [None], expect_path=1)


def test_mfma_varlen_batch_small():
    say("MFMA kernel: 7 requests U{1..700}, H=8, half with random init, 2 checkpoints each")
    shape = LayerShape(8, 64, 128, 1, 256, "bf16")
    wl = make_workload(2, DEV, seed=41, batch=7, len_range=(1, 700), shape=shape)
    init = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    check_workload(wl, init, expect_path=1)


def test_mfma_headdim_32_and_128():
    for P in (32, 128):
        say(f"MFMA kernel: headdim {P}")
        shape = LayerShape(4, P, 128, 4, 128, "bf16")
        wl = make_workload(1, DEV, seed=50 + P, seqlen=200, prefix_len=0, shape=shape)
        wl.ckpt_pos = [[77, 200]]
        check_workload(wl, [None], expect_path=1)


def test_chunk_parameter_only_changes_rounding():
    shape = LayerShape(4, 64, 128, 2, 256, "bf16")
    wl = make_workload(1, DEV, seed=61, seqlen=500, prefix_len=0, shape=shape)
    wl.ckpt_pos = [[123, 500]]
    ys = []
    for chunk in (16, 64, 256):
        say(f"chunk={chunk}")
        y, st = check_workload(wl, [None], chunk=chunk)
        ys.append((y.float().cpu().numpy(), st.cpu().numpy()))
    for y, st in ys[1:]:
        assert rel_err(y, ys[0][0])[0] <= 2e-2 and rel_err(st, ys[0][1])[0] <= 2e-2


def test_bitwise_determinism_and_packing_independence():
    say("two runs are bitwise equal; a sequence's results do not depend on its batch neighbours")
    shape = LayerShape(4, 64, 128, 2, 256, "bf16")
    wl = make_workload(2, DEV, seed=71, batch=4, len_range=(50, 400), shape=shape)
    init = to_dev([None if s is None else s.cpu().numpy() for s in wl.init_state])
    y1, s1, _ = gpu_run(wl, init)
    y2, s2, _ = gpu_run(wl, init)
    assert torch.equal(y1, y2) and torch.equal(s1, s2)
    k = 2
    a, b = int(wl.cu_seqlens[k]), int(wl.cu_seqlens[k + 1])
    inp = wl.inputs
    one = LayerInputs(x=inp.x[a:b].contiguous(), dt=inp.dt[a:b].contiguous(),
                      B=inp.B[a:b].contiguous(), C=inp.C[a:b].contiguous())
    y3, s3, _ = gpu_run(wl, [init[k]], inputs=one, cu=np.array([0, b - a], np.int32), ckpt_pos=[wl.ckpt_pos[k]])
    assert torch.equal(y3, y1[a:b])
    c0 = int(wl.cu_ckpt()[k])
    assert torch.equal(s3, s1[c0:c0 + len(wl.ckpt_pos[k])])


def test_off_by_one_checkpoint_is_detectable():
    shape = LayerShape(2, 64, 128, 1, 64, "bf16")
    wl = make_workload(1, DEV, seed=81, seqlen=130, prefix_len=0, shape=shape)
    wl.ckpt_pos = [[99, 100, 101]]
    _, st, _ = gpu_run(wl, None)
    _, st_ref = oracle_on_heads(wl, None, None)
    assert rel_err(st[1].cpu().numpy(), st_ref[1])[0] <= 2e-2
    assert rel_err(st[0].cpu().numpy(), st_ref[1])[0] > 5e-2
    assert rel_err(st[2].cpu().numpy(), st_ref[1])[0] > 5e-2


# ---------------------------------------------------------------- edge cases of the ABI on a GPU
def test_empty_batch_and_no_checkpoints():
    import paper_2411_19379_amd as ssm
    shape = LayerShape(4, 64, 128, 2, 256, "bf16")
    wl = make_workload(1, DEV, seed=91, seqlen=70, prefix_len=0, shape=shape)
    # no checkpoints at all: state_out may be NULL
    y, st, info = gpu_run(wl, None, ckpt_pos=[[]])
    assert st is None and info.n_ckpt == 0
    y_ref, _ = oracle_on_heads(wl, None, None, ckpt_pos=[[]])
    assert_close(y.float().cpu().numpy(), y_ref, 2e-2, "y without checkpoints")
    # zero tokens: succeeds, enqueues nothing
    plan = ssm.Plan(4, 64, 128, 2, 256, "bf16", [0, 0], [[]])
    empty = torch.empty((0, 4, 64), dtype=torch.bfloat16, device=DEV)
    ssm.ssm_prefill(plan.handle, 0, 0, 0, 0, 0, 0, None, 0, None, None, 0, None)
    plan.close()
    del empty


def test_misaligned_and_null_pointers_are_rejected():
    import paper_2411_19379_amd as ssm
    shape = LayerShape(4, 64, 128, 2, 256, "bf16")
    wl = make_workload(1, DEV, seed=92, seqlen=64, prefix_len=0, shape=shape)
    inp = wl.inputs
    plan = ssm.Plan(4, 64, 128, 2, 256, "bf16", [0, 64], [[64]])
    y = torch.empty_like(inp.x)
    st = torch.empty((1, 4, 64, 128), dtype=torch.float32, device=DEV)
    args = [inp.x.data_ptr(), inp.dt.data_ptr(), wl.A.data_ptr(), inp.B.data_ptr(), inp.C.data_ptr(),
            wl.D.data_ptr()]
    with pytest.raises(ssm.SsmError) as e:
        ssm.ssm_prefill(plan.handle, args[0] + 2, *args[1:], None, y.data_ptr(), st.data_ptr(), None, 0, None)
    assert e.value.status == "SSM_ERR_MISALIGNED"
    with pytest.raises(ssm.SsmError) as e:
        ssm.ssm_prefill(plan.handle, *args, None, y.data_ptr(), None, None, 0, None)
    assert e.value.status == "SSM_ERR_INVALID_ARG"
    plan.close()


def test_profile_mark_events_sit_between_the_kernels():
    """ssm_profile_mark: the events handed over are recorded on the call's stream after the operand preparation and
    after the scan, so start -> first, first -> second are positive and, with what follows the second, add up to the
    call; switching them off leaves a later call's timing events alone."""
    import paper_2411_19379_amd as ssm
    say("profile mark: event between the two kernels of the matrix-core scan")
    shape = LayerShape(8, 64, 128, 2, 256, "bf16")
    wl = make_workload(4, DEV, seed=3, shape=shape, seqlen=4096, ckpt_every=2048)
    plan = ssm.Plan(shape.nheads, shape.headdim, shape.d_state, shape.ngroups, shape.chunk, "bf16", wl.cu_seqlens,
                    wl.ckpt_pos)
    inp = wl.inputs
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()  # creates the HIP events
    y_ref, st_ref = ssm.prefill(plan, inp.x, inp.dt, wl.A, inp.B, inp.C, wl.D)
    torch.cuda.synchronize()
    ev[0].record()
    ssm.ssm_profile_mark(ev[1].cuda_event, ev[2].cuda_event)
    y, st = ssm.prefill(plan, inp.x, inp.dt, wl.A, inp.B, inp.C, wl.D)
    ev[3].record()
    ssm.ssm_profile_mark(None, None)
    torch.cuda.synchronize()
    prep, scan, rest = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]), ev[2].elapsed_time(ev[3])
    call = ev[0].elapsed_time(ev[3])
    say(f"    prep {prep * 1e3:.1f} us, scan {scan * 1e3:.1f} us, after it {rest * 1e3:.1f} us, call {call * 1e3:.1f} us")
    assert prep > 0 and scan > 0 and rest >= 0 and abs(prep + scan + rest - call) <= 0.05 * call + 0.01
    assert torch.equal(y, y_ref) and torch.equal(st, st_ref), "the mark must not change results"
    plan.close()


def test_decay_rates_far_beyond_the_usual_range():
    """A scaled by up to 1000: tiles whose total decay falls below 2^-100 take the exact per-entry exponential in the
    score mask instead of the two-factor form, decay-weighted inputs underflow to zero where the true weights are
    negligible, and cached states are forgotten within a few tokens.  Nothing may overflow or turn into NaN, and the
    oracle still agrees within the tolerance on every head."""
    say("decay rates x1 .. x1000: H=6 P=64 N=128 G=2, 3 requests with cached states and mid-tile checkpoints")
    shape = LayerShape(6, 64, 128, 2, 256, "bf16")
    wl = make_workload(2, DEV, seed=77, batch=3, len_range=(150, 500), shape=shape)
    wl.A = wl.A * torch.tensor([1.0, 5.0, 20.0, 60.0, 200.0, 1000.0], device=DEV)
    init_np = [None if s is None else s.cpu().numpy() for s in wl.init_state]
    check_workload(wl, init_np, expect_path=1)


@pytest.mark.parametrize("entry_name", ["ssm_prefill", "ssm_prefill_noalloc"])
def test_many_short_sequences(entry_name):
    """600 requests of 0 to 5 tokens, a third of them resuming from a cached state: sequence, tile and state-pointer
    tables longer than one upload, empty sequences among them, every tile partial."""
    import paper_2411_19379_amd as ssm
    say(f"600 sequences of 0..5 tokens through {entry_name}")
    shape = LayerShape(2, 64, 128, 1, 256, "bf16")
    rs = np.random.RandomState(5)
    lens = [int(v) for v in rs.randint(0, 6, size=600)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    g = torch.Generator(device=DEV).manual_seed(99)
    from workloads.gen import draw_layer_inputs, draw_layer_params
    A, D = draw_layer_params(shape, g, DEV)
    inp = draw_layer_inputs(shape, T, g, DEV)
    init = [torch.randn((2, 64, 128), generator=g, device=DEV) if (i % 3 == 0 and lens[i]) else None for i in range(600)]
    ckpt = [[L] if L else [] for L in lens]
    plan = ssm.Plan(2, 64, 128, 1, 256, "bf16", cu, ckpt)
    y, st = ssm.prefill(plan, inp.x, inp.dt, A, inp.B, inp.C, D, init, entry=getattr(ssm, entry_name))
    torch.cuda.synchronize()
    assert plan.info.batch == 600 and plan.info.n_tiles == sum(1 for L in lens if L)
    plan.close()
    from oracle import ssm_prefill_oracle
    y_ref, st_ref = ssm_prefill_oracle(inp.x.float().cpu().numpy(), inp.dt.float().cpu().numpy(), A.cpu().numpy(),
                                       inp.B.float().cpu().numpy(), inp.C.float().cpu().numpy(), D.cpu().numpy(), cu,
                                       [None if s is None else s.cpu().numpy() for s in init], ckpt)
    e_y = assert_close(y.float().cpu().numpy(), y_ref, TOL["bf16"], "y")
    e_s = assert_close(st.cpu().numpy(), st_ref, TOL["bf16"], "states")
    say(f"    err_y={e_y:.2e} err_state={e_s:.2e}")
