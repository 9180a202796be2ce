"""ssm_prefill_noalloc against ssm_prefill through the C ABI: two calls in a row, the second with a smaller input.
The file name sorts last so that a failure here hides no other test."""
import pytest
import torch

from workloads import LayerShape, make_workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(entry, wl, init):
    import paper_2411_19379_amd as ssm
    s = wl.shape
    plan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, s.io_dtype, wl.cu_seqlens, wl.ckpt_pos)
    y = torch.full_like(wl.inputs.x, float("nan"))
    st = torch.full((max(wl.n_ckpt, 1), s.nheads, s.headdim, s.d_state), float("nan"), dtype=torch.float32, device=DEV)
    ssm.prefill(plan, wl.inputs.x, wl.inputs.dt, wl.A, wl.inputs.B, wl.inputs.C, wl.D, init, y_out=y, state_out=st,
                entry=entry)
    torch.cuda.synchronize()
    plan.close()
    return y, st


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_noalloc_entry_matches_ssm_prefill(io):
    import paper_2411_19379_amd as ssm
    shape = LayerShape(4, 64, 128, 2, 256, io) if io == "bf16" else LayerShape(4, 16, 16, 1, 64, io)
    big = make_workload(2, DEV, seed=301, batch=5, len_range=(1, 500), shape=shape)
    small = make_workload(2, DEV, seed=302, batch=2, len_range=(1, 90), shape=shape)
    for wl in (big, small):  # the second call is smaller: stale table entries of the first must not matter
        print(f"noalloc {io}: {wl.batch} sequences, {wl.total_tokens} tokens", flush=True)
        init = list(wl.init_state)
        y_ref, st_ref = _run(ssm.ssm_prefill, wl, init)
        y, st = _run(ssm.ssm_prefill_noalloc, wl, init)
        # same kernels, same tables: bit-identical
        bits = torch.int16 if io == "bf16" else torch.int32
        assert torch.equal(y.view(bits), y_ref.view(bits))
        assert torch.equal(st[: wl.n_ckpt].view(torch.int32), st_ref[: wl.n_ckpt].view(torch.int32))
        assert not torch.isnan(y.float()).any() and not torch.isnan(st[: wl.n_ckpt]).any()


def test_noalloc_entry_with_sequences_cut_into_stretches():
    """A batch small enough for the plan to cut its long sequence into stretches: the stretch table travels through
    the fixed device array too, and the kernels behind the scan run in the same call."""
    import paper_2411_19379_amd as ssm
    shape = LayerShape(8, 64, 128, 2, 256, "bf16")
    big = make_workload(2, DEV, seed=311, batch=2, len_range=(10300, 13000), shape=shape)
    small = make_workload(2, DEV, seed=312, batch=1, len_range=(10300, 10300), shape=shape)
    for wl in (big, small):
        s = wl.shape
        plan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, s.io_dtype, wl.cu_seqlens, wl.ckpt_pos)
        n_stretches = plan.info.n_stretches
        plan.close()
        print(f"noalloc, cut: {wl.seqlens} tokens in {n_stretches} stretches", flush=True)
        assert n_stretches > wl.batch
        init = list(wl.init_state)
        y_ref, st_ref = _run(ssm.ssm_prefill, wl, init)
        y, st = _run(ssm.ssm_prefill_noalloc, wl, init)
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16))
        assert torch.equal(st[: wl.n_ckpt].view(torch.int32), st_ref[: wl.n_ckpt].view(torch.int32))
        assert not torch.isnan(y.float()).any() and not torch.isnan(st[: wl.n_ckpt]).any()


def test_noalloc_rejects_oversized_plans():
    import paper_2411_19379_amd as ssm
    # one checkpoint per token makes one tile per token: 17000 tiles > 16384
    T = 17000
    plan = ssm.Plan(1, 16, 16, 1, 16, "f32", [0, T], [list(range(1, T + 1))])
    with pytest.raises(ssm.SsmError) as e:
        ssm.ssm_prefill_noalloc(plan.handle, 256, 256, 256, 256, 256, 256, None, 256, 256, None, 0, None)
    assert e.value.code == ssm.SSM_ERR_UNSUPPORTED_SHAPE
    plan.close()


@pytest.mark.parametrize("lens", [(100, 700), (10300, 11000)])
def test_noalloc_entry_under_graph_capture(lens):
    """What the entry point is for: a caller that records its work into a HIP graph and may not allocate while it
    does.  The call is captured once (after one eager call, which sets the per-device tables' address up) and
    replayed several times with eager work and synchronisations in between; every replay, on inputs refreshed in
    place, equals the eager result.  With the longer requests the plan cuts sequences into stretches, and the kernels
    that carry the states over are part of the recorded call."""
    import paper_2411_19379_amd as ssm
    shape = LayerShape(8, 64, 128, 2, 256, "bf16")
    wl = make_workload(2, DEV, seed=303, batch=3, len_range=lens, shape=shape)
    init = list(wl.init_state)
    s = wl.shape
    plan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, s.io_dtype, wl.cu_seqlens, wl.ckpt_pos)
    plan.workspace(torch.device(DEV))  # allocated before the capture
    x = wl.inputs.x.clone()
    y = torch.empty_like(x)
    st = torch.empty((wl.n_ckpt, s.nheads, s.headdim, s.d_state), dtype=torch.float32, device=DEV)

    def call(xin, y_out, st_out):
        ssm.prefill(plan, xin, wl.inputs.dt, wl.A, wl.inputs.B, wl.inputs.C, wl.D, init, y_out=y_out, state_out=st_out,
                    entry=ssm.ssm_prefill_noalloc)

    call(x, y, st)  # eager: first use on this device
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(x, y, st)
    g = torch.Generator(device=DEV).manual_seed(7)
    for rep in range(4):
        print(f"noalloc under graph capture: replay {rep}", flush=True)
        x.copy_(torch.randn(x.shape, generator=g, device=DEV).to(x.dtype))  # new inputs, same buffers
        y_ref, st_ref = torch.empty_like(y), torch.empty_like(st)
        call(x, y_ref, st_ref)  # eager work between the replays
        torch.cuda.synchronize()
        y.fill_(float("nan"))
        st.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), f"replay {rep}: y differs from the eager call"
        assert torch.equal(st.view(torch.int32), st_ref.view(torch.int32)), f"replay {rep}: states differ"
    plan.close()
