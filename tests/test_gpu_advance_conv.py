"""GPU parity of ssm_state_advance (roll-forward / decode step) and ssm_conv1d_prefill (the convolution in front of
the scan) against the oracles, through the C ABI."""
import numpy as np
import pytest
import torch

from helpers import rel_err
from oracle import conv1d_prefill_oracle, ssm_prefill_oracle
from workloads import LayerShape
from workloads.gen import _gen, draw_layer_inputs, draw_layer_params

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# (H, P, N, G, chunk), tokens per sequence
ADVANCE = {"decode": ((4, 64, 128, 2, 64), [1] * 5), "roll": ((2, 64, 128, 1, 64), [17, 0, 3, 64]),
           "small": ((4, 16, 16, 1, 64), [5, 2]), "odd_p": ((3, 24, 64, 3, 16), [9, 33]), "wide": ((1, 8, 256, 1, 64), [4]),
           "decode_7b": ((128, 64, 128, 8, 256), [1] * 4), "roll_k_le_chunk_7b": ((128, 64, 128, 8, 256), [256, 100])}
TORCH_ST = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.mark.parametrize("state_dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("case", sorted(ADVANCE))
def test_state_advance(io, case, state_dtype):
    import paper_2411_19379_amd as ssm
    (H, P, N, G, chunk), seqlens = ADVANCE[case]
    if io == "f32" and P * N > 8192:
        pytest.skip("no fp32 plan for this shape")
    if state_dtype != "f32" and (io == "f32" or case not in ("decode", "roll", "decode_7b")):
        pytest.skip("reduced-precision states are exercised on the bf16 cases only")
    print(f"advance {case} io={io} states={state_dtype}", flush=True)
    shape = LayerShape(H, P, N, G, chunk, io)
    g = _gen(DEV, 5)
    A, D = draw_layer_params(shape, g, DEV)
    T = int(sum(seqlens))
    inp = draw_layer_inputs(shape, T, g, DEV)
    tdt = TORCH_ST[state_dtype]
    states = [(torch.randn((H, P, N), generator=g, device=DEV) if b % 2 == 0 else torch.zeros((H, P, N), device=DEV)).to(tdt)
              for b in range(len(seqlens))]
    before = [s.float().cpu().numpy().copy() for s in states]   # representable starts
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    plan = ssm.Plan(H, P, N, G, chunk, io, cu, [[] for _ in seqlens], state_dtype=state_dtype)
    y = torch.full_like(inp.x, float("nan"))
    ssm.ssm_state_advance(plan.handle, inp.x.data_ptr(), inp.dt.data_ptr(), A.data_ptr(), inp.B.data_ptr(),
                          inp.C.data_ptr(), D.data_ptr(), [s.data_ptr() for s in states], y.data_ptr(),
                          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    plan.close()
    y_ref, st_ref = ssm_prefill_oracle(inp.x.cpu(), inp.dt.cpu(), A.cpu(), inp.B.cpu(), inp.C.cpu(), D.cpu(), cu, before,
                                       [[n] if n else [] for n in seqlens])
    assert max(rel_err(y.float().cpu().numpy(), y_ref)) <= (5e-3 if io == "bf16" else 1e-5)
    ulp = {"f32": 0.0, "f16": 2.0 ** -10, "bf16": 2.0 ** -7}[state_dtype]
    k = 0
    for b, n in enumerate(seqlens):
        got = states[b].float().cpu().numpy()
        if n == 0:
            assert np.array_equal(got, before[b])
        else:
            ref = st_ref[k]
            if state_dtype == "f32":
                assert max(rel_err(got, ref)) <= 1e-5
            else:  # one rounding on the way out, on top of fp32 arithmetic
                rms = float(np.sqrt(np.mean(ref * ref)))
                assert np.all(np.abs(got - ref) <= ulp * np.maximum(np.abs(ref), 2.0 ** -14) + 1e-5 * rms)
            k += 1


# (H, P, N, G, chunk) of the layer whose x, B and C pass through the convolution; sequence lengths; checkpoints
CONV = {"ragged": ((2, 64, 128, 1, 64), [79, 0, 1, 130], [[37, 79], [], [1], [2, 64, 65, 130]]),
        "short": ((1, 32, 128, 1, 64), [1, 2, 3], [[1], [1, 2], [3]]),
        "small": ((4, 16, 16, 1, 64), [40, 21], [[5, 40], []]),
        "7b_slice": ((128, 64, 128, 8, 256), [300], [[300]])}


@pytest.mark.parametrize("K", [1, 2, 4])
@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("case", sorted(CONV))
def test_conv1d(io, case, K):
    import paper_2411_19379_amd as ssm
    (H, P, N, G, chunk), seqlens, ckpts = CONV[case]
    if io == "f32" and P * N > 8192:
        pytest.skip("no fp32 plan for this shape")
    print(f"conv1d {case} io={io} K={K}", flush=True)
    C = H * P + 2 * G * N
    T = int(sum(seqlens))
    tdt = torch.float32 if io == "f32" else torch.bfloat16
    g = torch.Generator(device=DEV).manual_seed(1234 + K)
    xin = torch.randn((T, C), generator=g, device=DEV).to(tdt)
    w = (torch.randn((C, K), generator=g, device=DEV) / K ** 0.5).float()
    bias = torch.randn((C,), generator=g, device=DEV).float()
    init = [torch.randn((C, K), generator=g, device=DEV).to(tdt) if (n > 0 and b % 2 == 0) else None
            for b, n in enumerate(seqlens)]
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    plan = ssm.Plan(H, P, N, G, chunk, io, cu, ckpts)
    n_ck = sum(len(c) for c in ckpts)
    out = torch.full_like(xin, float("nan"))
    st = torch.full((max(n_ck, 1), C, K), float("nan"), dtype=tdt, device=DEV)
    ssm.ssm_conv1d_prefill(plan.handle, C, K, xin.data_ptr(), w.data_ptr(), bias.data_ptr(),
                           [None if v is None else v.data_ptr() for v in init], out.data_ptr(), st.data_ptr(), 1,
                           torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    plan.close()
    out_ref, st_ref = conv1d_prefill_oracle(xin.cpu(), w.cpu(), bias.cpu(), cu, [None if v is None else v.cpu() for v in init],
                                            ckpts, silu=True)
    assert max(rel_err(out.float().cpu().numpy(), out_ref)) <= (5e-3 if io == "bf16" else 1e-5)
    assert np.array_equal(st[:n_ck].float().cpu().numpy().astype(np.float64), st_ref)
