#!/usr/bin/env python3
"""Benchmark of the SSM-layer prefill on one MI355X.

A step is one pass of the whole hot path (plan reuse, one `ssm_prefill` call:
operand preparation, decay prefix, masked scores, intra-chunk term, chunk
states, state passing, checkpoint emission, fused output) over one batch of
synthetic input that is already resident in HBM.  Prints ONE JSON line.
`value` and `ms_per_step` come from exactly K calls between two
synchronisations with nothing else in the stream; the per-kernel durations
(`roofline`) from the same K calls run once more with HIP events on the launch
stream, because events between a call's kernels keep them a few microseconds
apart (`config.ms_per_step_with_events`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]
                    [--no-checkpoints] [--calibrate-copy] [--no-cpu-baseline]

`--no-checkpoints` drops every checkpoint of the configuration (the cost of
checkpoint emission is the difference to the run with them).
`--calibrate-copy` also runs a plain device copy of 1 GiB a few times, which a
counter run (`rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`) needs to turn
counter units into bytes.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 / fp16, published
ROOT = os.path.dirname(os.path.abspath(__file__))

# HBM bytes per launch of the scan kernel, from two counter runs of this file
# (profiles/ssm_scan_mfma_kernel_cfg3_cfg4_hbm_bytes.txt gives the commands and the raw
# readings): FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each divided by
# what the same counter reads per KiB actually moved by the 1 GiB copy of
# --calibrate-copy.  Keyed by the hash of the kernel source the counters were
# taken on: once that source changes the figure is reported as null.
MEASURED_TRAFFIC = {
    "09ebaa5b38e19117bfe1aefad4dbf491f5e77987": {
        "cfg3_7b_32k_bf16": {"fetch_bytes": 845699359, "write_bytes": 546151619},
        "cfg4_7b_128k_ckpt4096_bf16": {"fetch_bytes": 3466112151, "write_bytes": 2289241906},
    },
}


def kernel_source_hash() -> str:
    with open(os.path.join(ROOT, "paper_2411_19379_amd", "csrc", "scan_mfma.hip"), "rb") as f:
        return hashlib.sha1(f.read()).hexdigest()


def algorithmic_bytes(wl, n_ckpt: int) -> int:
    """Compulsory HBM bytes of one call: x and y once, dt, B, C once, every
    non-null initial state read once, every checkpoint written once."""
    s = wl.shape
    esz = 4 if s.io_dtype == "f32" else 2
    per_token = (2 * s.nheads * s.headdim + s.nheads + 2 * s.ngroups * s.d_state) * esz
    state = s.nheads * s.headdim * s.d_state * 4
    n_init = sum(1 for k in wl.init_kind if k != "zeros")
    return wl.total_tokens * per_token + (n_init + n_ckpt) * state


def algorithmic_flops(wl, tile: int) -> float:
    """Dense-tile flops of the chunked form with tiles of `tile` tokens, per
    (token, head): masked scores 2*q*N shared by the heads of a group, intra
    term 2*q*P, state update 2*P*N, state-times-C 2*P*N."""
    s = wl.shape
    per_th = 2 * tile * s.d_state * s.ngroups / s.nheads + 2 * tile * s.headdim + 4 * s.headdim * s.d_state
    return float(wl.total_tokens) * s.nheads * per_th


def cpu_baseline(wl, sample_tokens: int, min_seconds: float = 10.0, max_repeats: int = 16):
    """The oracle as it stands on the host cores, on the first `sample_tokens`
    tokens of the first sequence (all heads, zero initial state), repeated
    until about `min_seconds` of CPU work have been timed."""
    import oracle

    n = min(sample_tokens, wl.seqlens[0])
    inp = wl.inputs
    x = inp.x[:n].float().cpu().numpy()
    dt = inp.dt[:n].float().cpu().numpy()
    B = inp.B[:n].float().cpu().numpy()
    C = inp.C[:n].float().cpu().numpy()
    A = wl.A.cpu().numpy()
    D = wl.D.cpu().numpy()
    threads = oracle.max_threads()
    oracle.ssm_prefill_oracle(x[:16], dt[:16], A, B[:16], C[:16], D, [0, 16], None, [[16]])  # load + warm
    reps = 0
    t0 = time.perf_counter()
    while reps < max_repeats:
        oracle.ssm_prefill_oracle(x, dt, A, B, C, D, [0, n], None, [[n]], nthreads=threads)
        reps += 1
        if time.perf_counter() - t0 >= min_seconds:
            break
    el = time.perf_counter() - t0
    return {"value": n * reps / el, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n} tokens of the workload, all {wl.shape.nheads} heads, zero initial state, "
                      f"one checkpoint, {reps} passes; {el:.1f} s"}


def side_op(args, ssm, torch, dev) -> int:
    """The kernels beside the scan at the 7B layer shape, each HBM-streaming: the decode step over a batch of cached
    states (`ssm_state_advance`, one token per sequence: every state is read and written once) and the causal
    convolution in front of the scan over 32768 tokens (`ssm_conv1d_prefill`: input read once, output written once).
    One JSON line with the achieved fraction of the HBM roofline on the algorithmic bytes."""
    from workloads import LayerShape
    from workloads.gen import _gen, draw_layer_inputs, draw_layer_params

    shape = LayerShape(128, 64, 128, 8, 256, "bf16")
    H, P, N, G = shape.nheads, shape.headdim, shape.d_state, shape.ngroups
    g = _gen(dev, 77)
    stream = torch.cuda.current_stream().cuda_stream
    if args.op == "advance":
        batch = args.decode_batch
        A, D = draw_layer_params(shape, g, dev)
        inp = draw_layer_inputs(shape, batch, g, dev)
        states = [torch.randn((H, P, N), generator=g, device=dev) for _ in range(batch)]
        plan = ssm.Plan(H, P, N, G, shape.chunk, "bf16", list(range(batch + 1)), [[] for _ in range(batch)])
        y = torch.empty_like(inp.x)
        ptrs = [t.data_ptr() for t in states]

        def step():
            ssm.ssm_state_advance(plan.handle, inp.x.data_ptr(), inp.dt.data_ptr(), A.data_ptr(), inp.B.data_ptr(),
                                  inp.C.data_ptr(), D.data_ptr(), ptrs, y.data_ptr(), stream)

        tokens = batch
        abytes = batch * (2 * H * P * N * 4 + (2 * H * P + H + 2 * G * N) * 2)
        name, kernel, metric = f"advance_7b_decode_b{batch}", "ssm_advance_kernel", "decode-step tokens/s per SSM layer (1 GPU)"
    else:
        T, K = 32768, 4
        C = H * P + 2 * G * N
        xin = torch.randn((T, C), generator=g, device=dev).to(torch.bfloat16)
        w = (torch.randn((C, K), generator=g, device=dev) / K ** 0.5).float()
        bias = torch.randn((C,), generator=g, device=dev).float()
        plan = ssm.Plan(H, P, N, G, shape.chunk, "bf16", [0, T], [[T]])
        out = torch.empty_like(xin)
        st = torch.empty((1, C, K), dtype=torch.bfloat16, device=dev)

        def step():
            ssm.ssm_conv1d_prefill(plan.handle, C, K, xin.data_ptr(), w.data_ptr(), bias.data_ptr(), None,
                                   out.data_ptr(), st.data_ptr(), 1, stream)

        tokens = T
        abytes = 2 * T * C * 2 + C * K * 2
        name, kernel, metric = "conv1d_7b_32k_k4", "ssm_conv1d_kernel", "convolution tokens/s per SSM layer (1 GPU)"
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ev = []
    for _ in range(args.steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step()
        b.record()
        ev.append((a, b))
    torch.cuda.synchronize()
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    plan.close()
    achieved = abytes / (kern_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": metric, "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "tokens": tokens, "nheads": H, "headdim": P, "d_state": N, "ngroups": G},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": kernel, "kernel_ms": kern_ms,
                     "algorithmic_bytes": abytes}}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=3, help="named configuration 0..4 (default: the 7B 32K one)")
    ap.add_argument("--no-checkpoints", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=32768)
    ap.add_argument("--decode-batch", type=int, default=64, help="sequences of --op advance (one token each)")
    ap.add_argument("--op", choices=["prefill", "advance", "conv1d"], default="prefill",
                    help="prefill: the hot path (default); advance / conv1d: the two kernels beside it, one line each")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1", file=sys.stderr)
        return 2

    import torch

    import paper_2411_19379_amd as ssm
    from workloads import make_workload

    ssm.load_library()  # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.op != "prefill":
        return side_op(args, ssm, torch, dev)
    wl = make_workload(args.config, dev)
    s = wl.shape
    inp = wl.inputs
    ckpt_pos = [[] for _ in wl.ckpt_pos] if args.no_checkpoints else wl.ckpt_pos
    n_ckpt = sum(len(c) for c in ckpt_pos)

    # Initial states: random fp32 ones come with the workload; a "prefix" one
    # is the library's own state after scanning the random prefix from zero,
    # i.e. the cache entry a previous request would have left behind.
    init = list(wl.init_state)
    if wl.prefix is not None:
        pplan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, s.io_dtype,
                         [0, wl.prefix_len], [[wl.prefix_len]])
        _, pst = ssm.prefill(pplan, wl.prefix.x, wl.prefix.dt, wl.A, wl.prefix.B, wl.prefix.C, wl.D)
        torch.cuda.synchronize()
        pplan.close()
        init = [pst[0].contiguous()]
        wl.prefix = None
    if all(v is None for v in init):
        init = None

    t0 = time.perf_counter()
    plan = ssm.Plan(s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, s.io_dtype, wl.cu_seqlens, ckpt_pos)
    plan_ms = (time.perf_counter() - t0) * 1e3
    mfma = plan.info.path == ssm.SSM_PATH_MFMA_BF16
    y = torch.empty_like(inp.x)
    st = torch.empty((max(n_ckpt, 1), s.nheads, s.headdim, s.d_state), dtype=torch.float32, device=dev)

    def step():
        ssm.prefill(plan, inp.x, inp.dt, wl.A, inp.B, inp.C, wl.D, init, y_out=y, state_out=st)

    def new_event():
        e = torch.cuda.Event(enable_timing=True)
        e.record()  # creates the underlying HIP event, whose handle ssm_profile_mark takes
        return e

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region: exactly `steps` calls between two synchronisations, nothing else in the stream.
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    T = wl.total_tokens

    # The same `steps` calls once more with HIP events on the stream the kernels are launched on (torch's current
    # stream): start, after the operand preparation and after the scan kernel of the matrix-core path (both recorded by
    # the library), end.  Kept out of the region above because every event between two kernels keeps them some
    # microseconds apart; the kernels' own durations are the same in both.
    ev = [(new_event(), new_event(), new_event(), new_event()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # kernels behind the scan exist only when long sequences were cut into stretches (the carried states'
    # contribution); only then is the second event recorded
    cut = mfma and plan.info.n_stretches > wl.batch
    for a, m, m2, b in ev:
        a.record()
        if mfma:
            ssm.ssm_profile_mark(m.cuda_event, m2.cuda_event if cut else None)
        step()
        b.record()
    torch.cuda.synchronize()
    events_ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ssm.ssm_profile_mark(None, None)
    call_ms = np.array([a.elapsed_time(b) for a, _, _, b in ev])
    scan_ms = np.array([m.elapsed_time(m2 if cut else b) for _, m, m2, b in ev]) if mfma else call_ms
    prep_ms = np.array([a.elapsed_time(m) for a, m, _, _ in ev]) if mfma else np.zeros_like(call_ms)
    tail_ms = np.array([m2.elapsed_time(b) for _, _, m2, b in ev]) if cut else np.zeros_like(call_ms)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    kern_ms = float(scan_ms.mean())
    abytes = algorithmic_bytes(wl, n_ckpt)
    achieved = abytes / (kern_ms * 1e-3) / 1e9
    flops = algorithmic_flops(wl, plan.info.tile_tokens)
    traffic = None
    if mfma:
        m = MEASURED_TRAFFIC.get(kernel_source_hash(), {}).get(wl.name + ("_nockpt" if args.no_checkpoints else ""))
        if m:
            traffic = m["fetch_bytes"] + m["write_bytes"]
    out = {
        "metric": "SSM-layer prefill tokens/s (1 GPU) with state checkpoints",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if s.io_dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "tokens": T, "batch": wl.batch, "nheads": s.nheads,
                   "headdim": s.headdim, "d_state": s.d_state, "ngroups": s.ngroups, "chunk": s.chunk,
                   "checkpoints": n_ckpt,
                   "initial_states": 0 if init is None else sum(1 for v in init if v is not None),
                   "kernel_path": "mfma_bf16" if mfma else "valu_f32",
                   "workgroups": plan.info.n_workgroups, "stretches": plan.info.n_stretches, "plan_ms": plan_ms,
                   "call_ms_mean": float(call_ms.mean()), "call_ms_median": float(np.median(call_ms)),
                   "call_ms_min": float(call_ms.min()), "ms_per_step_with_events": events_ms_per_step},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "ssm_scan_mfma_kernel" if mfma else "ssm_scan_valu_kernel",
                     "kernel_ms": kern_ms, "kernel_ms_median": float(np.median(scan_ms)),
                     "kernel_ms_min": float(scan_ms.min()),
                     "prep_kernel": "ssm_prep_kernel" if mfma else None, "prep_kernel_ms": float(prep_ms.mean()),
                     "carry_kernels_ms": float(tail_ms.mean()),
                     "algorithmic_bytes": abytes,
                     "whole_call_frac": abytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "mfma_tflops_dense_tile": flops / (kern_ms * 1e-3) / 1e12,
                     "mfma_frac": flops / (kern_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_tokens)
    plan.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
