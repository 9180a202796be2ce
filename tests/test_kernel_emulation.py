"""The shipped scan kernels, compiled for the CPU and run on a SIMT emulator.

No GPU is involved and nothing here is reachable from the library: the kernel
sources of `paper_2411_19379_amd/csrc` are compiled as plain C++ against
`tests/kernel_emu` (one fiber per lane; matrix-core products, LDS transpose
reads, DPP shifts and lane reads evaluated per wave from the gfx950 operand
layouts) and driven on seeded workloads.  Checked:

* results against the fp64 oracle, to the tolerance of the storage type;
* LDS ordering: between two workgroup barriers the emulator runs the waves one
  after another in forward, reverse and shuffled order, and every order must
  give bit-identical outputs (a read/write race between two waves cannot);
* bounds: LDS and every global buffer sit flush against an inaccessible page,
  once with the end and once with the start of the buffer at the page, so any
  access outside a buffer kills the run; LDS and the outputs start as NaN
  patterns, so a value read before it is written, or an output never written,
  shows up as a non-finite result;
* the checker itself: with one barrier made not to wait, the orders disagree.

The same checks run on the roll-forward kernel (`state_advance.hip`) and on the convolution in front of the scan
(`conv1d_prefill.hip`).

The only edits to the kernel sources are textual and listed in `_convert`: the
two LDS-wait/barrier instructions become emulator calls and the dynamic LDS
array becomes a pointer to the emulated LDS.
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess

import numpy as np
import pytest
import torch

from helpers import TOL, rel_err
from oracle import ssm_prefill_oracle
from workloads import LayerShape, make_workload

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMU = os.path.join(ROOT, "tests", "kernel_emu")
CSRC = os.path.join(ROOT, "paper_2411_19379_amd", "csrc")
CLANG = shutil.which("amdclang++") or "/opt/rocm/lib/llvm/bin/clang++"

_SUBST = [
    (r'asm volatile\("s_waitcnt lgkmcnt\(0\)\\n\\ts_barrier" ::: "memory"\);', "emu::barrier(__LINE__);"),
    (r'asm volatile\("s_waitcnt lgkmcnt\(0\)" ::: "memory"\);', "emu::wave_sync(__LINE__);"),
    (r"extern __shared__ __align__\(16\) unsigned char lds_raw\[\];", "unsigned char *lds_raw = emu::lds_base();"),
    (r'asm volatile\("" ::: "memory"\);', ";"),  # compiler-only fence: nothing to emulate
    (r'asm volatile\("" : "\+v"\(Sl\[c\]\)\);', ";"),  # pins a value in front of what follows: nothing to emulate
]


def _convert(src: str, dst: str) -> None:
    text = open(src).read()
    for pat, rep in _SUBST:
        text = re.sub(pat, rep, text)
    assert "asm volatile" not in text and "__shared__" not in text, f"{src}: construct the emulator does not know"
    open(dst, "w").write(text)


def _build(tmp_path_factory, name, mfma_source, extra_flags=(), extra_sources=()):
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with bf16 vector support found")
    d = str(tmp_path_factory.mktemp(name))
    _convert(mfma_source, os.path.join(d, "scan_mfma.cpp"))
    _convert(os.path.join(CSRC, "scan_valu.hip"), os.path.join(d, "scan_valu.cpp"))
    flags = ["-std=c++17", "-O2", "-fno-strict-aliasing", "-ffp-contract=off", "-Wno-psabi", "-Wno-unused-value",
             "-I", EMU, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra_flags]
    _convert(os.path.join(CSRC, "state_advance.hip"), os.path.join(d, "state_advance.cpp"))
    srcs = [os.path.join(d, "scan_mfma.cpp"), os.path.join(d, "scan_valu.cpp"), os.path.join(d, "state_advance.cpp"),
            os.path.join(CSRC, "plan.cpp"), os.path.join(EMU, "emu_rt.cpp"), os.path.join(EMU, "emu_main.cpp")]
    for k, src in enumerate(extra_sources):
        _convert(src, os.path.join(d, f"extra{k}.cpp"))
        srcs.append(os.path.join(d, f"extra{k}.cpp"))
    objs = []
    procs = []
    for s in srcs:
        o = os.path.join(d, os.path.basename(s) + ".o")
        objs.append(o)
        procs.append(subprocess.Popen([CLANG, *flags, "-c", s, "-o", o], stderr=subprocess.PIPE, text=True))
    for p in procs:
        _, err = p.communicate()
        assert p.returncode == 0, err[-3000:]
    out = os.path.join(d, "emu_main")
    subprocess.run([CLANG, *objs, "-o", out], check=True)
    return out


@pytest.fixture(scope="session")
def emu_binary(tmp_path_factory):
    """The shipped kernels."""
    return _build(tmp_path_factory, "kernel_emu", os.path.join(CSRC, "scan_mfma.hip"))


@pytest.fixture(scope="session")
def emu_binary_4waves(tmp_path_factory):
    """The matrix-core scan with 4 waves per workgroup instead of the shipped 12 (32 channels) or 8 (64 channels)."""
    return _build(tmp_path_factory, "kernel_emu4", os.path.join(CSRC, "scan_mfma.hip"), ["-DSSM_SCAN_WAVES=4", "-DSSM_SCAN_WAVES_NARROW=4", "-DSSM_FIX_FINE_TILES=8"])


@pytest.fixture(scope="session")
def emu_conv_binary(tmp_path_factory):
    """The convolution kernel with its own driver."""
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with bf16 vector support found")
    d = str(tmp_path_factory.mktemp("kernel_emu_conv"))
    _convert(os.path.join(CSRC, "conv1d_prefill.hip"), os.path.join(d, "conv1d_prefill.cpp"))
    flags = ["-std=c++17", "-O2", "-fno-strict-aliasing", "-ffp-contract=off", "-Wno-psabi", "-Wno-unused-value",
             "-I", EMU, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    srcs = [os.path.join(d, "conv1d_prefill.cpp"), os.path.join(CSRC, "plan.cpp"), os.path.join(EMU, "emu_rt.cpp"),
            os.path.join(EMU, "emu_conv_main.cpp")]
    out = os.path.join(d, "emu_conv_main")
    subprocess.run([CLANG, *flags, *srcs, "-o", out], check=True, capture_output=True)
    return out


def _write_problem(path, wl, init_states):
    s = wl.shape
    io = 0 if s.io_dtype == "f32" else 1
    with open(path, "wb") as f:
        np.asarray([0x53534D31, io, wl.total_tokens, s.nheads, s.headdim, s.d_state, s.ngroups, s.chunk, wl.batch,
                    wl.n_ckpt], dtype=np.int32).tofile(f)
        np.asarray(wl.cu_seqlens, dtype=np.int32).tofile(f)
        np.asarray(wl.cu_ckpt(), dtype=np.int32).tofile(f)
        np.asarray(wl.ckpt_flat(), dtype=np.int32)[: wl.n_ckpt].tofile(f)
        np.asarray([0 if v is None else 1 for v in init_states], dtype=np.int32).tofile(f)
        for t in (wl.inputs.x, wl.inputs.dt, wl.inputs.B, wl.inputs.C):
            t = t.contiguous().cpu()
            (t.view(torch.int16) if io else t).numpy().tofile(f)
        wl.A.cpu().numpy().astype(np.float32).tofile(f)
        wl.D.cpu().numpy().astype(np.float32).tofile(f)
        for v in init_states:
            if v is not None:
                np.ascontiguousarray(v.cpu().numpy(), dtype=np.float32).tofile(f)


def _read_result(path, wl, n_states=None):
    s = wl.shape
    nx = wl.total_tokens * s.nheads * s.headdim
    raw = np.fromfile(path, dtype=np.uint8)
    if s.io_dtype == "f32":
        y = raw[: nx * 4].view(np.float32).astype(np.float64)
        off = nx * 4
    else:
        y = torch.from_numpy(raw[: nx * 2].view(np.int16).copy()).view(torch.bfloat16).float().numpy().astype(np.float64)
        off = nx * 2
    st = raw[off:].view(np.float32).reshape(wl.n_ckpt if n_states is None else n_states, s.nheads, s.headdim,
                                            s.d_state)
    return y.reshape(wl.total_tokens, s.nheads, s.headdim), st, raw


def _emulate(binary, wl, init, tmp_path, order, align, drop=None, advance=False, state_type=None, wide=False,
             split=None):
    pin = str(tmp_path / "in.bin")
    pout = str(tmp_path / f"out_{order}_{align}_{drop}_{advance}_{state_type}_{wide}_{split}.bin".replace(":", "-"))
    if not os.path.exists(pin):
        _write_problem(pin, wl, init)
    cmd = [binary, pin, pout, str(order), align]
    if drop is not None or advance or state_type:
        cmd.append(str(-1 if drop is None else drop))
    if advance or state_type:
        cmd.append("advance" if advance else "scan")
        if state_type:
            cmd.append(state_type)
    env = dict(os.environ, EMU_WIDE="1") if wide else None  # the 64-channel variant of the matrix-core scan
    if split:  # "K:min": sequences cut into up to K stretches of at least `min` tiles
        env = dict(os.environ, EMU_SPLIT=split)
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, f"emulated kernel died (rc {r.returncode}): {r.stderr[-800:]}"
    return _read_result(pout, wl, n_states=wl.batch if advance else None)


def _oracle(wl, init):
    return ssm_prefill_oracle(wl.inputs.x, wl.inputs.dt, wl.A, wl.inputs.B, wl.inputs.C, wl.D, wl.cu_seqlens,
                              [None if v is None else v.cpu().numpy() for v in init], wl.ckpt_pos)


def _with_empty_sequence(wl):
    """Insert a zero-length sequence in the middle of the packed batch."""
    wl.seqlens.insert(1, 0)
    wl.cu_seqlens = np.concatenate([[0], np.cumsum(wl.seqlens)]).astype(np.int32)
    wl.ckpt_pos.insert(1, [])
    wl.init_kind.insert(1, "zeros")
    wl.init_state.insert(1, None)
    return wl


# name: (H, P, N, G, chunk), configuration of the generator, its overrides
CASES = {
    # ragged packed batch: partial tiles, checkpoints inside tiles, sequences starting from a cached state
    "ragged": ((2, 64, 128, 1, 64), 2, dict(batch=3, len_range=(1, 300))),
    # one sequence over several tiles, periodic checkpoints, no checkpoint at the end
    "long": ((2, 64, 128, 1, 64), 4, dict(seqlen=450, ckpt_every=100)),
    # sequences shorter than any tile
    "tiny": ((2, 64, 128, 1, 64), 2, dict(batch=2, len_range=(1, 3))),
    # one 32-channel slice per head, several groups with several heads each, 32-token tiles
    "p32_groups": ((4, 32, 128, 2, 32), 2, dict(batch=2, len_range=(20, 120))),
    # seven heads per group: the four workgroups per (tile, group) of the kernel in front of the scan share them 1, 2, 2, 2
    "heads7": ((7, 32, 128, 1, 64), 2, dict(batch=2, len_range=(40, 150))),
    # one head, 21 tiles: cut in two, the second stretch is longer than the 8 tiles that the small build of the
    # second kernel gives workgroups of their own, so its coarse groups get the rest
    "long2": ((1, 64, 128, 1, 64), 4, dict(seqlen=1300, ckpt_every=500)),
    # four slices per head, large chunk
    "p128": ((1, 128, 128, 1, 256), 4, dict(seqlen=200, ckpt_every=64)),
    # shapes outside the matrix-core path (any storage type takes the fp32 vector kernel)
    "odd": ((6, 24, 40, 3, 64), 2, dict(batch=4, len_range=(1, 90))),
    # a zero-length sequence inside the batch
    "empty_seq": ((2, 64, 128, 1, 64), 2, dict(batch=3, len_range=(30, 100))),
    # decay rates from the usual range up to 400 times it: tiles whose total decay is below 2^-100 take one exponential
    # per score instead of the two-factor form, and weights underflow to zero where the true ones are negligible
    "strong_decay": ((3, 64, 128, 1, 64), 2, dict(batch=2, len_range=(60, 200), a_scale=[1.0, 40.0, 400.0])),
}


def _check_case(binary, tmp_path, io, case, state_tol=None, y_tol=None, wide=False, split=None):
    (H, P, N, G, chunk), cfg, kw = CASES[case]
    if io == "f32" and P * N > 8192:
        pytest.skip("the fp32 vector kernel holds at most 8192 state elements per head")
    shape = LayerShape(nheads=H, headdim=P, d_state=N, ngroups=G, chunk=chunk, io_dtype=io)
    kw = dict(kw)
    a_scale = kw.pop("a_scale", None)
    wl = make_workload(cfg, "cpu", seed=11, shape=shape, **kw)
    if a_scale is not None:
        wl.A = wl.A * torch.tensor(a_scale, dtype=wl.A.dtype)
    if case == "empty_seq":
        wl = _with_empty_sequence(wl)
    init = list(wl.init_state)
    y_ref, st_ref = _oracle(wl, init)
    first = None
    for order, align in ((0, "end"), (1, "start"), (7, "end"), (12, "start")):
        y, st, raw = _emulate(binary, wl, init, tmp_path, order, align, wide=wide, split=split)
        assert np.all(np.isfinite(y)) and np.all(np.isfinite(st)), "an output was never written, or LDS was read before written"
        assert max(rel_err(y, y_ref)) <= (y_tol or TOL[io])
        assert max(rel_err(st.astype(np.float64), st_ref)) <= (state_tol or TOL[io])
        if first is None:
            first = raw
        assert np.array_equal(first, raw), f"wave order {order} changes the result: LDS race"


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("case", sorted(CASES))
def test_emulated_kernel_matches_oracle_in_any_wave_order(emu_binary, tmp_path, io, case):
    _check_case(emu_binary, tmp_path, io, case)


ADVANCE_CASES = {
    # decode step: one token per sequence, some sequences with a cached state, some from zero
    "decode": ((4, 64, 128, 2, 64), [1, 1, 1, 1, 1]),
    # roll-forward by a few tokens, one sequence left alone (no tokens)
    "roll": ((2, 64, 128, 1, 64), [17, 0, 3, 64]),
    # small and unusual shapes: N = 16 (4 lanes per row), P not a multiple of the rows per pass
    "small": ((4, 16, 16, 1, 64), [5, 2]),
    "odd_p": ((3, 24, 64, 3, 16), [9, 33]),
    "wide": ((1, 8, 256, 1, 64), [4]),
}


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("case", sorted(ADVANCE_CASES))
def test_state_advance_matches_oracle(emu_binary, tmp_path, io, case):
    """The roll-forward kernel: states advanced in place and y against the oracle started from the same states.
    All arithmetic is fp32, so states are held to 1e-5 whatever the storage type; y carries its storage rounding."""
    (H, P, N, G, chunk), seqlens = ADVANCE_CASES[case]
    shape = LayerShape(nheads=H, headdim=P, d_state=N, ngroups=G, chunk=chunk, io_dtype=io)
    wl = make_workload(2, "cpu", seed=23, shape=shape, batch=len(seqlens), len_range=(1, 2))
    # impose the lengths of the case on the drawn batch (inputs are per token, so redraw them at the new total)
    from workloads.gen import _gen, draw_layer_inputs
    wl.seqlens = list(seqlens)
    wl.cu_seqlens = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    wl.inputs = draw_layer_inputs(shape, int(sum(seqlens)), _gen("cpu", 77), "cpu")
    wl.ckpt_pos = [[n] if n > 0 else [] for n in seqlens]  # the oracle's checkpoint = the state after the last token
    init = list(wl.init_state)
    y_ref, st_ref = _oracle(wl, init)
    first = None
    for order, align in ((0, "end"), (1, "start")):
        y, st, raw = _emulate(emu_binary, wl, init, tmp_path, order, align, advance=True)
        assert np.all(np.isfinite(y)) and np.all(np.isfinite(st))
        assert max(rel_err(y, y_ref)) <= (5e-3 if io == "bf16" else 1e-5)
        k = 0
        for b, n in enumerate(seqlens):
            if n == 0:  # untouched: still the initial state (or zeros)
                want = np.zeros_like(st[b]) if init[b] is None else init[b].numpy()
                assert np.array_equal(st[b], want)
            else:
                assert max(rel_err(st[b].astype(np.float64), st_ref[k])) <= 1e-5
                k += 1
        if first is None:
            first = raw
        assert np.array_equal(first, raw)


CONV_CASES = {
    # (H, P, N, G, chunk) of the layer whose x, B and C pass through the convolution; sequence lengths; checkpoints
    "ragged": ((2, 64, 128, 1, 64), [79, 0, 1, 130], [[37, 79], [], [1], [2, 64, 65, 130]]),
    "short": ((1, 32, 128, 1, 64), [1, 2, 3], [[1], [1, 2], [3]]),
    "small_f32_tiles": ((4, 16, 16, 1, 64), [40, 21], [[5, 40], []]),
}


@pytest.mark.parametrize("K", [1, 2, 4])
@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("case", sorted(CONV_CASES))
def test_conv1d_matches_oracle(emu_conv_binary, tmp_path, io, case, K):
    """Outputs against the convolution oracle from the same cached states; checkpointed states are copies of
    inputs and must be bit-exact."""
    from oracle import conv1d_prefill_oracle
    (H, P, N, G, chunk), seqlens, ckpts = CONV_CASES[case]
    if io == "f32" and P * N > 8192:
        pytest.skip("no fp32 plan for this layer shape")
    C = H * P + 2 * G * N
    T = int(sum(seqlens))
    g = torch.Generator().manual_seed(1234 + K)
    tdt = torch.float32 if io == "f32" else torch.bfloat16
    xin = torch.randn((T, C), generator=g).to(tdt)
    w = (torch.randn((C, K), generator=g) / K ** 0.5).float()
    bias = torch.randn((C,), generator=g).float()
    init = [torch.randn((C, K), generator=g).to(tdt) if (n > 0 and b % 2 == 0) else None for b, n in enumerate(seqlens)]
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    cu_ck = np.concatenate([[0], np.cumsum([len(c) for c in ckpts])]).astype(np.int32)
    flat = np.asarray([p for c in ckpts for p in c], dtype=np.int32)
    out_ref, st_ref = conv1d_prefill_oracle(xin, w, bias, cu, init, ckpts, silu=True)

    pin = str(tmp_path / "in.bin")
    raw = (lambda t: t.contiguous().view(torch.int16).numpy()) if io == "bf16" else (lambda t: t.contiguous().numpy())
    with open(pin, "wb") as f:
        np.asarray([0x434F4E56, 0 if io == "f32" else 1, T, H, P, N, G, chunk, len(seqlens), len(flat), K, 1, 1],
                   dtype=np.int32).tofile(f)
        cu.tofile(f), cu_ck.tofile(f), flat.tofile(f)
        np.asarray([0 if v is None else 1 for v in init], dtype=np.int32).tofile(f)
        raw(xin).tofile(f), w.numpy().tofile(f), bias.numpy().tofile(f)
        for v in init:
            if v is not None:
                raw(v).tofile(f)
    first = None
    for order, align in ((0, "end"), (1, "start")):
        pout = str(tmp_path / f"out_{order}.bin")
        r = subprocess.run([emu_conv_binary, pin, pout, str(order), align], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, f"emulated kernel died (rc {r.returncode}): {r.stderr[-800:]}"
        got = np.fromfile(pout, dtype=np.uint8)
        esz = 4 if io == "f32" else 2
        def dec(b):
            if io == "f32":
                return b.view(np.float32).astype(np.float64)
            return torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).float().numpy().astype(np.float64)
        out = dec(got[: T * C * esz]).reshape(T, C)
        st = dec(got[T * C * esz:]).reshape(len(flat), C, K)
        assert np.all(np.isfinite(out)) and np.all(np.isfinite(st))
        assert max(rel_err(out, out_ref)) <= (5e-3 if io == "bf16" else 1e-5)
        assert np.array_equal(st, st_ref), "a checkpointed state is not the last K inputs"
        if first is None:
            first = got
        assert np.array_equal(first, got)


@pytest.mark.parametrize("state_type,ulp", [("f16", 2.0 ** -10), ("bf16", 2.0 ** -7)])
def test_state_advance_with_reduced_precision_states(emu_binary, tmp_path, state_type, ulp):
    """States kept as a cache stores them (Section 5.1: FP16): read, advanced in fp32, rounded once on the way back.
    Expected: the oracle's state from the same (representable) start, to one unit in the last place of the type."""
    (H, P, N, G, chunk), seqlens = (4, 64, 128, 2, 64), [1, 7, 0, 2]
    shape = LayerShape(nheads=H, headdim=P, d_state=N, ngroups=G, chunk=chunk, io_dtype="bf16")
    wl = make_workload(2, "cpu", seed=29, shape=shape, batch=len(seqlens), len_range=(1, 2))
    from workloads.gen import _gen, draw_layer_inputs
    wl.seqlens = list(seqlens)
    wl.cu_seqlens = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    wl.inputs = draw_layer_inputs(shape, int(sum(seqlens)), _gen("cpu", 78), "cpu")
    wl.ckpt_pos = [[n] if n > 0 else [] for n in seqlens]
    tdt = torch.float16 if state_type == "f16" else torch.bfloat16
    init = [None if v is None else v.to(tdt).float() for v in wl.init_state]   # representable starts
    wl.init_state = init
    y_ref, st_ref = _oracle(wl, init)
    y, st, _ = _emulate(emu_binary, wl, init, tmp_path, 0, "end", advance=True, state_type=state_type)
    assert max(rel_err(y, y_ref)) <= 5e-3
    k = 0
    for b, n in enumerate(seqlens):
        if n == 0:
            want = np.zeros_like(st[b]) if init[b] is None else init[b].numpy()
            assert np.array_equal(st[b], want)
        else:
            ref = st_ref[k]
            assert np.all(np.abs(st[b] - ref) <= ulp * np.maximum(np.abs(ref), 2.0 ** -14))
            # and the stored values are values of the type
            assert np.array_equal(torch.from_numpy(st[b].copy()).to(tdt).float().numpy(), st[b])
            k += 1


def test_full_size_spot_check(tmp_path_factory):
    """The 7B-shaped 32K-token configuration (H=128, P=64, N=128, G=8, one checkpoint at the end) on the emulator:
    only the first two and the last workgroup run, on guarded buffers of the full size, and are compared with a
    plain fp64 recurrence inside the driver.  Token offsets, group indexing and the workgroup renumbering are the
    real ones."""
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with bf16 vector support found")
    d = str(tmp_path_factory.mktemp("kernel_emu_big"))
    _convert(os.path.join(CSRC, "scan_mfma.hip"), os.path.join(d, "scan_mfma.cpp"))
    flags = ["-std=c++17", "-O2", "-fno-strict-aliasing", "-ffp-contract=off", "-Wno-psabi", "-Wno-unused-value",
             "-I", EMU, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    out = os.path.join(d, "emu_big")
    r = subprocess.run([CLANG, *flags, os.path.join(d, "scan_mfma.cpp"), os.path.join(CSRC, "plan.cpp"),
                        os.path.join(EMU, "emu_rt.cpp"), os.path.join(EMU, "emu_big.cpp"), "-o", out],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([out, "32768", "32768"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "BIG CHECK OK" in r.stdout, r.stdout[-1500:] + r.stderr[-500:]


@pytest.mark.parametrize("case", sorted(CASES))
def test_emulated_4wave_scan_matches_oracle_in_any_wave_order(emu_binary_4waves, tmp_path, case):
    _check_case(emu_binary_4waves, tmp_path, "bf16", case)


@pytest.mark.parametrize("case", ["ragged", "long", "tiny", "p128", "empty_seq", "strong_decay"])
def test_emulated_64_channel_scan_matches_oracle_in_any_wave_order(emu_binary, tmp_path, case):
    """The variant of the matrix-core scan whose workgroups own 64 channels (the plan picks it for grids that fill a
    GPU; the emulation driver forces it): same checks as for the 32-channel kernel."""
    _check_case(emu_binary, tmp_path, "bf16", case, wide=True)


@pytest.mark.parametrize("split", ["2:1", "3:1", "5:2"])
@pytest.mark.parametrize("case", ["ragged", "long", "tiny", "p128", "empty_seq", "strong_decay", "heads7"])
def test_emulated_scan_of_sequences_cut_into_stretches_matches_oracle(emu_binary, tmp_path, case, split):
    """Sequences cut into stretches that are scanned at the same time, the later ones from a zero state, and the
    kernels that carry the states over and add their contribution (the plan cuts only long sequences of batches that
    would leave a GPU idle; the emulation driver forces it on small ones): same checks as for the uncut scan.  Covers
    two stretches, chains of three and more, stretches of a single tile, checkpoints and cached initial states in
    any stretch, and decay so strong that the carried state adds nothing."""
    if CASES[case][0][1] % 64:
        pytest.skip("sequences are cut only where workgroups own 64 channels")
    _check_case(emu_binary, tmp_path, "bf16", case, split=split)


@pytest.mark.parametrize("case", ["ragged", "long2"])
def test_emulated_stretches_with_coarse_groups_in_the_second_kernel(emu_binary_4waves, tmp_path, case):
    """As above, built so that only the first 8 tiles of a stretch get the second kernel's small workgroups (96 in
    the shipped build): the tiles beyond them go to the workgroups of 32 tiles, eight per wave."""
    _check_case(emu_binary_4waves, tmp_path, "bf16", case, split="2:1")


@pytest.mark.parametrize("order", [0, 1, 9])
def test_emulator_runs_workgroups_that_wait_for_each_other(tmp_path_factory, order):
    """Self-test of the emulator's cooperative mode: a relay through all workgroups of a launch, in any wave order."""
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with bf16 vector support found")
    d = str(tmp_path_factory.mktemp("kernel_emu_coop"))
    out = os.path.join(d, "coop_selftest")
    r = subprocess.run([CLANG, "-std=c++17", "-O2", "-Wno-psabi", "-I", EMU, os.path.join(EMU, "coop_selftest.cpp"),
                        os.path.join(EMU, "emu_rt.cpp"), "-o", out], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([out, str(order)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "COOP OK" in r.stdout, r.stdout + r.stderr[-500:]


def test_a_barrier_that_does_not_wait_is_noticed(emu_binary, tmp_path):
    """Self-test of the race check on the bf16 kernel.  The scan has one workgroup barrier, between the write of the
    starting state into LDS and the first hand-off; with it made not to wait, a wave reads the state before it is
    there (LDS starts as a NaN pattern) in at least one wave order."""
    shape = LayerShape(nheads=1, headdim=32, d_state=128, ngroups=1, chunk=64, io_dtype="bf16")
    wl = make_workload(4, "cpu", seed=5, shape=shape, seqlen=450, ckpt_every=200)
    g = torch.Generator().manual_seed(9)
    init = [torch.randn((1, 32, 128), generator=g)]
    ref = _emulate(emu_binary, wl, init, tmp_path, 0, "end")[2]
    # every block counts its barriers from zero: ordinal 0 is the scan's only one (and the first of the kernel in
    # front of it, whose second one publishes nothing the dropped one did not)
    outs = [_emulate(emu_binary, wl, init, tmp_path, order, "end", 0)[2] for order in (0, 1, 5)]
    assert not all(np.array_equal(o, ref) for o in outs)
