"""Seeded synthetic SSM-layer prefill workloads.

The five named configurations stand in for the hybrid-model serving workloads
of the paper's evaluation (Section 5.1: chat traces whose requests are mostly
under 2K or 10K tokens, agent traces that reach tens of thousands of tokens,
SSM state dimension 128; Section 4.1: at most two state checkpoints per
request under judicious admission, one per token block under fine-grained
checkpointing).  The traces and model weights themselves are not available, so
tensors are drawn from fixed distributions with the same shapes and lengths.

Only random draws and storage-dtype rounding happen here.  Every tensor is a
torch tensor on the requested device; bf16 tensors are rounded once
(round-to-nearest-even), so all consumers see the same bits.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch


@dataclass(frozen=True)
class LayerShape:
    nheads: int
    headdim: int
    d_state: int
    ngroups: int
    chunk: int
    io_dtype: str  # "f32" or "bf16": storage type of x, dt, B, C and y

    @property
    def torch_io_dtype(self) -> torch.dtype:
        return torch.float32 if self.io_dtype == "f32" else torch.bfloat16

    @property
    def state_elems(self) -> int:
        return self.nheads * self.headdim * self.d_state


@dataclass
class LayerInputs:
    """Per-token tensors of one packed batch (T tokens in total)."""
    x: torch.Tensor    # [T, H, P] io dtype
    dt: torch.Tensor   # [T, H]    io dtype, positive
    B: torch.Tensor    # [T, G, N] io dtype
    C: torch.Tensor    # [T, G, N] io dtype


@dataclass
class Workload:
    name: str
    shape: LayerShape
    seqlens: List[int]
    cu_seqlens: np.ndarray            # int32 [batch+1]
    inputs: LayerInputs
    A: torch.Tensor                   # [H] fp32, negative
    D: torch.Tensor                   # [H] fp32
    ckpt_pos: List[List[int]]         # per sequence: ascending token counts p, 1 <= p <= len
    # Per sequence: "zeros", "random" (init_state[i] holds an fp32 [H,P,N]
    # tensor) or "prefix" (the state after scanning `prefix` from zero; the
    # caller computes it with whichever implementation it is testing).
    init_kind: List[str]
    init_state: List[Optional[torch.Tensor]]
    prefix: Optional[LayerInputs] = None
    prefix_len: int = 0
    seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def batch(self) -> int:
        return len(self.seqlens)

    @property
    def n_ckpt(self) -> int:
        return sum(len(c) for c in self.ckpt_pos)

    def cu_ckpt(self) -> np.ndarray:
        out = np.zeros(self.batch + 1, dtype=np.int32)
        for i, c in enumerate(self.ckpt_pos):
            out[i + 1] = out[i] + len(c)
        return out

    def ckpt_flat(self) -> np.ndarray:
        flat = [p for c in self.ckpt_pos for p in c]
        return np.asarray(flat, dtype=np.int32)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def draw_layer_inputs(shape: LayerShape, T: int, g: torch.Generator, device) -> LayerInputs:
    """x ~ N(0,1); dt = exp(U(ln 1e-3, ln 1e-1)); B, C ~ N(0,1)/sqrt(N)."""
    H, P, N, G = shape.nheads, shape.headdim, shape.d_state, shape.ngroups
    io = shape.torch_io_dtype
    x = torch.randn((T, H, P), generator=g, device=device, dtype=torch.float32).to(io)
    lo, hi = math.log(1e-3), math.log(1e-1)
    u = torch.rand((T, H), generator=g, device=device, dtype=torch.float32)
    dt = torch.exp(lo + (hi - lo) * u).to(io)
    s = 1.0 / math.sqrt(N)
    B = (torch.randn((T, G, N), generator=g, device=device, dtype=torch.float32) * s).to(io)
    C = (torch.randn((T, G, N), generator=g, device=device, dtype=torch.float32) * s).to(io)
    return LayerInputs(x=x, dt=dt, B=B, C=C)


def draw_layer_params(shape: LayerShape, g: torch.Generator, device):
    """A = -exp(U(ln 1, ln 16)) per head; D ~ N(0,1) per head; both fp32."""
    H = shape.nheads
    u = torch.rand((H,), generator=g, device=device, dtype=torch.float32)
    A = -torch.exp(math.log(16.0) * u)
    D = torch.randn((H,), generator=g, device=device, dtype=torch.float32)
    return A, D


# name, layer shape, and the request mix of each configuration
CONFIGS = {
    0: dict(name="cfg0_tiny_f32",
            shape=LayerShape(4, 16, 16, 1, 64, "f32")),
    1: dict(name="cfg1_2p7b_2k_bf16",
            shape=LayerShape(80, 64, 128, 1, 256, "bf16")),
    2: dict(name="cfg2_varlen16_bf16",
            shape=LayerShape(80, 64, 128, 1, 256, "bf16")),
    3: dict(name="cfg3_7b_32k_bf16",
            shape=LayerShape(128, 64, 128, 8, 256, "bf16")),
    4: dict(name="cfg4_7b_128k_ckpt4096_bf16",
            shape=LayerShape(128, 64, 128, 8, 256, "bf16")),
}


def make_workload(cfg: int, device="cpu", seed: Optional[int] = None, *,
                  seqlen: Optional[int] = None, prefix_len: Optional[int] = None,
                  batch: Optional[int] = None, len_range=None,
                  ckpt_every: Optional[int] = None,
                  shape: Optional[LayerShape] = None) -> Workload:
    """Build configuration `cfg` (0..4).  The keyword overrides shrink a
    configuration for tests that need the CPU oracle to finish quickly; with
    none given the sizes are the full ones."""
    spec = CONFIGS[cfg]
    shape = shape or spec["shape"]
    seed = cfg if seed is None else seed
    g = _gen(device, seed)
    A, D = draw_layer_params(shape, g, device)
    notes = {}
    prefix = None
    plen = 0

    if cfg == 0:
        T = seqlen or 256
        seqlens = [T]
        ckpts = [[T // 2, T]]
        kinds = ["zeros"]
    elif cfg == 1:
        T = seqlen or 2048
        plen = 1024 if prefix_len is None else prefix_len
        seqlens = [T]
        ckpts = [[T]]
        kinds = ["prefix"]
    elif cfg == 2:
        nb = batch or 16
        lo, hi = len_range or (512, 8192)
        rs = np.random.RandomState(1000 + seed)
        seqlens = [int(v) for v in rs.randint(lo, hi + 1, size=nb)]
        ckpts = []
        for L in seqlens:
            mid = int(rs.randint(1, L)) if L > 1 else None  # U{1..L-1}, not chunk aligned
            ckpts.append(([mid] if mid is not None else []) + [L])
        perm = rs.permutation(nb)
        kinds = ["zeros"] * nb
        for i in perm[: nb // 2]:
            kinds[int(i)] = "random"
    elif cfg == 3:
        T = seqlen or 32768
        plen = 16384 if prefix_len is None else prefix_len
        seqlens = [T]
        ckpts = [[T]]
        kinds = ["prefix"]
    elif cfg == 4:
        T = seqlen or 131072
        every = ckpt_every or 4096
        seqlens = [T]
        ckpts = [list(range(every, T + 1, every))]
        kinds = ["zeros"]
        notes["ckpt_every"] = every
    else:
        raise KeyError(cfg)

    total = sum(seqlens)
    inputs = draw_layer_inputs(shape, total, g, device)
    init_state: List[Optional[torch.Tensor]] = []
    for k in kinds:
        if k == "random":
            init_state.append(torch.randn((shape.nheads, shape.headdim, shape.d_state),
                                          generator=g, device=device, dtype=torch.float32))
        else:
            init_state.append(None)
    if plen > 0:
        gp = _gen(device, 7919 + seed)  # the prefix has a random stream of its own
        prefix = draw_layer_inputs(shape, plen, gp, device)

    cu = np.zeros(len(seqlens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seqlens)
    return Workload(name=spec["name"], shape=shape, seqlens=seqlens, cu_seqlens=cu,
                    inputs=inputs, A=A, D=D, ckpt_pos=ckpts, init_kind=kinds,
                    init_state=init_state, prefix=prefix, prefix_len=plen,
                    seed=seed, notes=notes)
