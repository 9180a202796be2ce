"""ctypes binding of the C ABI in include/ssm_prefill.h.

Argument marshalling only: every step of the scan runs in the HIP kernels.
There is no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libssm_prefill.so")
_lib = None

SSM_DT_F32, SSM_DT_BF16 = 0, 1
SSM_ST_F32, SSM_ST_F16, SSM_ST_BF16 = 0, 1, 2
_STATE_DTYPES = {"f32": SSM_ST_F32, "f16": SSM_ST_F16, "bf16": SSM_ST_BF16}
SSM_PATH_VALU_F32, SSM_PATH_MFMA_BF16 = 0, 1

SSM_ERR_UNSUPPORTED_SHAPE = -4

_STATUS = {0: "SSM_OK", -1: "SSM_ERR_INVALID_ARG", -2: "SSM_ERR_BAD_CU_SEQLENS",
           -3: "SSM_ERR_BAD_CHECKPOINT", -4: "SSM_ERR_UNSUPPORTED_SHAPE",
           -5: "SSM_ERR_WORKSPACE_TOO_SMALL", -6: "SSM_ERR_MISALIGNED", -7: "SSM_ERR_HIP"}


class SsmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code
        self.status = _STATUS.get(code, str(code))


class SsmShape(ctypes.Structure):
    _fields_ = [("nheads", ctypes.c_int32), ("headdim", ctypes.c_int32),
                ("d_state", ctypes.c_int32), ("ngroups", ctypes.c_int32),
                ("chunk", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("state_dtype", ctypes.c_int32)]


class SsmPlanInfo(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_ckpt", ctypes.c_int32),
                ("total_tokens", ctypes.c_int64), ("n_tiles", ctypes.c_int32),
                ("tile_tokens", ctypes.c_int32), ("path", ctypes.c_int32),
                ("n_workgroups", ctypes.c_int32), ("n_stretches", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libssm_prefill.so (built by `python -m paper_2411_19379_amd.build`
    or `__graft_entry__.build()`); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch owns device memory and streams here, so its HIP runtime must be
    # the one this library binds to: load torch's copy first.
    import torch  # noqa: F401

    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is not built; run `python paper_2411_19379_amd/build.py` first")
    lib = ctypes.CDLL(_LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    vp = ctypes.c_void_p
    lib.ssm_plan_create.restype = ctypes.c_int
    lib.ssm_plan_create.argtypes = [ctypes.POINTER(SsmShape), ctypes.c_int32, i32p, i32p, i32p,
                                    ctypes.POINTER(vp)]
    lib.ssm_plan_info.restype = ctypes.c_int
    lib.ssm_plan_info.argtypes = [vp, ctypes.POINTER(SsmPlanInfo)]
    lib.ssm_plan_launch_order.restype = ctypes.c_int
    lib.ssm_plan_launch_order.argtypes = [vp, i32p, i32p, i32p, ctypes.POINTER(ctypes.c_int64)]
    lib.ssm_plan_launch_item.restype = ctypes.c_int
    lib.ssm_plan_launch_item.argtypes = [vp, ctypes.c_int64, i32p]
    lib.ssm_plan_stretch.restype = ctypes.c_int
    lib.ssm_plan_stretch.argtypes = [vp, ctypes.c_int32, i32p, i32p, i32p]
    lib.ssm_plan_tile.restype = ctypes.c_int
    lib.ssm_plan_tile.argtypes = [vp, ctypes.c_int32, i32p, i32p, i32p, i32p]
    lib.ssm_plan_workspace_bytes.restype = ctypes.c_int
    lib.ssm_plan_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
    lib.ssm_prefill.restype = ctypes.c_int
    lib.ssm_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp), vp, vp, vp,
                                ctypes.c_size_t, vp]
    lib.ssm_prefill_noalloc.restype = ctypes.c_int
    lib.ssm_prefill_noalloc.argtypes = lib.ssm_prefill.argtypes
    lib.ssm_state_advance.restype = ctypes.c_int
    lib.ssm_state_advance.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp), vp, vp]
    lib.ssm_conv1d_prefill.restype = ctypes.c_int
    lib.ssm_conv1d_prefill.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, ctypes.POINTER(vp), vp, vp,
                                       ctypes.c_int32, vp]
    lib.ssm_profile_mark.restype = None
    lib.ssm_profile_mark.argtypes = [vp, vp]
    lib.ssm_plan_destroy.restype = None
    lib.ssm_plan_destroy.argtypes = [vp]
    lib.ssm_last_error.restype = ctypes.c_char_p
    lib.ssm_last_error.argtypes = []
    _lib = lib
    return lib


def ssm_last_error() -> str:
    return load_library().ssm_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise SsmError(rc, ssm_last_error())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def ssm_plan_create(shape: SsmShape, cu_seqlens, cu_ckpt=None, ckpt_pos=None) -> int:
    """Returns the opaque plan handle (an integer address)."""
    lib = load_library()
    i32p = ctypes.POINTER(ctypes.c_int32)
    cu = _i32(cu_seqlens)
    batch = cu.shape[0] - 1
    cu_ck = _i32(cu_ckpt) if cu_ckpt is not None else None
    pos = _i32(ckpt_pos) if ckpt_pos is not None and len(ckpt_pos) else None
    out = ctypes.c_void_p()
    rc = lib.ssm_plan_create(ctypes.byref(shape), batch, cu.ctypes.data_as(i32p),
                             cu_ck.ctypes.data_as(i32p) if cu_ck is not None else None,
                             pos.ctypes.data_as(i32p) if pos is not None else None,
                             ctypes.byref(out))
    _check(rc)
    return out.value


def ssm_plan_info(plan: int) -> SsmPlanInfo:
    info = SsmPlanInfo()
    _check(load_library().ssm_plan_info(plan, ctypes.byref(info)))
    return info


def ssm_plan_tile(plan: int, i: int):
    v = [ctypes.c_int32() for _ in range(4)]
    _check(load_library().ssm_plan_tile(plan, i, *[ctypes.byref(c) for c in v]))
    return tuple(c.value for c in v)  # tok0, len, seq, ckpt_slot


def ssm_plan_stretch(plan: int, i: int):
    v = [ctypes.c_int32() for _ in range(3)]
    _check(load_library().ssm_plan_stretch(plan, i, *[ctypes.byref(c) for c in v]))
    return v[0].value, v[1].value, bool(v[2].value)  # tile_begin, tile_end, starts_from_zero


def ssm_plan_launch_order(plan: int, batch: int):
    by_length = (ctypes.c_int32 * max(batch, 1))()
    slices, n_items, n_blocks = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
    _check(load_library().ssm_plan_launch_order(plan, by_length, ctypes.byref(slices), ctypes.byref(n_items),
                                                ctypes.byref(n_blocks)))
    return list(by_length)[:batch], slices.value, n_items.value, n_blocks.value


def ssm_plan_launch_item(plan: int, block: int) -> int:
    item = ctypes.c_int32()
    _check(load_library().ssm_plan_launch_item(plan, block, ctypes.byref(item)))
    return item.value


def ssm_plan_workspace_bytes(plan: int) -> int:
    n = ctypes.c_size_t()
    _check(load_library().ssm_plan_workspace_bytes(plan, ctypes.byref(n)))
    return n.value


def ssm_profile_mark(after_first: Optional[int], after_second: Optional[int] = None):
    """Have later prefill calls of this thread record the given raw hipEvent_t handles (e.g.
    torch.cuda.Event(...).cuda_event after a first record) after their first and after their second kernel;
    None switches an event off."""
    load_library().ssm_profile_mark(ctypes.c_void_p(after_first) if after_first else None,
                                    ctypes.c_void_p(after_second) if after_second else None)


def ssm_plan_destroy(plan: Optional[int]):
    if plan:
        load_library().ssm_plan_destroy(plan)


def _ptr_array(plan: int, ptrs):
    """Host array of device addresses, one per sequence of the plan (the C side reads exactly `batch` entries)."""
    if ptrs is None:
        return None
    batch = ssm_plan_info(plan).batch
    if len(ptrs) != batch:
        raise ValueError(f"expected one state pointer per sequence ({batch}), got {len(ptrs)}")
    arr = (ctypes.c_void_p * max(batch, 1))()
    for i, p in enumerate(ptrs):
        arr[i] = p if p else None
    return arr


def ssm_prefill(plan: int, x: int, dt: int, A: int, B: int, C: int, D: int,
                init_state_ptrs: Optional[Sequence[Optional[int]]], y_out: int, state_out: Optional[int],
                workspace: Optional[int], workspace_bytes: int, hip_stream: Optional[int]):
    """Raw call: every tensor argument is a device address (int)."""
    _check(load_library().ssm_prefill(plan, x, dt, A, B, C, D, _ptr_array(plan, init_state_ptrs), y_out, state_out,
                                      workspace, workspace_bytes, hip_stream))


def ssm_prefill_noalloc(plan: int, x: int, dt: int, A: int, B: int, C: int, D: int,
                        init_state_ptrs: Optional[Sequence[Optional[int]]], y_out: int, state_out: Optional[int],
                        workspace: Optional[int], workspace_bytes: int, hip_stream: Optional[int]):
    """Raw call of the entry point that allocates nothing; arguments as ssm_prefill."""
    _check(load_library().ssm_prefill_noalloc(plan, x, dt, A, B, C, D, _ptr_array(plan, init_state_ptrs), y_out,
                                              state_out, workspace, workspace_bytes, hip_stream))


def ssm_state_advance(plan: int, x: int, dt: int, A: int, B: int, C: int, D: int,
                      state_ptrs: Sequence[Optional[int]], y_out: Optional[int], hip_stream: Optional[int]):
    """Raw call: advance every sequence's [H,P,N] state (in the plan's state dtype) in place."""
    _check(load_library().ssm_state_advance(plan, x, dt, A, B, C, D, _ptr_array(plan, state_ptrs), y_out,
                                            hip_stream))


def ssm_conv1d_prefill(plan: int, channels: int, kernel_width: int, xin: int, weight: int, bias: Optional[int],
                       init_state_ptrs: Optional[Sequence[Optional[int]]], out: int, state_out: Optional[int],
                       activation: int, hip_stream: Optional[int]):
    """Raw call of the causal convolution with cached-state resume; tensor arguments are device addresses."""
    _check(load_library().ssm_conv1d_prefill(plan, channels, kernel_width, xin, weight, bias,
                                             _ptr_array(plan, init_state_ptrs), out, state_out, activation,
                                             hip_stream))


class Plan:
    """Owns an ssm_plan_t for one packed batch."""

    def __init__(self, nheads: int, headdim: int, d_state: int, ngroups: int, chunk: int,
                 io_dtype: str, cu_seqlens, ckpt_pos: Optional[List[List[int]]] = None,
                 state_dtype: str = "f32"):
        self.shape = SsmShape(nheads, headdim, d_state, ngroups, chunk,
                              SSM_DT_F32 if io_dtype == "f32" else SSM_DT_BF16, _STATE_DTYPES[state_dtype])
        self._workspace = {}
        cu = _i32(cu_seqlens)
        batch = cu.shape[0] - 1
        cu_ck = flat = None
        if ckpt_pos is not None:
            assert len(ckpt_pos) == batch
            cu_ck = np.zeros(batch + 1, dtype=np.int32)
            for i, c in enumerate(ckpt_pos):
                cu_ck[i + 1] = cu_ck[i] + len(c)
            flat = [p for c in ckpt_pos for p in c]
        self.handle = ssm_plan_create(self.shape, cu, cu_ck, flat)
        self.info = ssm_plan_info(self.handle)

    def tiles(self):
        return [ssm_plan_tile(self.handle, i) for i in range(self.info.n_tiles)]

    def launch_order(self):
        return ssm_plan_launch_order(self.handle, self.info.n_stretches)

    def stretches(self):
        return [ssm_plan_stretch(self.handle, i) for i in range(self.info.n_stretches)]

    def workspace(self, device):
        """The plan's device workspace as a torch tensor (allocated once per device, reused by every call)."""
        import torch

        key = str(device)
        if key not in self._workspace:
            n = ssm_plan_workspace_bytes(self.handle)
            self._workspace[key] = torch.empty((n,), dtype=torch.uint8, device=device) if n else None
        return self._workspace[key]

    def close(self):
        if getattr(self, "handle", None):
            ssm_plan_destroy(self.handle)
            self.handle = None
            self._workspace = {}

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _state_torch_dtype(shape):
    import torch

    return {SSM_ST_F32: torch.float32, SSM_ST_F16: torch.float16, SSM_ST_BF16: torch.bfloat16}[shape.state_dtype]


def prefill(plan: Plan, x, dt, A, B, C, D, init_states=None, y_out=None, state_out=None,
            stream=None, entry=None):
    """Scan one layer on torch CUDA tensors.  Allocates y/state_out with torch
    if not given; returns (y, state_out).  `init_states` is None or a list
    with one [H,P,N] CUDA tensor (in the plan's state dtype) or None per
    sequence.  `entry` selects the raw entry point (default ssm_prefill)."""
    import torch

    s = plan.shape
    io = torch.float32 if s.io_dtype == SSM_DT_F32 else torch.bfloat16
    sdt = _state_torch_dtype(s)
    T = int(plan.info.total_tokens)
    for name, t, shp, dty in (("x", x, (T, s.nheads, s.headdim), io), ("dt", dt, (T, s.nheads), io),
                              ("A", A, (s.nheads,), torch.float32),
                              ("B", B, (T, s.ngroups, s.d_state), io),
                              ("C", C, (T, s.ngroups, s.d_state), io),
                              ("D", D, (s.nheads,), torch.float32)):
        if not t.is_cuda or tuple(t.shape) != shp or t.dtype != dty or not t.is_contiguous():
            raise ValueError(f"{name}: expected contiguous CUDA {dty} tensor of shape {shp}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")
    dev = x.device
    if y_out is None:
        y_out = torch.empty((T, s.nheads, s.headdim), dtype=io, device=dev)
    n_ckpt = int(plan.info.n_ckpt)
    if state_out is None and n_ckpt:
        state_out = torch.empty((n_ckpt, s.nheads, s.headdim, s.d_state), dtype=sdt, device=dev)
    ptrs = None
    if init_states is not None:
        if len(init_states) != int(plan.info.batch):
            raise ValueError(f"init_states needs one entry per sequence ({plan.info.batch}), got {len(init_states)}")
        ptrs = []
        for st in init_states:
            if st is None:
                ptrs.append(None)
            else:
                if (not st.is_cuda or st.dtype != sdt or not st.is_contiguous()
                        or tuple(st.shape) != (s.nheads, s.headdim, s.d_state)):
                    raise ValueError(f"initial states must be contiguous {sdt} CUDA [H,P,N] tensors")
                ptrs.append(st.data_ptr())
    ws = plan.workspace(dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    (entry or ssm_prefill)(plan.handle, x.data_ptr(), dt.data_ptr(), A.data_ptr(), B.data_ptr(), C.data_ptr(),
                           D.data_ptr(), ptrs, y_out.data_ptr(),
                           state_out.data_ptr() if state_out is not None else None,
                           ws.data_ptr() if ws is not None else None, ws.numel() if ws is not None else 0, stream)
    return y_out, state_out
