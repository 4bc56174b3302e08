"""Thin Python binding of the C-ABI library (include/lobra_mlora.h): argument marshalling only.

Tensors are PyTorch-ROCm tensors used for device memory and streams; every step of the layer
runs in the library's HIP kernels.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LOBRA_MLORA_LIB points at another build of the same library (kernel tuning variants).
LIB_PATH = os.environ.get("LOBRA_MLORA_LIB") or os.path.join(_HERE, "liblobra_mlora.so")

OK = 0
F32, BF16 = 0, 1
FLAG_ACCUMULATE_GRADS, FLAG_NO_DX = 1, 2
PLAN_HOST_ONLY, PLAN_PLAIN_KERNELS = 1, 2
Q_SEGMENTS, Q_ROWBLOCK_SEG, Q_TOKEN_BLOCKS, Q_GRAD_CHUNKS, Q_TASK_CHUNKS, Q_BLOCK_RUNS = 0, 1, 2, 3, 4, 5
Q_BLOCK_ORDER, Q_RUN_ORDER = 6, 7
Q_SLICED, Q_FUSED_WG_RUNS, Q_FUSED_RUN_ROW, Q_FUSED_COUNT, Q_FUSED_TASK_ROW = 8, 9, 10, 11, 12
Q_GEMM_TILE_ROWS = 13
MAX_RANK = 128

EXPORTS = [
    "lobra_mlora_validate", "lobra_mlora_workspace_bytes", "lobra_mlora_fwd", "lobra_mlora_bwd", "lobra_token_task_map",
    "lobra_mlora_plan_create", "lobra_mlora_plan_device_bytes", "lobra_mlora_plan_init", "lobra_mlora_plan_destroy",
    "lobra_mlora_plan_sizes", "lobra_mlora_plan_query", "lobra_mlora_plan_fwd", "lobra_mlora_plan_bwd",
    "lobra_mlora_plan_token_task_map", "lobra_mlora_fwd_static_ws", "lobra_mlora_adam_step", "lobra_dynamic_buckets",
    "lobra_padded_segments",
    "lobra_mlora_plan_set_trace", "lobra_status_string", "lobra_version",
]


class Desc(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32),
        ("T", ctypes.c_int64), ("n_tasks", ctypes.c_int32), ("S", ctypes.c_int32),
        ("rank_off", ctypes.POINTER(ctypes.c_int32)),
        ("seg_off", ctypes.POINTER(ctypes.c_int32)),
        ("seg_task", ctypes.POINTER(ctypes.c_int32)),
        ("n_proj", ctypes.c_int32),
    ]


class AdamConfig(ctypes.Structure):
    _fields_ = [("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float)]


class LobraError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


_lib = None


def lib():
    """The loaded library.  Build it first with ``python -m paper_2509_01193_amd.build``."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                LIB_PATH + " is missing: build it with `python -m paper_2509_01193_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_size_t
        szp = ctypes.POINTER(sz)
        L.lobra_mlora_validate.restype = ctypes.c_int
        L.lobra_mlora_validate.argtypes = [ctypes.POINTER(Desc)]
        L.lobra_mlora_plan_create.restype = ctypes.c_int
        L.lobra_mlora_plan_create.argtypes = [ctypes.POINTER(Desc), u32, ctypes.POINTER(vp)]
        L.lobra_mlora_plan_destroy.restype = ctypes.c_int
        L.lobra_mlora_plan_destroy.argtypes = [vp]
        L.lobra_mlora_plan_sizes.restype = ctypes.c_int
        L.lobra_mlora_plan_sizes.argtypes = [vp, szp, szp, szp]
        L.lobra_mlora_plan_query.restype = ctypes.c_int
        L.lobra_mlora_plan_query.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), sz, szp]
        for name in ("lobra_mlora_plan_fwd", "lobra_mlora_fwd"):      # (plan | desc, x, W, A, B, s, y, h_save, ws, bytes, stream)
            getattr(L, name).restype = ctypes.c_int
        L.lobra_mlora_plan_fwd.argtypes = [vp] * 8 + [vp, sz, vp]
        L.lobra_mlora_fwd.argtypes = [ctypes.POINTER(Desc)] + [vp] * 7 + [vp, sz, vp]
        L.lobra_mlora_fwd_static_ws.restype = ctypes.c_int
        L.lobra_mlora_fwd_static_ws.argtypes = [vp] * 7 + [vp]
        L.lobra_mlora_plan_bwd.restype = L.lobra_mlora_bwd.restype = ctypes.c_int
        L.lobra_mlora_plan_bwd.argtypes = [vp] * 11 + [u32, vp, sz, vp]
        L.lobra_mlora_bwd.argtypes = [ctypes.POINTER(Desc)] + [vp] * 10 + [u32, vp, sz, vp]
        L.lobra_mlora_plan_token_task_map.restype = L.lobra_token_task_map.restype = ctypes.c_int
        L.lobra_mlora_plan_token_task_map.argtypes = [vp, vp, vp, vp]
        L.lobra_token_task_map.argtypes = [ctypes.POINTER(Desc), vp, vp, vp]
        L.lobra_mlora_workspace_bytes.restype = ctypes.c_int
        L.lobra_mlora_workspace_bytes.argtypes = [ctypes.POINTER(Desc), szp, szp]
        L.lobra_mlora_plan_device_bytes.restype = ctypes.c_int
        L.lobra_mlora_plan_device_bytes.argtypes = [ctypes.POINTER(Desc), u32, szp]
        L.lobra_mlora_plan_init.restype = ctypes.c_int
        L.lobra_mlora_plan_init.argtypes = [ctypes.POINTER(Desc), u32, vp, sz, vp, ctypes.POINTER(vp)]
        L.lobra_mlora_adam_step.restype = ctypes.c_int
        L.lobra_mlora_adam_step.argtypes = [vp, ctypes.POINTER(AdamConfig)] + [vp] * 13 + [vp]
        L.lobra_status_string.restype = ctypes.c_char_p
        L.lobra_status_string.argtypes = [ctypes.c_int]
        L.lobra_version.restype = ctypes.c_int
        L.lobra_version.argtypes = []
        _lib = L
    return _lib


def status_string(st) -> str:
    return lib().lobra_status_string(int(st)).decode()


def version() -> int:
    return lib().lobra_version()


def _check(st, where):
    if st != OK:
        raise LobraError(st, where)


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def make_desc(dtype, T, d_in, d_out, rank_off, seg_off, seg_task, n_proj=1):
    """Returns (Desc, keepalive).  `dtype` is "f32"/"bf16" or the enum value."""
    code = {"f32": F32, "bf16": BF16}.get(dtype, dtype)
    keep = []
    d = Desc()
    d.dtype, d.d_in, d.d_out, d.T = int(code), int(d_in), int(d_out), int(T)
    n_tasks = 0
    if rank_off is not None:
        ro = _i32(rank_off)
        keep.append(ro)
        n_tasks = max(int(ro.shape[0]) - 1, 0)
        d.rank_off = ro.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    d.n_tasks = n_tasks
    S = 0
    if seg_task is not None:
        so, stk = _i32(seg_off), _i32(seg_task)
        keep += [so, stk]
        S = int(stk.shape[0])
        d.seg_off = so.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
        d.seg_task = stk.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    d.S = S
    d.n_proj = int(n_proj)
    return d, keep


def validate(desc: Desc) -> int:
    return lib().lobra_mlora_validate(ctypes.byref(desc))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    assert t.is_contiguous(), "tensors must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(int(getattr(stream, "cuda_stream", stream)))


class Plan:
    """Owns a ``lobra_mlora_plan``.  One plan per packed batch, shared by every layer's calls."""

    def __init__(self, dtype, T, d_in, d_out, rank_off, seg_off, seg_task, flags=0, n_proj=1, device_mem=None,
                 stream=None):
        """device_mem (a device uint8 tensor of at least plan_device_bytes(...)): lobra_mlora_plan_init places
        the plan there with an asynchronous copy on `stream`; None: lobra_mlora_plan_create allocates."""
        self.desc, self._keep = make_desc(dtype, T, d_in, d_out, rank_off, seg_off, seg_task, n_proj)
        self.handle = ctypes.c_void_p()
        if device_mem is None:
            _check(lib().lobra_mlora_plan_create(ctypes.byref(self.desc), int(flags),
                                                 ctypes.byref(self.handle)), "lobra_mlora_plan_create")
        else:
            self._keep.append(device_mem)
            _check(lib().lobra_mlora_plan_init(ctypes.byref(self.desc), int(flags), _ptr(device_mem),
                                               device_mem.numel() * device_mem.element_size(), _stream(stream),
                                               ctypes.byref(self.handle)), "lobra_mlora_plan_init")
        a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
        _check(lib().lobra_mlora_plan_sizes(self.handle, ctypes.byref(a), ctypes.byref(b),
                                            ctypes.byref(c)), "lobra_mlora_plan_sizes")
        self.h_save_bytes, self.fwd_ws_bytes, self.bwd_ws_bytes = a.value, b.value, c.value
        self.T, self.d_in, self.d_out = int(T), int(d_in), int(d_out)
        self.n_tasks = self.desc.n_tasks
        self.R_tot = int(np.asarray(rank_off)[-1]) if self.n_tasks > 0 else 0

    @classmethod
    def for_problem(cls, p, flags=0):
        return cls(p.dtype, p.T, p.d_in, p.d_out, p.rank_off, p.seg_off, p.seg_task, flags,
                   getattr(p, "n_proj", 1))

    def query(self, what) -> np.ndarray:
        n = ctypes.c_size_t()
        _check(lib().lobra_mlora_plan_query(self.handle, int(what), None, 0, ctypes.byref(n)),
               "lobra_mlora_plan_query")
        out = np.zeros(max(n.value, 1), dtype=np.int32)
        _check(lib().lobra_mlora_plan_query(
            self.handle, int(what), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
            n.value, ctypes.byref(n)), "lobra_mlora_plan_query")
        return out[: n.value]

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle.value:
            lib().lobra_mlora_plan_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_device_bytes(desc: Desc, flags=0) -> int:
    n = ctypes.c_size_t()
    _check(lib().lobra_mlora_plan_device_bytes(ctypes.byref(desc), int(flags), ctypes.byref(n)),
           "lobra_mlora_plan_device_bytes")
    return n.value


def lobra_mlora_workspace_bytes(desc: Desc):
    """(fwd bytes, bwd bytes) of workspace the one-shot calls need for this descriptor."""
    a, b = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().lobra_mlora_workspace_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b)),
           "lobra_mlora_workspace_bytes")
    return a.value, b.value


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def lobra_mlora_fwd(desc: Desc, x, W, A, B, s, y, h_save=None, ws=None, stream=None, check=True):
    """One-shot forward on a descriptor (no plan object).  Returns the status."""
    st = lib().lobra_mlora_fwd(ctypes.byref(desc), _ptr(x), _ptr(W), _ptr(A), _ptr(B), _ptr(s), _ptr(y),
                               _ptr(h_save), _ptr(ws), _nbytes(ws), _stream(stream))
    if check:
        _check(st, "lobra_mlora_fwd")
    return st


def lobra_mlora_bwd(desc: Desc, x, W, A, B, s, dy, h_saved, dx, dA, dB, flags=0, ws=None, stream=None, check=True):
    """One-shot backward on a descriptor.  Returns the status."""
    st = lib().lobra_mlora_bwd(ctypes.byref(desc), _ptr(x), _ptr(W), _ptr(A), _ptr(B), _ptr(s), _ptr(dy),
                               _ptr(h_saved), _ptr(dx), _ptr(dA), _ptr(dB), int(flags), _ptr(ws), _nbytes(ws),
                               _stream(stream))
    if check:
        _check(st, "lobra_mlora_bwd")
    return st


def lobra_token_task_map(desc: Desc, out_task, out_count, stream=None, check=True):
    st = lib().lobra_token_task_map(ctypes.byref(desc), _ptr(out_task), _ptr(out_count), _stream(stream))
    if check:
        _check(st, "lobra_token_task_map")
    return st


def lobra_mlora_plan_fwd(plan: Plan, x, W, A, B, s, y, h_save=None, ws=None, stream=None, check=True):
    """y = x W + s_t (A_t x) B_t.  Tensors are device tensors; returns the status."""
    st = lib().lobra_mlora_plan_fwd(plan.handle, _ptr(x), _ptr(W), _ptr(A), _ptr(B), _ptr(s), _ptr(y),
                               _ptr(h_save), _ptr(ws),
                               0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    if check:
        _check(st, "lobra_mlora_plan_fwd")
    return st


STATIC_WS_BYTES = 16 * 1024 * 1024


def lobra_mlora_fwd_static_ws(plan: Plan, x, W, A, B, s, y, stream=None, check=True):
    """lobra_mlora_fwd with the library's own static scratch array (no allocation anywhere)."""
    st = lib().lobra_mlora_fwd_static_ws(plan.handle, _ptr(x), _ptr(W), _ptr(A), _ptr(B), _ptr(s), _ptr(y),
                                         _stream(stream))
    if check:
        _check(st, "lobra_mlora_fwd_static_ws")
    return st


def lobra_mlora_plan_bwd(plan: Plan, x, W, A, B, s, dy, h_saved, dx, dA, dB, flags=0, ws=None,
                         stream=None, check=True):
    """dx, dA, dB of the layer.  Returns the status."""
    st = lib().lobra_mlora_plan_bwd(plan.handle, _ptr(x), _ptr(W), _ptr(A), _ptr(B), _ptr(s), _ptr(dy),
                               _ptr(h_saved), _ptr(dx), _ptr(dA), _ptr(dB), int(flags), _ptr(ws),
                               0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    if check:
        _check(st, "lobra_mlora_plan_bwd")
    return st


def lobra_mlora_adam_step(plan: Plan, cfg: AdamConfig, lr, step, grad_scale, dA, dB, master_A, master_B,
                          m_A, v_A, m_B, v_B, A=None, B=None, stream=None, check=True):
    """Fused Adam over all tasks' adapters (device tensors, updated in place). Returns the status."""
    st = lib().lobra_mlora_adam_step(plan.handle, ctypes.byref(cfg), _ptr(lr), _ptr(step), _ptr(grad_scale),
                                     _ptr(dA), _ptr(dB), _ptr(master_A), _ptr(master_B), _ptr(m_A),
                                     _ptr(v_A), _ptr(m_B), _ptr(v_B), _ptr(A), _ptr(B), _stream(stream))
    if check:
        _check(st, "lobra_mlora_adam_step")
    return st


def lobra_dynamic_buckets(seq_len, bounds, R):
    """Host-side dynamic bucketing: returns (chosen boundaries ascending, total pad tokens)."""
    L = lib()
    L.lobra_dynamic_buckets.restype = ctypes.c_int
    i32p = ctypes.POINTER(ctypes.c_int32)
    L.lobra_dynamic_buckets.argtypes = [i32p, ctypes.c_int64, i32p, ctypes.c_int32, ctypes.c_int32, i32p, i32p,
                                        ctypes.POINTER(ctypes.c_int64)]
    sl, bo = _i32(seq_len), _i32(bounds)
    out = np.zeros(max(int(R), 1), np.int32)
    n, pad = ctypes.c_int32(), ctypes.c_int64()
    _check(L.lobra_dynamic_buckets(sl.ctypes.data_as(i32p), int(sl.shape[0]), bo.ctypes.data_as(i32p),
                                   int(bo.shape[0]), int(R), out.ctypes.data_as(i32p), ctypes.byref(n),
                                   ctypes.byref(pad)), "lobra_dynamic_buckets")
    return out[: n.value].tolist(), int(pad.value)


def lobra_padded_segments(valid_len, task, n_tasks, padded_len=None, uniform_len=0, check=True):
    """Segment table (seg_off, seg_task) and token count of a padded chunk; returns (status, ...) when check=False."""
    L = lib()
    i32p = ctypes.POINTER(ctypes.c_int32)
    L.lobra_padded_segments.restype = ctypes.c_int
    L.lobra_padded_segments.argtypes = [ctypes.c_int64, i32p, ctypes.c_int32, i32p, i32p, ctypes.c_int32, i32p, i32p,
                                        ctypes.POINTER(ctypes.c_int64)]
    vl, tk = _i32(valid_len), _i32(task)
    n = int(vl.shape[0])
    pl = None if padded_len is None else _i32(padded_len)
    so, stk, T = np.full(2 * n + 1, -9, np.int32), np.full(max(2 * n, 1), -9, np.int32), ctypes.c_int64(-9)
    st = L.lobra_padded_segments(n, None if pl is None else pl.ctypes.data_as(i32p), int(uniform_len),
                                 vl.ctypes.data_as(i32p), tk.ctypes.data_as(i32p), int(n_tasks),
                                 so.ctypes.data_as(i32p), stk.ctypes.data_as(i32p), ctypes.byref(T))
    if check:
        _check(st, "lobra_padded_segments")
        return so, stk[: 2 * n], int(T.value)
    return st, so, stk[: 2 * n], int(T.value)


def lobra_mlora_plan_token_task_map(plan: Plan, out_task, out_count, stream=None):
    _check(lib().lobra_mlora_plan_token_task_map(plan.handle, _ptr(out_task), _ptr(out_count), _stream(stream)),
           "lobra_mlora_plan_token_task_map")


# ---------------------------------------------------------------------------------------------
# device-side convenience used by tests, smoke and bench: upload a workload, allocate buffers
# ---------------------------------------------------------------------------------------------
class DeviceProblem:
    """A workloads.Problem resident on the GPU with all outputs and scratch allocated."""

    def __init__(self, p, plan_flags=0, device="cuda:0"):
        import torch
        self.p = p
        self.torch = torch
        self.dev = torch.device(device)
        self.plan = Plan.for_problem(p, plan_flags)
        self.edt = torch.float32 if p.dtype == "f32" else torch.bfloat16

        def up(a):
            if p.dtype == "f32":
                return torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
            return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(self.dev).view(torch.bfloat16)
        self.x, self.W, self.dy = up(p.x), up(p.W), up(p.dy)
        self.A = up(p.A) if p.R_tot else None
        self.B = up(p.B) if p.R_tot else None
        self.s = torch.from_numpy(np.asarray(p.s, np.float32)).to(self.dev) if p.n_tasks else None
        # every buffer the library writes sits between two sentinel margins (guards_intact() checks them)
        self._guards = []
        self.y = self._guarded((p.T, p.d_out), self.edt)
        self.dx = self._guarded((p.T, p.d_in), self.edt)
        self.dA = self._guarded((p.R_tot, p.d_in), torch.float32).zero_()
        self.dB = self._guarded((p.R_tot, p.d_out // getattr(p, "n_proj", 1)), torch.float32).zero_()
        self.h_save = self._guarded((max(self.plan.h_save_bytes, 16),), torch.uint8)
        self.ws = self._guarded((max(self.plan.fwd_ws_bytes, self.plan.bwd_ws_bytes, 16),), torch.uint8)

    GUARD_BYTES, GUARD_VALUE = 4096, 0xC3

    def _guarded(self, shape, dtype):
        torch = self.torch
        n = int(np.prod(shape)) * torch.empty(0, dtype=dtype).element_size()
        n16 = (n + 15) // 16 * 16
        buf = torch.full((n16 + 2 * self.GUARD_BYTES,), self.GUARD_VALUE, dtype=torch.uint8, device=self.dev)
        self._guards.append((buf, n))
        return buf[self.GUARD_BYTES:self.GUARD_BYTES + n].view(dtype).view(*shape)

    def guards_intact(self):
        """True when no byte of the margins around y, dx, dA, dB, h_save and the workspace has changed."""
        g = self.GUARD_BYTES
        return all(bool((buf[:g] == self.GUARD_VALUE).all()) and bool((buf[g + n:] == self.GUARD_VALUE).all())
                   for buf, n in self._guards)

    def fwd(self, save_h=True):
        lobra_mlora_plan_fwd(self.plan, self.x, self.W, self.A, self.B, self.s, self.y,
                             self.h_save if save_h else None, self.ws)

    def bwd(self, use_saved_h=True, flags=0):
        lobra_mlora_plan_bwd(self.plan, self.x, self.W, self.A, self.B, self.s, self.dy,
                             self.h_save if use_saved_h else None, self.dx, self.dA, self.dB,
                             flags, self.ws)

    def step(self):
        self.fwd(True)
        self.bwd(True)

    def clone_io(self):
        """The same layer and batch (plan, W, A, B, s, scratch shared) on its own copies of x and dy and its own
        outputs: benchmarks rotate over several of these so that no call finds its inputs in a cache."""
        torch = self.torch
        o = DeviceProblem.__new__(DeviceProblem)
        o.__dict__.update(self.__dict__)
        o.x, o.dy = self.x.clone(), self.dy.clone()
        o.y, o.dx = torch.empty_like(self.y), torch.empty_like(self.dx)
        o.dA, o.dB = torch.zeros_like(self.dA), torch.zeros_like(self.dB)
        return o

    def base_only(self):
        """The same x, W, dy, y, dx under a plan without adapters: the base products alone."""
        torch, p = self.torch, self.p
        o = DeviceProblem.__new__(DeviceProblem)
        o.p, o.torch, o.dev, o.edt = p, torch, self.dev, self.edt
        o.plan = Plan(p.dtype, p.T, p.d_in, p.d_out, None, [0, p.T], [-1])
        o.x, o.W, o.dy, o.y, o.dx = self.x, self.W, self.dy, self.y, self.dx
        o.A = o.B = o.s = None
        o.dA = torch.zeros((0, p.d_in), dtype=torch.float32, device=self.dev)
        o.dB = torch.zeros((0, p.d_out), dtype=torch.float32, device=self.dev)
        o.h_save = o.ws = torch.empty(16, dtype=torch.uint8, device=self.dev)
        return o

    def host(self, t):
        """Device tensor -> float64 numpy."""
        return t.detach().to(self.torch.float32).cpu().numpy().astype(np.float64)


# ---------------------------------------------------------------------------------------------
# launch trace: per-kernel durations from HIP events recorded on the stream the kernels run on
# ---------------------------------------------------------------------------------------------
KERNEL_NAMES = {1: "shrink", 2: "gemm", 3: "grad_stage1", 4: "grad_stage2", 5: "token_task", 6: "adam"}


class LaunchTrace:
    """Attaches hipEvent pairs to a plan; after a synchronize, ``durations()`` lists
    (kernel name, milliseconds) for every launch made since ``attach()``."""

    def __init__(self, plan: Plan, max_launches=32):
        self.plan, self.n = plan, int(max_launches)
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.events = (ctypes.c_void_p * (2 * self.n))()
        for i in range(2 * self.n):
            e = ctypes.c_void_p()
            if self.hip.hipEventCreate(ctypes.byref(e)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.events[i] = e
        self.ids = (ctypes.c_int32 * self.n)()
        self.count = ctypes.c_int32(0)
        L = lib()
        L.lobra_mlora_plan_set_trace.restype = ctypes.c_int
        L.lobra_mlora_plan_set_trace.argtypes = [
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32,
            ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]

    def attach(self):
        _check(lib().lobra_mlora_plan_set_trace(self.plan.handle, self.events, self.n, self.ids,
                                                ctypes.byref(self.count)), "lobra_mlora_plan_set_trace")

    def detach(self):
        _check(lib().lobra_mlora_plan_set_trace(self.plan.handle, None, 0, None, None),
               "lobra_mlora_plan_set_trace")

    def durations(self):
        out = []
        for i in range(min(self.count.value, self.n)):
            ms = ctypes.c_float()
            if self.hip.hipEventElapsedTime(ctypes.byref(ms), self.events[2 * i], self.events[2 * i + 1]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            out.append((KERNEL_NAMES.get(self.ids[i], "?"), float(ms.value)))
        return out

    def close(self):
        self.detach()
        for i in range(2 * self.n):
            self.hip.hipEventDestroy(self.events[i])
