"""Python binding of libfinch.so (the C ABI declared in include/finch.h).

Argument marshalling only: every step of the path (scoring, top-r, compaction)
runs in the HIP kernels behind the C ABI.  There is no CPU or PyTorch fallback: if
the shared library is missing or no GPU is usable, the calls raise.

PyTorch is used for device memory and streams: tensors supply device pointers,
`torch.cuda.current_stream()` supplies the stream.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
# FINCH_LIBRARY names another build of the same sources to load instead (the measurement build
# with phase timers, libfinch_phases.so); it must exist - there is no fallback.
LIB_PATH = os.environ.get("FINCH_LIBRARY") or os.path.join(_PKG_DIR, "libfinch.so")

FINCH_OK = 0
FINCH_ERR_INVALID_ARG = -1
FINCH_ERR_UNSUPPORTED = -2
FINCH_ERR_CAPACITY = -3
FINCH_ERR_WORKSPACE = -4
FINCH_ERR_HIP = -5
FINCH_ERR_TIMEOUT = -6

FINCH_F32 = 0
FINCH_BF16 = 1

EXPORTED_SYMBOLS = (
    "finch_create", "finch_destroy", "finch_workspace_size", "finch_score", "finch_topk",
    "finch_compact", "finch_step", "finch_schedule", "finch_schedule_mode", "finch_last_hip_error",
    "finch_status_string", "finch_version", "finch_profile", "finch_profile_read",
    "finch_set_option", "finch_set_reposition", "finch_prompt_lse", "finch_loop", "finch_loop_workspace_size",
    "finch_step_static", "finch_static_scratch_bytes", "finch_loop_check",
    "finch_workspace_status",
)

KERNEL_NAMES = ("rowstats", "lse", "colsum", "select", "gather", "owner", "prompt_lse")

FINCH_OPT_STEP_PATH = 1
FINCH_OPT_SLICE_KEYS = 3
FINCH_OPT_LAYER_GROUP = 4
FINCH_OPT_LAYER_WAIT_TICKS = 5
FINCH_SCHEDULE_PROPORTIONAL, FINCH_SCHEDULE_CONSTANT = 0, 1
FINCH_PATH_AUTO = 0
FINCH_PATH_SEPARATE = 1
FINCH_PATH_OWNER = 3
FINCH_ROPE_OFF, FINCH_ROPE_HALF, FINCH_ROPE_INTERLEAVED = 0, 1, 2
FINCH_ORDER_ASCENDING, FINCH_ORDER_RANK = 0, 1


class FinchError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


class finch_reposition(ctypes.Structure):
    _fields_ = [("pairing", ctypes.c_int32), ("order", ctypes.c_int32), ("base", ctypes.c_double)]


class finch_config(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class finch_problem(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("k_chunk", ctypes.c_void_p), ("v_chunk", ctypes.c_void_p),
                ("k_out", ctypes.c_void_p), ("v_out", ctypes.c_void_p),
                ("scores", ctypes.c_void_p), ("idx", ctypes.c_void_p),
                ("n_que", ctypes.c_int32), ("c", ctypes.c_int32), ("m", ctypes.c_int32),
                ("r", ctypes.c_int32), ("k_que", ctypes.c_void_p), ("lse_extra", ctypes.c_void_p),
                ("q_doc", ctypes.c_void_p)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libfinch.so (built in-tree by `python -m paper_2408_00167_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        how = ("python -m paper_2408_00167_amd.build --phase-timers" if LIB_PATH.endswith("libfinch_phases.so")
               else "python -m paper_2408_00167_amd.build")
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `{how}` (there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.finch_create.argtypes = [P(finch_config), P(vp)]
    lib.finch_create.restype = ctypes.c_int
    lib.finch_destroy.argtypes = [vp]
    lib.finch_destroy.restype = ctypes.c_int
    lib.finch_workspace_size.argtypes = [vp, P(finch_problem), i32, P(sz)]
    lib.finch_workspace_size.restype = ctypes.c_int
    for name in ("finch_score", "finch_topk", "finch_compact", "finch_step"):
        fn = getattr(lib, name)
        fn.argtypes = [vp, P(finch_problem), vp, i32, vp, sz, vp]
        fn.restype = ctypes.c_int
    lib.finch_schedule.argtypes = [i64, i32, i64, P(i32), i32]
    lib.finch_schedule.restype = ctypes.c_int
    lib.finch_schedule_mode.argtypes = [i64, i32, i64, i32, P(i32), i32]
    lib.finch_schedule_mode.restype = ctypes.c_int
    lib.finch_last_hip_error.argtypes = [vp]
    lib.finch_last_hip_error.restype = i32
    lib.finch_status_string.argtypes = [ctypes.c_int]
    lib.finch_status_string.restype = ctypes.c_char_p
    lib.finch_profile.argtypes = [vp, i32]
    lib.finch_profile.restype = ctypes.c_int
    lib.finch_profile_read.argtypes = [vp, P(ctypes.c_float), P(i32)]
    lib.finch_profile_read.restype = ctypes.c_int
    lib.finch_loop_workspace_size.argtypes = [vp, P(finch_problem), P(i32), i32, P(sz)]
    lib.finch_loop_workspace_size.restype = ctypes.c_int
    lib.finch_loop.argtypes = [vp, P(finch_problem), vp, P(i32), vp, i32, vp, sz, vp]
    lib.finch_loop.restype = ctypes.c_int
    lib.finch_prompt_lse.argtypes = [vp, P(finch_problem), vp, i32, vp]
    lib.finch_prompt_lse.restype = ctypes.c_int
    lib.finch_set_reposition.argtypes = [vp, P(finch_reposition)]
    lib.finch_set_reposition.restype = ctypes.c_int
    lib.finch_step_static.argtypes = [vp, P(finch_problem), vp, i32, vp]
    lib.finch_step_static.restype = ctypes.c_int
    lib.finch_static_scratch_bytes.argtypes = []
    lib.finch_static_scratch_bytes.restype = sz
    lib.finch_workspace_status.argtypes = [vp, vp, vp, P(i32)]
    lib.finch_workspace_status.restype = ctypes.c_int
    lib.finch_loop_check.argtypes = [P(finch_config), P(finch_problem), P(i32), i32]
    lib.finch_loop_check.restype = ctypes.c_int
    lib.finch_set_option.argtypes = [vp, i32, i64]
    lib.finch_set_option.restype = ctypes.c_int
    lib.finch_version.argtypes = []
    lib.finch_version.restype = i32
    _lib = lib
    return lib


def _check(status: int, where: str, ctx=None):
    if status != FINCH_OK:
        lib = load_library()
        detail = lib.finch_status_string(status).decode()
        if status == FINCH_ERR_HIP and ctx is not None:
            detail += f", hipError {lib.finch_last_hip_error(ctx)}"
        raise FinchError(status, where, detail)


# ------------------------------------------------------------------ C ABI mirrors

def finch_create(dtype: int, head_dim: int, group_size: int) -> ctypes.c_void_p:
    lib = load_library()
    cfg = finch_config(dtype, head_dim, group_size, 0)
    ctx = ctypes.c_void_p()
    _check(lib.finch_create(ctypes.byref(cfg), ctypes.byref(ctx)), "finch_create")
    return ctx


def finch_destroy(ctx) -> None:
    _check(load_library().finch_destroy(ctx), "finch_destroy")


def finch_workspace_size(ctx, host_desc, n: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().finch_workspace_size(ctx, host_desc, n, ctypes.byref(out)),
           "finch_workspace_size", ctx)
    return out.value


def _call(name: str, ctx, host_desc, dev_desc_ptr: int, n: int, ws_ptr: int, ws_bytes: int,
          stream: int) -> None:
    fn = getattr(load_library(), name)
    _check(fn(ctx, host_desc, ctypes.c_void_p(dev_desc_ptr), n, ctypes.c_void_p(ws_ptr),
              ws_bytes, ctypes.c_void_p(stream)), name, ctx)


def finch_prompt_lse(ctx, host_desc, dev_desc_ptr: int, n: int, stream: int = 0) -> None:
    _check(load_library().finch_prompt_lse(ctx, host_desc, ctypes.c_void_p(dev_desc_ptr), n,
                                           ctypes.c_void_p(stream)), "finch_prompt_lse", ctx)


def finch_score(ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream=0):
    _call("finch_score", ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream)


def finch_topk(ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream=0):
    _call("finch_topk", ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream)


def finch_compact(ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream=0):
    _call("finch_compact", ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream)


def finch_step(ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream=0):
    _call("finch_step", ctx, host_desc, dev_desc_ptr, n, ws_ptr, ws_bytes, stream)


def finch_step_static(ctx, host_desc, dev_desc_ptr, n, stream=0):
    _check(load_library().finch_step_static(ctx, host_desc, ctypes.c_void_p(dev_desc_ptr), n,
                                            ctypes.c_void_p(stream)), "finch_step_static", ctx)


def finch_static_scratch_bytes() -> int:
    return int(load_library().finch_static_scratch_bytes())


def finch_schedule(n_cont: int, m: int, k: int, constant_budget: bool = False) -> List[int]:
    steps = max(0, -(-n_cont // m)) if m > 0 else 0
    buf = (ctypes.c_int32 * max(1, steps))()
    if constant_budget:
        _check(load_library().finch_schedule_mode(n_cont, m, k, FINCH_SCHEDULE_CONSTANT, buf, steps),
               "finch_schedule_mode")
    else:
        _check(load_library().finch_schedule(n_cont, m, k, buf, steps), "finch_schedule")
    return list(buf[:steps])


def finch_profile(ctx, enable: bool) -> None:
    _check(load_library().finch_profile(ctx, 1 if enable else 0), "finch_profile", ctx)


def finch_profile_read(ctx) -> Dict[str, Dict[str, float]]:
    n = len(KERNEL_NAMES)
    ms = (ctypes.c_float * n)()
    cnt = (ctypes.c_int32 * n)()
    _check(load_library().finch_profile_read(ctx, ms, cnt), "finch_profile_read", ctx)
    return {KERNEL_NAMES[i]: {"ms": float(ms[i]), "launches": int(cnt[i])} for i in range(n)}


def finch_set_option(ctx, option: int, value: int) -> None:
    _check(load_library().finch_set_option(ctx, option, value), "finch_set_option", ctx)


def finch_set_reposition(ctx, pairing: int = FINCH_ROPE_OFF, order: int = FINCH_ORDER_ASCENDING,
                         base: float = 10000.0) -> None:
    how = finch_reposition(pairing, order, base)
    _check(load_library().finch_set_reposition(ctx, ctypes.byref(how)), "finch_set_reposition", ctx)


def finch_loop_workspace_size(ctx, host_desc, host_step_first, n_steps: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().finch_loop_workspace_size(ctx, host_desc, host_step_first, n_steps,
                                                    ctypes.byref(out)),
           "finch_loop_workspace_size", ctx)
    return out.value


def finch_loop(ctx, host_desc, dev_desc: int, host_step_first, dev_step_first: int, n_steps: int,
               workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    _check(load_library().finch_loop(ctx, host_desc, ctypes.c_void_p(dev_desc), host_step_first,
                                     ctypes.c_void_p(dev_step_first), n_steps,
                                     ctypes.c_void_p(workspace), workspace_bytes,
                                     ctypes.c_void_p(stream)),
           "finch_loop", ctx)


def finch_loop_check(dtype: int, head_dim: int, group_size: int, host_desc, host_step_first,
                     n_steps: int) -> int:
    """Host-only argument checks of finch_loop; returns the status (no exception)."""
    cfg = finch_config(dtype, head_dim, group_size, 0)
    return int(load_library().finch_loop_check(ctypes.byref(cfg), host_desc, host_step_first, n_steps))


def finch_version() -> int:
    return load_library().finch_version()


# ----------------------------------------------------------------- marshalling help

def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return t.data_ptr() if t.numel() > 0 else None


class Batch:
    """A descriptor array on the host and its copy on the device.

    `problems` is a sequence of dicts with tensors q, k_cache, v_cache, k_chunk,
    v_chunk, k_out, v_out, scores, idx, and optionally k_que, lse_extra, q_doc (any may be
    None where the C ABI allows NULL) and ints n_que, c, m, r.  The tensors are only read for their device
    pointers; the caller keeps them alive.
    """

    def __init__(self, problems: Sequence[Dict], device="cuda"):
        import torch
        n = len(problems)
        self.n = n
        self.host = (finch_problem * max(1, n))()
        for i, pb in enumerate(problems):
            d = self.host[i]
            for name in ("q", "k_cache", "v_cache", "k_chunk", "v_chunk", "k_out", "v_out",
                         "scores", "idx", "k_que", "lse_extra", "q_doc"):
                setattr(d, name, _ptr(pb.get(name)))
            d.n_que, d.c, d.m, d.r = int(pb["n_que"]), int(pb["c"]), int(pb["m"]), int(pb["r"])
        raw = bytes(self.host)[: n * ctypes.sizeof(finch_problem)]
        self.dev = torch.frombuffer(bytearray(raw if raw else b"\0" * 8), dtype=torch.uint8).to(device)
        self.dev_ptr = self.dev.data_ptr()


class LoopBatch:
    """The descriptor arrays of all steps of a chunk loop, step after step, with the
    table of where each step starts, on the host and on the device (finch_loop).

    `steps` is a sequence of per-step problem lists as `Batch` takes them; slot j of
    every step must describe the same problem and later steps may only drop slots
    from the end."""

    def __init__(self, steps: Sequence[Sequence[Dict]], device="cuda"):
        import torch
        flat = [pb for st in steps for pb in st]
        self.batch = Batch(flat, device=device)
        self.n_steps = len(steps)
        first = [0]
        for st in steps:
            first.append(first[-1] + len(st))
        self.host_first = (ctypes.c_int32 * len(first))(*first)
        self.dev_first = torch.tensor(first, dtype=torch.int32, device=device)


class Finch:
    """A context plus a workspace tensor that grows on demand (outside any timed
    or captured region the caller should pre-size it with `reserve`)."""

    def __init__(self, dtype: int, head_dim: int, group_size: int, device="cuda"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2408_00167_amd needs a GPU: there is no CPU fallback")
        self.device = torch.device(device)
        self.ctx = finch_create(dtype, head_dim, group_size)
        self.ws = None

    def close(self):
        if self.ctx is not None:
            finch_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_step_path(self, path: int) -> None:
        finch_set_option(self.ctx, FINCH_OPT_STEP_PATH, path)

    def set_reposition(self, pairing: int = FINCH_ROPE_OFF, order: int = FINCH_ORDER_ASCENDING,
                       base: float = 10000.0) -> None:
        finch_set_reposition(self.ctx, pairing, order, base)

    def reserve(self, batch: Batch) -> int:
        import torch
        need = finch_workspace_size(self.ctx, batch.host, batch.n)
        self._grow(need)
        return need

    def _grow(self, need: int) -> None:
        """A larger workspace replaces the present one only once nothing enqueued on any
        stream can still be using it (growth is rare; pre-size with reserve outside hot
        loops)."""
        import torch
        if self.ws is None or self.ws.numel() < need:
            if self.ws is not None:
                torch.cuda.synchronize(self.device)
            self.ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)

    def _run(self, name: str, batch: Batch, stream=None):
        import torch
        self.reserve(batch)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        _call(name, self.ctx, batch.host, batch.dev_ptr, batch.n, self.ws.data_ptr(),
              self.ws.numel(), s)

    def score(self, batch: Batch, stream=None):
        self._run("finch_score", batch, stream)

    def topk(self, batch: Batch, stream=None):
        self._run("finch_topk", batch, stream)

    def compact(self, batch: Batch, stream=None):
        self._run("finch_compact", batch, stream)

    def step(self, batch: Batch, stream=None):
        self._run("finch_step", batch, stream)

    def step_static(self, batch: Batch, stream=None):
        """finch_step on the library's own scratch: no workspace, nothing allocated."""
        import torch
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        finch_step_static(self.ctx, batch.host, batch.dev_ptr, batch.n, s)

    def workspace_status(self, stream=None) -> int:
        """Waits for the stream; 0, or the status word of the last launches (FINCH_ERR_TIMEOUT raised)."""
        import torch
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        flags = ctypes.c_int32(0)
        if self.ws is None:
            return 0
        _check(load_library().finch_workspace_status(self.ctx, ctypes.c_void_p(self.ws.data_ptr()),
                                                     ctypes.c_void_p(s), ctypes.byref(flags)),
               "finch_workspace_status", self.ctx)
        return int(flags.value)

    def prompt_lse(self, batch: Batch, stream=None):
        import torch
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        finch_prompt_lse(self.ctx, batch.host, batch.dev_ptr, batch.n, s)

    def reserve_loop(self, lb: LoopBatch) -> int:
        import torch
        need = finch_loop_workspace_size(self.ctx, lb.batch.host, lb.host_first, lb.n_steps)
        self._grow(need)
        return need

    def loop(self, lb: LoopBatch, stream=None):
        import torch
        self.reserve_loop(lb)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        finch_loop(self.ctx, lb.batch.host, lb.batch.dev_ptr, lb.host_first, lb.dev_first.data_ptr(),
                   lb.n_steps, self.ws.data_ptr(), self.ws.numel(), s)
