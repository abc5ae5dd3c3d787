"""ctypes binding of libteraio.so: argument marshalling only, same names as the C ABI.

Every step of the method runs inside the library; nothing here computes.  The
library must be present: loading fails loudly otherwise (there is no fallback).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libteraio.so")

ARCH = {"gpt": 0, "llama": 1}
PREC = {"fp32": 0, "bf16": 1}
PROFILE_MEASURED, PROFILE_MODELLED, PROFILE_OFFLOADED = 0, 1, 2
OFFLOAD, PREFETCH = 0, 1


class TioError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"teraio error {code}: {msg}")
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("arch", "n_layers", "d_model", "n_heads", "d_ff", "vocab", "seq_len",
                                          "batch", "precision")] + \
               [(n, C.c_float) for n in ("lr", "beta1", "beta2", "adam_eps", "weight_decay", "norm_eps", "rope_theta")] + \
               [("micro_batches", C.c_int32)]


class RuntimeCfg(C.Structure):
    _fields_ = [("arena", C.c_void_p), ("arena_bytes", C.c_uint64), ("host_pool", C.c_void_p),
                ("host_bytes", C.c_uint64), ("compute_stream", C.c_void_p), ("d2h_stream", C.c_void_p),
                ("h2d_stream", C.c_void_p), ("slow_tier_bw", C.c_uint64), ("poison_freed", C.c_int32),
                ("pool_on_device", C.c_int32), ("host_tier_pool", C.c_void_p), ("host_tier_bytes", C.c_uint64),
                ("host_tier_d2h_stream", C.c_void_p), ("host_tier_h2d_stream", C.c_void_p), ("host_tier_bw", C.c_uint64),
                ("slow_tier_file", C.c_char_p), ("staging", C.c_void_p), ("staging_bytes", C.c_uint64),
                ("file_chunk_bytes", C.c_uint64), ("file_buffered_io", C.c_int32)]


class FileTierStats(C.Structure):
    _fields_ = [("direct_io", C.c_int32), ("file_bytes", C.c_uint64), ("bytes_written", C.c_uint64),
                ("bytes_read", C.c_uint64)]


class TraceView(C.Structure):
    _fields_ = [("n_kernels", C.c_int32), ("n_tensors", C.c_int32), ("n_persistent", C.c_int32),
                ("n_operands", C.c_int32),
                ("op", C.POINTER(C.c_int32)), ("operand_off", C.POINTER(C.c_int32)),
                ("operand_tensor", C.POINTER(C.c_int32)), ("operand_flags", C.POINTER(C.c_int32)),
                ("flops", C.POINTER(C.c_int64)), ("tau_ns", C.POINTER(C.c_int64)),
                ("tensor_bytes", C.POINTER(C.c_uint64)), ("tensor_kind", C.POINTER(C.c_int32))]


class LifetimesView(C.Structure):
    _fields_ = [("n_kernels", C.c_int32), ("n_periods", C.c_int32), ("M", C.POINTER(C.c_uint64)),
                ("tensor", C.POINTER(C.c_int32)), ("bytes", C.POINTER(C.c_uint64)),
                ("start", C.POINTER(C.c_int32)), ("end", C.POINTER(C.c_int32))]


class PlanEntry(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tensor", "kind", "trigger", "deadline", "urgent", "pair")]


class Alloc(C.Structure):
    _fields_ = [("tensor", C.c_int32), ("first_kernel", C.c_int32), ("last_kernel", C.c_int32),
                ("address", C.c_uint64)]


class PlanView(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_kernels", "n_entries", "n_greedy", "n_forced", "n_allocs", "reserved")] + \
               [("entries", C.POINTER(PlanEntry)), ("Mp", C.POINTER(C.c_uint64)), ("allocs", C.POINTER(Alloc))] + \
               [(n, C.c_uint64) for n in ("cap_bytes", "planning_cap_bytes", "arena_bytes_needed",
                                          "host_bytes_needed", "bytes_per_direction")] + \
               [("n_pairs", C.c_int32), ("reserved2", C.c_int32), ("pair_tier", C.POINTER(C.c_int32))] + \
               [(n, C.c_uint64) for n in ("host_tier_bytes_needed", "host_tier_peak_bytes", "host_tier_bw")] + \
               [("retime_pass", C.c_int32), ("reserved3", C.c_int32)]


class PlanOpts(C.Structure):
    _fields_ = [("duplex", C.c_int32), ("layout_retries", C.c_int32), ("min_bytes", C.c_uint64),
                ("arena_bytes", C.c_uint64), ("host_bw", C.c_uint64), ("host_budget", C.c_uint64),
                ("clamp_benefit", C.c_int32), ("retime_passes", C.c_int32)]


class StepStats(C.Structure):
    _fields_ = [("loss", C.c_float), ("step", C.c_int32), ("wall_ns", C.c_int64), ("kernel_ns", C.c_int64),
                ("d2h_bytes", C.c_uint64), ("h2d_bytes", C.c_uint64), ("d2h_busy_ns", C.c_int64),
                ("h2d_busy_ns", C.c_int64), ("n_kernels", C.c_int32), ("n_migrations", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch owns the arena, the pinned pool and the streams: its HIP runtime must be the one in
        # the process before the library (which needs libamdhip64 too) is mapped
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        _lib.tio_last_error.restype = C.c_char_p
        _lib.tio_version.restype = C.c_char_p
        for name in ("tio_trace_free", "tio_lifetimes_free", "tio_plan_free"):
            getattr(_lib, name).restype = None
            getattr(_lib, name).argtypes = [C.c_void_p]
    return _lib


def _check(rc):
    if rc != 0:
        raise TioError(rc, lib().tio_last_error().decode())


def model_cfg(cfg: dict) -> ModelCfg:
    return ModelCfg(ARCH[cfg["arch"]], cfg["L"], cfg["d"], cfg["H"], cfg["f"], cfg["V"], cfg["T"], cfg["B"],
                    PREC[cfg["precision"]], cfg.get("lr", 1e-3), cfg.get("beta1", 0.9), cfg.get("beta2", 0.999),
                    cfg.get("adam_eps", 1e-8), cfg.get("weight_decay", 0.01), cfg.get("eps", 1e-5),
                    cfg.get("rope_theta", 10000.0), int(cfg.get("micro_batches", 1) or 1))


def _arr(ptr, n, dtype):
    if n == 0:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype, copy=True)


# ------------------------------------------------------------------ model description
def tio_param_list(cfg: dict):
    """[(name, rows, cols)] in parameter-list order."""
    mc = model_cfg(cfg)
    n = C.c_int32()
    _check(lib().tio_param_count(C.byref(mc), C.byref(n)))
    out = []
    buf = C.create_string_buffer(64)
    for i in range(n.value):
        r, c = C.c_int64(), C.c_int64()
        _check(lib().tio_param_info(C.byref(mc), i, buf, 64, C.byref(r), C.byref(c)))
        out.append((buf.value.decode(), r.value, c.value))
    return out


# ------------------------------------------------------------------ trace / lifetimes / plan handles
class Trace:
    def __init__(self, handle):
        self.h = handle

    def __del__(self):
        if getattr(self, "h", None):
            lib().tio_trace_free(self.h)
            self.h = None

    def export(self):
        v = TraceView()
        _check(lib().tio_trace_export(self.h, C.byref(v)))
        return dict(n_kernels=v.n_kernels, n_tensors=v.n_tensors, n_persistent=v.n_persistent,
                    op=_arr(v.op, v.n_kernels, np.int32), operand_off=_arr(v.operand_off, v.n_kernels + 1, np.int32),
                    operand_tensor=_arr(v.operand_tensor, v.n_operands, np.int32),
                    operand_flags=_arr(v.operand_flags, v.n_operands, np.int32),
                    flops=_arr(v.flops, v.n_kernels, np.int64), tau=_arr(v.tau_ns, v.n_kernels, np.int64),
                    tensor_bytes=_arr(v.tensor_bytes, v.n_tensors, np.uint64),
                    tensor_kind=_arr(v.tensor_kind, v.n_tensors, np.int32))

    def set_tau(self, tau):
        t = np.ascontiguousarray(tau, dtype=np.int64)
        _check(lib().tio_trace_set_tau(self.h, t.ctypes.data_as(C.POINTER(C.c_int64)), len(t)))


def tio_trace_build(cfg: dict) -> Trace:
    mc = model_cfg(cfg)
    h = C.c_void_p()
    _check(lib().tio_trace_build(C.byref(mc), C.byref(h)))
    return Trace(h)


def tio_trace_import(n_persistent, operand_lists, tensor_bytes, tau, tensor_kind=None, op=None) -> Trace:
    """operand_lists: per kernel a sorted list of (tensor, flags)."""
    nk, nt = len(operand_lists), len(tensor_bytes)
    off = np.zeros(nk + 1, dtype=np.int32)
    ten, fl = [], []
    for k, ops in enumerate(operand_lists):
        for t, f in ops:
            ten.append(t)
            fl.append(f)
        off[k + 1] = len(ten)
    ten = np.asarray(ten, dtype=np.int32)
    fl = np.asarray(fl, dtype=np.int32)
    tb = np.asarray(tensor_bytes, dtype=np.uint64)
    ta = np.asarray(tau, dtype=np.int64)
    kind = np.asarray(tensor_kind if tensor_kind is not None else [5] * nt, dtype=np.int32)
    opc = np.asarray(op if op is not None else [0] * nk, dtype=np.int32)
    fz = np.zeros(nk, dtype=np.int64)
    p = lambda a, ty: a.ctypes.data_as(C.POINTER(ty))
    v = TraceView(nk, nt, n_persistent, len(ten), p(opc, C.c_int32), p(off, C.c_int32), p(ten, C.c_int32),
                  p(fl, C.c_int32), p(fz, C.c_int64), p(ta, C.c_int64), p(tb, C.c_uint64), p(kind, C.c_int32))
    h = C.c_void_p()
    _check(lib().tio_trace_import(C.byref(v), C.byref(h)))
    return Trace(h)


class Lifetimes:
    def __init__(self, handle):
        self.h = handle

    def __del__(self):
        if getattr(self, "h", None):
            lib().tio_lifetimes_free(self.h)
            self.h = None

    def export(self):
        v = LifetimesView()
        _check(lib().tio_lifetimes_export(self.h, C.byref(v)))
        n = v.n_periods
        return dict(M=_arr(v.M, v.n_kernels, np.uint64), tensor=_arr(v.tensor, n, np.int32),
                    bytes=_arr(v.bytes, n, np.uint64), start=_arr(v.start, n, np.int32), end=_arr(v.end, n, np.int32))


def tio_analyze_lifetimes(trace: Trace) -> Lifetimes:
    h = C.c_void_p()
    _check(lib().tio_analyze_lifetimes(trace.h, C.byref(h)))
    return Lifetimes(h)


class Plan:
    def __init__(self, handle):
        self.h = handle

    def __del__(self):
        if getattr(self, "h", None):
            lib().tio_plan_free(self.h)
            self.h = None

    def export(self):
        v = PlanView()
        _check(lib().tio_plan_export(self.h, C.byref(v)))
        entries = [(e.tensor, e.kind, e.trigger, e.deadline, e.urgent, e.pair)
                   for e in (v.entries[i] for i in range(v.n_entries))]
        allocs = [(a.tensor, a.first_kernel, a.last_kernel, a.address) for a in (v.allocs[i] for i in range(v.n_allocs))]
        return dict(entries=entries, Mp=[int(x) for x in _arr(v.Mp, v.n_kernels, np.uint64)], allocs=allocs,
                    n_greedy=v.n_greedy, n_forced=v.n_forced, cap=v.cap_bytes, planning_cap=v.planning_cap_bytes,
                    arena_needed=v.arena_bytes_needed, host_needed=v.host_bytes_needed,
                    bytes_per_direction=v.bytes_per_direction,
                    tier=[int(x) for x in _arr(v.pair_tier, v.n_pairs, np.int32)],
                    host_tier_needed=v.host_tier_bytes_needed, host_peak=v.host_tier_peak_bytes, host_bw=v.host_tier_bw, retime_pass=v.retime_pass)


def tio_build_plan(trace: Trace, life: Lifetimes, mem_cap_bytes: int, slow_tier_bw: int, duplex=True,
                   min_bytes=0, arena_bytes=0, layout_retries=24, host_bw=0, host_budget=0, clamp_benefit=False,
                   retime_passes=0) -> Plan:
    o = PlanOpts(1 if duplex else 0, layout_retries, min_bytes, arena_bytes, int(host_bw), int(host_budget),
                 1 if clamp_benefit else 0, int(retime_passes))
    h = C.c_void_p()
    _check(lib().tio_build_plan(trace.h, life.h, C.c_uint64(mem_cap_bytes), C.c_uint64(slow_tier_bw), C.byref(o),
                                C.byref(h)))
    return Plan(h)


def tio_plan_validate(trace: Trace, life: Lifetimes, plan: Plan):
    _check(lib().tio_plan_validate(trace.h, life.h, plan.h))


def tio_plan_simulate(trace: Trace, plan: Plan, slow_tier_bw: int, duplex=True, iterations=3):
    """Performance model: (ns of a steady-state iteration under the plan, ns of the kernels alone)."""
    step, comp = C.c_int64(), C.c_int64()
    _check(lib().tio_plan_simulate(trace.h, plan.h, C.c_uint64(int(slow_tier_bw)), 1 if duplex else 0, int(iterations),
                                   C.byref(step), C.byref(comp)))
    return step.value, comp.value


def tio_plan_simulate_engine(trace: Trace, plan: Plan, slow_tier_bw: int, duplex=True, iterations=3, chunk_bytes=16 << 20,
                             urgent_first=True):
    """Performance model of the engine with ready queues, chunked transfers and urgent-first service."""
    step, comp = C.c_int64(), C.c_int64()
    _check(lib().tio_plan_simulate_engine(trace.h, plan.h, C.c_uint64(int(slow_tier_bw)), 1 if duplex else 0, int(iterations),
                                          C.c_uint64(int(chunk_bytes)), 1 if urgent_first else 0, C.byref(step), C.byref(comp)))
    return step.value, comp.value


def tio_engine_choose(ready, urgent, urgent_first=True, ready_queue=True):
    """Index of the queued request a free channel of the paced engine serves next (-1: none)."""
    r = (C.c_uint8 * max(1, len(ready)))(*[1 if x else 0 for x in ready])
    u = (C.c_uint8 * max(1, len(urgent)))(*[1 if x else 0 for x in urgent])
    return lib().tio_engine_choose(r, u, len(ready), 1 if urgent_first else 0, 1 if ready_queue else 0)


# ------------------------------------------------------------------ runtime (needs a GPU)
class Context:
    """Owns the arena (GPU), the slow-tier pool (pinned host) and three streams via torch,
    and a tio_ctx handle created on them."""

    def __init__(self, cfg: dict, arena_bytes: int, host_bytes: int, slow_tier_bw: int = 0, single_copy_stream=False,
                 arena=None, host=None, pool_on_device=False, host_tier_bytes: int = 0, host_tier_bw: int = 0,
                 host_tier=None, slow_tier_file=None, staging_bytes: int = 256 << 20, file_chunk_bytes: int = 0,
                 file_buffered_io: bool = False, poison_freed: bool = False):
        """host_tier_bytes > 0 (or a pinned uint8 tensor host_tier): a second, host-memory destination with its own
        two copy streams, for plans built with host_bw / host_budget.
        slow_tier_file: path of a file that is the slow tier instead of a memory pool (host_bytes is then the
        largest size it may grow to); transfers go through a pinned staging buffer of staging_bytes."""
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required for the runtime part of the library")
        self.torch = torch
        self.cfg = dict(cfg)
        self.params = tio_param_list(cfg)
        self.index = {n: i for i, (n, _, _) in enumerate(self.params)}
        arena_bytes = (int(arena_bytes) + 4096 + 255) // 256 * 256     # the library keeps the last 4 KiB for itself
        # buffers may be handed in (uint8 tensors, device / pinned) so that several contexts reuse them
        if arena is not None and arena.numel() < arena_bytes:
            raise ValueError("arena tensor too small")
        if host is not None and host.numel() < host_bytes:
            raise ValueError("host tensor too small")
        self.arena = arena if arena is not None else torch.empty(arena_bytes, dtype=torch.uint8, device="cuda:0")
        self.staging = None
        if slow_tier_file is not None:
            if host is not None or pool_on_device:
                raise ValueError("the slow tier is either a pool or a file")
            self.host = None
            staging_bytes = (int(staging_bytes) + 4095) // 4096 * 4096
            self.staging = torch.empty(staging_bytes + 4096, dtype=torch.uint8, pin_memory=True)
            self._staging_off = (-self.staging.data_ptr()) % 4096
        elif host is not None:
            self.host = host
            pool_on_device = host.is_cuda
        elif pool_on_device:
            self.host = torch.empty(int(host_bytes), dtype=torch.uint8, device="cuda:0")
        else:
            self.host = torch.empty(int(host_bytes), dtype=torch.uint8, pin_memory=True)
        self.s_compute = torch.cuda.Stream(device="cuda:0")
        self.s_d2h = torch.cuda.Stream(device="cuda:0")
        self.s_h2d = self.s_d2h if single_copy_stream else torch.cuda.Stream(device="cuda:0")
        self.host_tier = host_tier
        if host_tier is None and host_tier_bytes > 0:
            self.host_tier = torch.empty((int(host_tier_bytes) + 255) // 256 * 256, dtype=torch.uint8, pin_memory=True)
        self.s_d2h1 = self.s_h2d1 = None
        if self.host_tier is not None:
            self.s_d2h1 = torch.cuda.Stream(device="cuda:0")
            self.s_h2d1 = torch.cuda.Stream(device="cuda:0")
        rt = RuntimeCfg(self.arena.data_ptr(), arena_bytes, self.host.data_ptr() if self.host is not None else None, int(host_bytes),
                        self.s_compute.cuda_stream, self.s_d2h.cuda_stream, self.s_h2d.cuda_stream,
                        int(slow_tier_bw), 1 if poison_freed else 0, 1 if pool_on_device else 0,
                        self.host_tier.data_ptr() if self.host_tier is not None else None,
                        self.host_tier.numel() if self.host_tier is not None else 0,
                        self.s_d2h1.cuda_stream if self.s_d2h1 else None, self.s_h2d1.cuda_stream if self.s_h2d1 else None,
                        int(host_tier_bw),
                        os.fsencode(slow_tier_file) if slow_tier_file is not None else None,
                        self.staging.data_ptr() + self._staging_off if self.staging is not None else None,
                        staging_bytes if self.staging is not None else 0, int(file_chunk_bytes),
                        1 if file_buffered_io else 0)
        mc = model_cfg(cfg)
        self.h = C.c_void_p()
        torch.cuda.synchronize()
        _check(lib().tio_ctx_create(C.byref(mc), C.byref(rt), C.byref(self.h)))

    def close(self):
        if getattr(self, "h", None):
            lib().tio_ctx_destroy(self.h)
            self.h = None
            self.arena = self.host = self.host_tier = self.staging = None

    def __del__(self):
        self.close()

    def tio_params_load(self, params: dict):
        """params: {name: array}; every parameter must be loaded before the first step."""
        for name, arr in params.items():
            a = np.ascontiguousarray(arr, dtype=np.float32).reshape(-1)
            _check(lib().tio_params_load(self.h, self.index[name], a.ctypes.data_as(C.POINTER(C.c_float)),
                                         C.c_int64(a.size)))

    def tio_params_read(self, name: str, which: int = 0):
        _, r, c = self.params[self.index[name]]
        out = np.empty(r * c, dtype=np.float32)
        _check(lib().tio_params_read(self.h, self.index[name], which, out.ctypes.data_as(C.POINTER(C.c_float)),
                                     C.c_int64(out.size)))
        return out.reshape((r, c) if r > 1 else (c,))

    def tio_grads_read(self, name: str):
        _, r, c = self.params[self.index[name]]
        out = np.empty(r * c, dtype=np.float32)
        _check(lib().tio_grads_read(self.h, self.index[name], out.ctypes.data_as(C.POINTER(C.c_float)),
                                    C.c_int64(out.size)))
        return out.reshape((r, c) if r > 1 else (c,))

    def tio_file_tier_info(self) -> dict:
        st = FileTierStats()
        _check(lib().tio_file_tier_info(self.h, C.byref(st)))
        return {f: getattr(st, f) for f, _ in FileTierStats._fields_}

    def tio_set_slow_tier_bw(self, bw: int):
        _check(lib().tio_set_slow_tier_bw(self.h, C.c_uint64(int(bw))))

    def tio_train_step(self, tokens, labels, plan: Plan | None = None, capture_grads=False, time_kernels=False,
                       timeline=False):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        l = np.ascontiguousarray(labels, dtype=np.int32)
        st = StepStats()
        flags = (1 if capture_grads else 0) | (2 if time_kernels else 0) | (4 if timeline else 0)
        _check(lib().tio_train_step(self.h, t.ctypes.data_as(C.POINTER(C.c_int32)), l.ctypes.data_as(C.POINTER(C.c_int32)),
                                    plan.h if plan is not None else None, flags, C.byref(st)))
        return {f: getattr(st, f) for f, _ in StepStats._fields_}

    def tio_set_engine_policy(self, chunk_bytes=16 << 20, urgent_first=True, ready_queue=True):
        _check(lib().tio_set_engine_policy(self.h, C.c_uint64(int(chunk_bytes)), 1 if urgent_first else 0, 1 if ready_queue else 0))

    def tio_step_timeline(self, n_kernels: int, n_entries: int):
        a = [np.empty(n_kernels, dtype=np.int64) for _ in range(2)] + [np.empty(max(n_entries, 1), dtype=np.int64) for _ in range(2)]
        p = [x.ctypes.data_as(C.POINTER(C.c_int64)) for x in a]
        _check(lib().tio_step_timeline(self.h, p[0], p[1], n_kernels, p[2], p[3], n_entries))
        return a[0], a[1], a[2][:n_entries], a[3][:n_entries]

    def tio_kernel_times(self, n_kernels: int):
        out = np.empty(n_kernels, dtype=np.int64)
        _check(lib().tio_kernel_times(self.h, out.ctypes.data_as(C.POINTER(C.c_int64)), n_kernels))
        return out

    def tio_profile_iteration(self, tokens, labels, mode=PROFILE_MEASURED) -> Trace:
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        l = np.ascontiguousarray(labels, dtype=np.int32)
        h = C.c_void_p()
        _check(lib().tio_profile_iteration(self.h, t.ctypes.data_as(C.POINTER(C.c_int32)),
                                           l.ctypes.data_as(C.POINTER(C.c_int32)), mode, C.byref(h)))
        return Trace(h)

    def tio_op_bench(self, kernel_index: int, reps: int = 10) -> float:
        out = C.c_double()
        _check(lib().tio_op_bench(self.h, kernel_index, reps, C.byref(out)))
        return out.value


def tio_ctx_create(cfg, arena_bytes, host_bytes, slow_tier_bw=0, single_copy_stream=False, arena=None, host=None,
                   pool_on_device=False, host_tier_bytes=0, host_tier_bw=0, host_tier=None, slow_tier_file=None,
                   staging_bytes=256 << 20, file_chunk_bytes=0, file_buffered_io=False, poison_freed=False) -> Context:
    return Context(cfg, arena_bytes, host_bytes, slow_tier_bw, single_copy_stream, arena, host, pool_on_device,
                   host_tier_bytes, host_tier_bw, host_tier, slow_tier_file, staging_bytes, file_chunk_bytes,
                   file_buffered_io, poison_freed)


def tio_op_gemm(stream_handle, dtype, a_kmajor, b_kmajor, M, N, K, A_ptr, lda, B_ptr, ldb, bias_ptr, resid_ptr, ldr,
                C_ptr, ldc, rowsum_ptr=0, workspace_ptr=0, splits=1):
    """Raw pointers (ints) of device buffers; see include/teraio.h."""
    vp = lambda p: C.c_void_p(p) if p else None
    _check(lib().tio_op_gemm(vp(stream_handle), PREC[dtype], int(a_kmajor), int(b_kmajor), C.c_int64(M), C.c_int64(N),
                             C.c_int64(K), vp(A_ptr), C.c_int64(lda), vp(B_ptr), C.c_int64(ldb), vp(bias_ptr),
                             vp(resid_ptr), C.c_int64(ldr), vp(C_ptr), C.c_int64(ldc), vp(rowsum_ptr), vp(workspace_ptr), int(splits)))


def tio_op_gemm_static_ws(stream_handle, dtype, a_kmajor, b_kmajor, M, N, K, A_ptr, lda, B_ptr, ldb, C_ptr, ldc,
                          rowsum_ptr=0, splits=1):
    """tio_op_gemm with the split-contraction partials in the library's fixed device array; allocates nothing."""
    vp = lambda p: C.c_void_p(p) if p else None
    _check(lib().tio_op_gemm_static_ws(vp(stream_handle), PREC[dtype], int(a_kmajor), int(b_kmajor), C.c_int64(M),
                                       C.c_int64(N), C.c_int64(K), vp(A_ptr), C.c_int64(lda), vp(B_ptr), C.c_int64(ldb),
                                       vp(C_ptr), C.c_int64(ldc), vp(rowsum_ptr), int(splits)))


def tio_op_attention(stream_handle, dtype, B, T, H, dh, qkv_ptr, o_ptr, lse_ptr, dO_ptr=0, delta_ptr=0, dqkv_ptr=0):
    vp = lambda p: C.c_void_p(p) if p else None
    _check(lib().tio_op_attention(vp(stream_handle), PREC[dtype], C.c_int64(B), C.c_int64(T), C.c_int64(H), C.c_int64(dh),
                                  vp(qkv_ptr), vp(o_ptr), vp(lse_ptr), vp(dO_ptr), vp(delta_ptr), vp(dqkv_ptr)))
