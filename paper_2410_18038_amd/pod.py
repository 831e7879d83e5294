"""Thin ctypes binding over ``libpod_attn.so`` (argument marshalling only).

Function names mirror the C ABI in ``include/pod_attn.h``.  Torch is used for device
memory and streams; every step of the attention path runs in the library's HIP kernels.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpod_attn.so")

POD_OK = 0
F16, BF16 = 0, 1
MODE_FUSED, MODE_SERIAL, MODE_STREAMS, MODE_PREFILL_ONLY, MODE_DECODE_ONLY = range(5)
MODE_FLAG_NO_COMBINE = 0x100
MODE_FLAG_CTA_PARALLEL = 0x200
MODE_FLAG_PREFILL_HEAVY = 0x400
MODES = {"fused": MODE_FUSED, "serial": MODE_SERIAL, "streams": MODE_STREAMS,
         "prefill_only": MODE_PREFILL_ONLY, "decode_only": MODE_DECODE_ONLY,
         "fused_cta": MODE_FUSED | MODE_FLAG_CTA_PARALLEL,
         "fused_heavy": MODE_FUSED | MODE_FLAG_PREFILL_HEAVY,
         "prefill_only_heavy": MODE_PREFILL_ONLY | MODE_FLAG_PREFILL_HEAVY,
         "decode_only_lite": MODE_DECODE_ONLY | MODE_FLAG_PREFILL_HEAVY}
POLICY_AUTO, POLICY_ALTERNATE, POLICY_PROPORTIONAL = 0, 1, 2
KV_TOKEN_MAJOR, KV_HEAD_MAJOR = 0, 1

EXPORTS = ["pod_attn_plan_create", "pod_attn_plan_destroy", "pod_attn_plan_info_get",
           "pod_attn_workspace_size", "pod_attn_plan_set_trace", "pod_attn_plan_set_event_log",
           "pod_attn_plan_upload", "pod_attn_forward", "pod_attn_forward_static",
           "pod_attn_role_for_ticket", "pod_attn_simulate_launch", "pod_attn_plan_prefill_item", "pod_attn_plan_prefill_item_of_workgroup", "pod_attn_plan_decode_unit",
           "pod_attn_plan_decode_queue",
           "pod_attn_probe_hbm_read", "pod_attn_probe_mfma", "pod_attn_probe_issue", "pod_attn_probe_colocation",
           "pod_attn_last_error", "pod_attn_version"]


class PodError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pod_attn status {status}: {message}")
        self.status = status


class Params(ctypes.Structure):
    _fields_ = [("n_prefill", ctypes.c_int32), ("n_decode", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("block_size", ctypes.c_int32),
                ("max_blocks_per_seq", ctypes.c_int32), ("n_cache_rows", ctypes.c_int32),
                ("n_blocks", ctypes.c_int32), ("kv_seq_stride", ctypes.c_int64),
                ("policy", ctypes.c_int32), ("max_prefill_waves", ctypes.c_int32),
                ("decode_chunk", ctypes.c_int32), ("prefill_split_len", ctypes.c_int32),
                ("n_compute_units", ctypes.c_int32), ("kv_order", ctypes.c_int32)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("n_prefill_items", ctypes.c_int32), ("n_decode_units", ctypes.c_int32),
                ("n_combine", ctypes.c_int32), ("max_prefill_splits", ctypes.c_int32),
                ("max_decode_splits", ctypes.c_int32), ("decode_chunk", ctypes.c_int32),
                ("prefill_ratio", ctypes.c_int32), ("decode_ratio", ctypes.c_int32),
                ("fused_grid", ctypes.c_int32), ("n_compute_units", ctypes.c_int32),
                ("n_prefill_rows", ctypes.c_int64), ("n_partial_rows", ctypes.c_int64),
                ("workspace_bytes", ctypes.c_int64), ("prefill_heavy_advised", ctypes.c_int32),
                ("reserved0", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded C library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_18038_amd.build` "
                "(hipcc, gfx950). This package has no fallback path.")
        # The library must share torch's HIP runtime (streams, events and device memory are torch's):
        # torch bundles its own libamdhip64 under the same soname, so it has to be loaded first.
        import torch
        bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        if os.path.exists(bundled):
            ctypes.CDLL(bundled, mode=ctypes.RTLD_GLOBAL)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
        L.pod_attn_plan_create.restype = ctypes.c_int
        L.pod_attn_plan_create.argtypes = [ctypes.POINTER(Params), i32p, ctypes.POINTER(vp)]
        L.pod_attn_plan_destroy.restype = None
        L.pod_attn_plan_destroy.argtypes = [vp]
        L.pod_attn_plan_info_get.restype = ctypes.c_int
        L.pod_attn_plan_info_get.argtypes = [vp, ctypes.POINTER(PlanInfo)]
        L.pod_attn_plan_set_trace.restype = ctypes.c_int
        L.pod_attn_plan_set_trace.argtypes = [vp, vp, ctypes.c_size_t]
        L.pod_attn_plan_set_event_log.restype = ctypes.c_int
        L.pod_attn_plan_set_event_log.argtypes = [vp, vp, ctypes.c_size_t]
        L.pod_attn_workspace_size.restype = ctypes.c_size_t
        L.pod_attn_workspace_size.argtypes = [vp]
        L.pod_attn_plan_upload.restype = ctypes.c_int
        L.pod_attn_plan_upload.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.pod_attn_forward.restype = ctypes.c_int
        L.pod_attn_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t,
                                       ctypes.c_int32, vp]
        L.pod_attn_forward_static.restype = ctypes.c_int
        L.pod_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp]
        L.pod_attn_role_for_ticket.restype = ctypes.c_int32
        L.pod_attn_role_for_ticket.argtypes = [ctypes.c_int32] * 4
        L.pod_attn_simulate_launch.restype = ctypes.c_int32
        L.pod_attn_simulate_launch.argtypes = [vp, i32p, ctypes.c_int32, i32p, ctypes.c_int32, i32p, i32p, i32p, i32p]
        L.pod_attn_plan_prefill_item.restype = ctypes.c_int
        L.pod_attn_plan_prefill_item.argtypes = [vp, ctypes.c_int32, i32p]
        L.pod_attn_plan_prefill_item_of_workgroup.restype = ctypes.c_int
        L.pod_attn_plan_prefill_item_of_workgroup.argtypes = [vp, ctypes.c_int32, i32p]
        L.pod_attn_plan_decode_unit.restype = ctypes.c_int
        L.pod_attn_plan_decode_unit.argtypes = [vp, ctypes.c_int32, i32p]
        L.pod_attn_plan_decode_queue.restype = ctypes.c_int
        L.pod_attn_plan_decode_queue.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                                                 ctypes.POINTER(ctypes.c_int32)]
        L.pod_attn_probe_hbm_read.restype = ctypes.c_int
        L.pod_attn_probe_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.pod_attn_probe_mfma.restype = ctypes.c_int
        L.pod_attn_probe_mfma.argtypes = [ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pod_attn_probe_issue.restype = ctypes.c_int
        L.pod_attn_probe_issue.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp,
                                           ctypes.POINTER(ctypes.c_double), vp]
        L.pod_attn_probe_colocation.restype = ctypes.c_int
        L.pod_attn_probe_colocation.argtypes = [ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, ctypes.c_int32,
                                                ctypes.c_int32, ctypes.c_int32, vp, vp, vp]
        L.pod_attn_last_error.restype = ctypes.c_char_p
        L.pod_attn_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def pod_attn_last_error() -> str:
    return lib().pod_attn_last_error().decode()


def pod_attn_version() -> str:
    return lib().pod_attn_version().decode()


def _check(status: int):
    if status != POD_OK:
        raise PodError(status, pod_attn_last_error())


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


class Plan:
    """Owner of one ``pod_attn_plan`` handle."""

    def __init__(self, handle: int, params: Params):
        self.handle = ctypes.c_void_p(handle)
        self.params = params

    def close(self):
        if self.handle:
            lib().pod_attn_plan_destroy(self.handle)
            self.handle = ctypes.c_void_p(None)

    def __del__(self):  # pragma: no cover - best effort
        try:
            self.close()
        except Exception:
            pass

    def info(self) -> PlanInfo:
        return pod_attn_plan_info_get(self)

    def prefill_items(self) -> np.ndarray:
        n = self.info().n_prefill_items
        return np.array([pod_attn_plan_prefill_item(self, i) for i in range(n)], dtype=np.int32).reshape(n, 8)

    def prefill_items_by_workgroup(self) -> np.ndarray:
        n = self.info().n_prefill_items
        return np.array([pod_attn_plan_prefill_item_of_workgroup(self, i) for i in range(n)], dtype=np.int32).reshape(n, 8)

    def decode_units(self) -> np.ndarray:
        n = self.info().n_decode_units
        return np.array([pod_attn_plan_decode_unit(self, i) for i in range(n)], dtype=np.int32).reshape(n, 8)

    def decode_queues(self) -> list:
        """[(begin, end)] of the 8 per-XCD decode queues; units before the first begin are fixed."""
        return [pod_attn_plan_decode_queue(self, q) for q in range(8)]


def make_params(*, n_prefill, n_decode, n_q_heads, n_kv_heads, head_dim, dtype, softmax_scale,
                block_size=0, max_blocks_per_seq=0, n_cache_rows=1, n_blocks=0, kv_seq_stride=0,
                policy=POLICY_AUTO, max_prefill_waves=0, decode_chunk=0, prefill_split_len=0,
                n_compute_units=0, kv_order=KV_TOKEN_MAJOR) -> Params:
    return Params(n_prefill, n_decode, n_q_heads, n_kv_heads, head_dim, dtype, softmax_scale,
                  block_size, max_blocks_per_seq, n_cache_rows, n_blocks, kv_seq_stride, policy,
                  max_prefill_waves, decode_chunk, prefill_split_len, n_compute_units, kv_order)


def pod_attn_plan_create(params: Params, seq_meta_host) -> Plan:
    meta, meta_p = _i32(np.asarray(seq_meta_host).reshape(-1, 4))
    handle = ctypes.c_void_p()
    _check(lib().pod_attn_plan_create(ctypes.byref(params), meta_p, ctypes.byref(handle)))
    return Plan(handle.value, params)


def pod_attn_plan_destroy(plan: Plan):
    plan.close()


def pod_attn_plan_info_get(plan: Plan) -> PlanInfo:
    info = PlanInfo()
    _check(lib().pod_attn_plan_info_get(plan.handle, ctypes.byref(info)))
    return info


def pod_attn_plan_set_trace(plan: Plan, trace_ptr: int, trace_bytes: int):
    _check(lib().pod_attn_plan_set_trace(plan.handle, ctypes.c_void_p(trace_ptr), trace_bytes))


def pod_attn_plan_set_event_log(plan: Plan, log_ptr: int, log_bytes: int):
    _check(lib().pod_attn_plan_set_event_log(plan.handle, ctypes.c_void_p(log_ptr), log_bytes))


EVENT_DTYPE = np.dtype([("kind", np.int32), ("item", np.int32), ("cu", np.int32), ("wg", np.int32),
                        ("t_begin", np.uint64), ("t_end", np.uint64)])
TRACE_DTYPE = np.dtype([("cu", np.int32), ("first_role", np.int32), ("n_first", np.int32), ("n_second", np.int32),
                        ("t_begin", np.uint64), ("t_switch", np.uint64), ("t_end", np.uint64), ("pad", np.uint64)])


def pod_attn_workspace_size(plan: Plan) -> int:
    return int(lib().pod_attn_workspace_size(plan.handle))


def pod_attn_plan_prefill_item_of_workgroup(plan: Plan, workgroup: int):
    out = (ctypes.c_int32 * 8)()
    _check(lib().pod_attn_plan_prefill_item_of_workgroup(plan.handle, workgroup, out))
    return list(out)


def pod_attn_plan_prefill_item(plan: Plan, index: int):
    out = (ctypes.c_int32 * 8)()
    _check(lib().pod_attn_plan_prefill_item(plan.handle, index, out))
    return list(out)


def pod_attn_plan_decode_unit(plan: Plan, index: int):
    out = (ctypes.c_int32 * 8)()
    _check(lib().pod_attn_plan_decode_unit(plan.handle, index, out))
    return list(out)


def pod_attn_plan_decode_queue(plan: Plan, q: int):
    b, e = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().pod_attn_plan_decode_queue(plan.handle, q, ctypes.byref(b), ctypes.byref(e)))
    return int(b.value), int(e.value)


def pod_attn_plan_upload(plan: Plan, workspace_ptr: int, workspace_bytes: int, stream: int = 0):
    _check(lib().pod_attn_plan_upload(plan.handle, ctypes.c_void_p(workspace_ptr), workspace_bytes,
                                      ctypes.c_void_p(stream)))


def pod_attn_forward(prefill_q: int, decode_q: int, k_cache: int, v_cache: int, seq_meta: int,
                     block_table: int, out: int, plan: Plan, workspace: int, workspace_bytes: int,
                     mode: int = MODE_FUSED, stream: int = 0):
    """All tensor arguments are raw device addresses (``tensor.data_ptr()``), 0 for NULL."""
    vp = ctypes.c_void_p
    _check(lib().pod_attn_forward(vp(prefill_q), vp(decode_q), vp(k_cache), vp(v_cache), vp(seq_meta),
                                  vp(block_table), vp(out), plan.handle, vp(workspace), workspace_bytes,
                                  mode, vp(stream)))


STATIC_SCRATCH_BYTES = 64 << 20


def pod_attn_forward_static(prefill_q: int, decode_q: int, k_cache: int, v_cache: int, seq_meta: int,
                            block_table: int, out: int, plan: Plan, mode: int = MODE_FUSED, stream: int = 0):
    """pod_attn_forward on the library's own static scratch: no workspace argument, no allocation."""
    vp = ctypes.c_void_p
    _check(lib().pod_attn_forward_static(vp(prefill_q), vp(decode_q), vp(k_cache), vp(v_cache), vp(seq_meta),
                                         vp(block_table), vp(out), plan.handle, mode, vp(stream)))


def pod_attn_probe_hbm_read(buf: int, nbytes: int, sink: int, stream: int = 0):
    vp = ctypes.c_void_p
    status = lib().pod_attn_probe_hbm_read(vp(buf), nbytes, vp(sink), vp(stream))
    if status != POD_OK:
        raise PodError(status, "pod_attn_probe_hbm_read failed")


def pod_attn_probe_mfma(iters: int, sink: int, stream: int = 0) -> float:
    """Enqueue the MFMA issue loop; returns the flop count of the launch."""
    flops = ctypes.c_double(0.0)
    status = lib().pod_attn_probe_mfma(iters, ctypes.c_void_p(sink), ctypes.byref(flops), ctypes.c_void_p(stream))
    if status != POD_OK:
        raise PodError(status, "pod_attn_probe_mfma failed")
    return float(flops.value)


ISSUE_PROBE_VARIANTS = ["4 matrix instructions", "each + one 2^x", "each + the work of one softmax score (no dot product)",
                        "that + one 2-element dot product", "each + one 2-element dot product only",
                        "pipelined turn: LDS read, 1 matrix instruction, staged softmax of 1 score",
                        "pipelined turn: LDS read, 2 matrix instructions, staged softmax of 2 scores",
                        "no matrix instruction: 8 independent v_fma_f32 (ns per vector instruction)",
                        "no matrix instruction: 8 independent v_exp_f32 (ns per vector instruction)"]


def pod_attn_probe_issue(variant: int, iters: int, wgs_per_unit: int, sink: int, stream: int = 0) -> float:
    """Enqueue one instruction-mix probe; returns the matrix instructions (for the last two variants:
    the vector instructions) one wavefront issues."""
    n = ctypes.c_double(0.0)
    status = lib().pod_attn_probe_issue(variant, iters, wgs_per_unit, ctypes.c_void_p(sink), ctypes.byref(n),
                                        ctypes.c_void_p(stream))
    if status != POD_OK:
        raise PodError(status, "pod_attn_probe_issue failed")
    return float(n.value)


def pod_attn_probe_colocation(variant: int, a: int, b: int, c: int, bytes_per_item: int, n_memory_items: int,
                              n_compute_items: int, compute_iters: int, counters: int, sink: int, stream: int = 0):
    _check(lib().pod_attn_probe_colocation(variant, ctypes.c_void_p(a), ctypes.c_void_p(b), ctypes.c_void_p(c),
                                           bytes_per_item, n_memory_items, n_compute_items, compute_iters,
                                           ctypes.c_void_p(counters), ctypes.c_void_p(sink), ctypes.c_void_p(stream)))


def pod_attn_role_for_ticket(ticket: int, prefill_ratio: int, decode_ratio: int, unit: int = 0) -> int:
    return int(lib().pod_attn_role_for_ticket(ticket, prefill_ratio, decode_ratio, unit))


def pod_attn_simulate_launch(plan: Plan, unit_of_wg, order):
    """Host model of one fused launch; returns (steps, first_role, seat_of_wg, item_owner, unit_owner)."""
    units, units_p = _i32(np.asarray(unit_of_wg))
    order, order_p = _i32(np.asarray(order))
    info = plan.info()
    first = np.full(max(units.size, 1), -2, dtype=np.int32)
    seat = np.full(max(units.size, 1), -1, dtype=np.int32)
    items = np.full(max(info.n_prefill_items, 1), -2, dtype=np.int32)
    dunits = np.full(max(info.n_decode_units, 1), -2, dtype=np.int32)
    p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    steps = lib().pod_attn_simulate_launch(plan.handle, units_p, int(units.size), order_p, int(order.size),
                                           p(first), p(seat), p(items), p(dunits))
    return (int(steps), first[:units.size], seat[:units.size], items[:info.n_prefill_items],
            dunits[:info.n_decode_units])


# ----------------------------------------------------------------------------------------------
# Convenience wrapper for torch tensors (marshalling only).
# ----------------------------------------------------------------------------------------------
class HybridAttention:
    """Plan + workspace for one batch shape; ``forward`` may be called once per layer."""

    def __init__(self, batch, *, policy=POLICY_AUTO, max_prefill_waves=0, decode_chunk=0,
                 prefill_split_len=0, n_compute_units=0):
        import torch
        self.torch = torch
        self.batch_meta = np.ascontiguousarray(batch.seq_meta, dtype=np.int32)
        self.params = make_params(
            n_prefill=batch.n_prefill, n_decode=batch.n_decode, n_q_heads=batch.n_q_heads,
            n_kv_heads=batch.n_kv_heads, head_dim=batch.head_dim, dtype=batch.dtype,
            softmax_scale=batch.softmax_scale, block_size=batch.block_size,
            max_blocks_per_seq=batch.max_blocks_per_seq, n_cache_rows=batch.n_cache_rows,
            n_blocks=batch.n_blocks, kv_seq_stride=batch.kv_seq_stride, policy=policy,
            max_prefill_waves=max_prefill_waves, decode_chunk=decode_chunk,
            prefill_split_len=prefill_split_len, n_compute_units=n_compute_units,
            kv_order=KV_HEAD_MAJOR if batch.head_major else KV_TOKEN_MAJOR)
        self.plan = pod_attn_plan_create(self.params, self.batch_meta)
        self.info = self.plan.info()
        dev = batch.k_cache.device
        self.ws_bytes = pod_attn_workspace_size(self.plan)
        self.workspace = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=dev)
        base = self.workspace.data_ptr()
        self.ws_ptr = (base + 255) & ~255
        self.seq_meta_dev = torch.from_numpy(self.batch_meta).to(dev)
        stream = torch.cuda.current_stream(dev).cuda_stream
        pod_attn_plan_upload(self.plan, self.ws_ptr, self.ws_bytes, stream)

    def forward(self, batch, out=None, mode=MODE_FUSED):
        torch = self.torch
        dev = batch.k_cache.device
        if out is None:
            out = torch.empty((batch.n_rows, batch.n_q_heads, batch.head_dim), dtype=batch.torch_dtype,
                              device=dev)
        ptr = lambda t: 0 if t is None or t.numel() == 0 else t.data_ptr()
        stream = torch.cuda.current_stream(dev).cuda_stream
        pod_attn_forward(ptr(batch.prefill_q), ptr(batch.decode_q), ptr(batch.k_cache), ptr(batch.v_cache),
                         self.seq_meta_dev.data_ptr(), ptr(batch.block_table), out.data_ptr(), self.plan,
                         self.ws_ptr, self.ws_bytes, mode, stream)
        return out

    def enable_trace(self):
        """Allocate a trace buffer (one record per workgroup) and switch tracing on."""
        n = max(self.info.n_prefill_items + (self.info.n_decode_units + 3) // 4, self.info.fused_grid, 1)
        self.trace = self.torch.zeros(n * 48, dtype=self.torch.uint8, device=self.workspace.device)
        pod_attn_plan_set_trace(self.plan, self.trace.data_ptr(), self.trace.numel())

    def read_trace(self) -> np.ndarray:
        self.torch.cuda.synchronize()
        return self.trace.cpu().numpy().view(TRACE_DTYPE)[: self.info.fused_grid].copy()

    def disable_trace(self):
        pod_attn_plan_set_trace(self.plan, 0, 0)

    def enable_event_log(self):
        """Allocate an event log (one record per prefill item and decode unit) and switch it on."""
        n = self.info.n_prefill_items + self.info.n_decode_units + 1
        self.evlog = self.torch.zeros(16 + n * 32, dtype=self.torch.uint8, device=self.workspace.device)
        pod_attn_plan_set_event_log(self.plan, self.evlog.data_ptr(), self.evlog.numel())

    def read_event_log(self) -> np.ndarray:
        """Records of the forward call made since the log was last read; clears the log."""
        self.torch.cuda.synchronize()
        raw = self.evlog.cpu().numpy()
        n = min(int(raw[:4].view(np.uint32)[0]), (raw.size - 16) // 32)
        ev = raw[16:16 + n * 32].view(EVENT_DTYPE).copy()
        self.evlog[:16].zero_()
        return ev

    def disable_event_log(self):
        pod_attn_plan_set_event_log(self.plan, 0, 0)

    def close(self):
        self.plan.close()
