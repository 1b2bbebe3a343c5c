"""ctypes binding of libzbstage.so — argument marshalling only.

Every function here has the name of the C entry point it calls (include/zb_stage.h) minus
the ``zb_`` prefix; all arithmetic of the F / B / W passes, the schedule order and the
optimizer protocol runs inside the library.  PyTorch is used for exactly two things:
owning the device arena and the HIP stream.  There is no fallback: if the library is not
built (python paper_2401_10241_amd/build.py) importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np
# PyTorch ships its own copy of the HIP runtime; it must be the one already in the process when
# libzbstage.so is loaded, or the arena and the stream would belong to a different runtime.
import torch  # noqa: F401  (device memory and streams only)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libzbstage.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2401_10241_amd/build.py` "
                      "(there is no CPU fallback)")
lib = C.CDLL(_LIB_PATH)

# ---- enums (mirroring zb_stage.h) ---------------------------------------------------------
OK, EINVAL, EORDER, ENOMEM, EDEVICE, ESTATE = range(6)
STATUS_NAMES = ("ZB_OK", "ZB_EINVAL", "ZB_EORDER", "ZB_ENOMEM", "ZB_EDEVICE", "ZB_ESTATE")
FP32, BF16 = 0, 1
KIND = {"1F1B": 0, "H1": 1, "H2": 2}
PASS_F, PASS_B, PASS_W = 0, 1, 2
PARAM_INDEX = {n: i for i, n in enumerate(
    ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"))}
T_PARAM, T_GRAD, T_ADAM_M, T_ADAM_V = 0, 16, 32, 48
T_INPUT_X, T_INPUT_DY, T_OUTPUT_Y, T_OUTPUT_DX = 64, 65, 66, 67
T_FLAT_PARAMS, T_FLAT_GRADS, T_FLAT_ADAM_M, T_FLAT_ADAM_V = 80, 81, 82, 83
T_INPUT_IDS, T_TARGET_IDS, T_LOSS = 68, 69, 70
T_STAGE_PARAM, T_STAGE_GRAD, T_STAGE_ADAM_M, T_STAGE_ADAM_V = 96, 104, 112, 120
ROLE = {"middle": 0, "first": 1, "last": 2}
STAGE_PARAM_INDEX = {"emb_tok": 0, "emb_pos": 1, "lnf_g": 2, "lnf_b": 3, "w_head": 4}
S_QKV_IN, S_PROJ_IN, S_FC1_IN, S_FC2_IN, S_QKV_DOUT, S_PROJ_DOUT, S_FC1_DOUT, S_FC2_DOUT = range(8)
OUTCOME_NAMES = ("COMMITTED", "SKIPPED_LOCAL", "ROLLED_BACK_NONFINITE", "ROLLED_BACK_RECLIPPED",
                 "DEFERRED_CLIPPED", "DEFERRED_SKIPPED")


class zb_op(C.Structure):
    _fields_ = [("pass_", C.c_int32), ("mb", C.c_int32)]


class zb_config(C.Structure):
    _fields_ = [("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("seq", C.c_int32), ("mb_size", C.c_int32), ("max_microbatches", C.c_int32),
                ("max_pending_b", C.c_int32), ("max_pending_w", C.c_int32), ("max_inflight", C.c_int32),
                ("dtype", C.c_int32), ("journal", C.c_int32), ("group_w", C.c_int32), ("fuse_bw", C.c_int32), ("chunks", C.c_int32), ("role", C.c_int32), ("vocab", C.c_int32),
                ("ln_eps", C.c_float), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
                ("weight_decay", C.c_float), ("clip", C.c_float), ("hip_stream", C.c_void_p),
                ("arena", C.c_void_p), ("arena_bytes", C.c_size_t)]


class zb_global_state(C.Structure):
    _fields_ = [("prev_sq", C.c_double), ("rest_sq", C.c_double), ("prev_nonfinite", C.c_int32),
                ("rest_nonfinite", C.c_int32), ("force_optimistic", C.c_int32)]


class zb_step_report(C.Structure):
    _fields_ = [("outcome", C.c_int32), ("stepped_optimistically", C.c_int32), ("local_sq", C.c_double),
                ("global_norm", C.c_double), ("clip_coef", C.c_double), ("t", C.c_int64),
                ("alg1_mismatch_elems", C.c_uint64)]


class zb_pass_times(C.Structure):
    _fields_ = [("t_f", C.c_double), ("t_b", C.c_double), ("t_w", C.c_double), ("t_comm", C.c_double)]


class zb_memory_model(C.Structure):
    _fields_ = [("m_limit", C.c_double), ("m_b", C.c_double), ("m_w", C.c_double)]


class zb_kernel_stat(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


_P = C.POINTER
_sig = {
    "zb_config_defaults": [_P(zb_config)],
    "zb_stage_arena_bytes": [_P(zb_config), _P(C.c_size_t)],
    "zb_stage_init": [_P(zb_config), _P(C.c_void_p)],
    "zb_stage_free": [C.c_void_p],
    "zb_stage_flat_count": [C.c_void_p, _P(C.c_size_t)],
    "zb_begin_iteration": [C.c_void_p, C.c_int32, C.c_int32],
    "zb_forward": [C.c_void_p, C.c_int32],
    "zb_backward_input": [C.c_void_p, C.c_int32],
    "zb_backward_weight": [C.c_void_p, C.c_int32],
    "zb_backward_weight_group": [C.c_void_p, _P(C.c_int32), C.c_int32],
    "zb_backward_fused": [C.c_void_p, C.c_int32],
    "zb_schedule_order": [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P(zb_op), C.c_int32, _P(C.c_int32)],
    "zb_schedule_stash_need": [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P(C.c_int32), _P(C.c_int32),
                               _P(C.c_int32)],
    "zb_run_schedule": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32],
    "zb_order_stash_need": [_P(zb_op), C.c_int32, _P(C.c_int32), _P(C.c_int32), _P(C.c_int32)],
    "zb_run_order": [C.c_void_p, _P(zb_op), C.c_int32],
    "zb_simulate_pipeline": [C.c_int32, C.c_int32, _P(zb_op), _P(zb_pass_times), C.c_int32, _P(C.c_double),
                             _P(C.c_double), _P(C.c_double)],
    "zb_auto_schedule": [C.c_int32, C.c_int32, _P(zb_pass_times), _P(zb_memory_model), C.c_int32, C.c_int32,
                         _P(zb_op)],
    "zb_auto_schedule_search": [C.c_int32, C.c_int32, _P(zb_pass_times), _P(zb_memory_model), _P(zb_op),
                                _P(C.c_double), _P(C.c_double), _P(C.c_int32), _P(C.c_int32)],
    "zb_order_memory_peak": [_P(zb_op), C.c_int32, C.c_double, C.c_double, _P(C.c_double)],
    "zb_order_group_w": [_P(zb_op), C.c_int32, C.c_int32, _P(zb_op)],
    "zb_simulate_pipeline_w_runs": [C.c_int32, C.c_int32, _P(zb_op), _P(zb_pass_times), C.c_double, _P(C.c_double),
                                    _P(C.c_double)],
    "zb_schedule_order_v": [C.c_int32, C.c_int32, _P(zb_op)],
    "zb_simulate_pipeline_v": [C.c_int32, C.c_int32, _P(zb_op), _P(zb_pass_times), _P(C.c_double), _P(C.c_double),
                               _P(C.c_double)],
    "zb_optimizer_step_validated": [C.c_void_p, _P(zb_global_state), _P(zb_step_report)],
    "zb_get_tensor": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t],
    "zb_set_tensor": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t],
    "zb_inject": [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_float],
    "zb_get_stash_columns": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _P(C.c_int32), C.c_int32, C.c_void_p],
    "zb_synchronize": [C.c_void_p],
    "zb_stage_model_flops": [C.c_void_p, C.c_int32, _P(C.c_double)],
    "zb_stage_stash_bytes": [C.c_void_p, _P(C.c_double), _P(C.c_double)],
    "zb_profile_enable": [C.c_void_p, C.c_int32],
    "zb_profile_read": [C.c_void_p, _P(zb_kernel_stat), C.c_int32, _P(C.c_int32)],
    "zb_grad_norm_static": [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p],
}
for _name, _args in _sig.items():
    _f = getattr(lib, _name)
    _f.argtypes = _args
    _f.restype = C.c_int
lib.zb_last_error.argtypes = [C.c_void_p]
lib.zb_last_error.restype = C.c_char_p
EXPORTED = tuple(_sig) + ("zb_last_error",)


class ZbError(RuntimeError):
    def __init__(self, status: int, msg: str = ""):
        self.status = status
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {msg}")


def schedule_order(p: int, stage: int, m: int, kind: str) -> List[Tuple[int, int]]:
    """zb_schedule_order: per-stage list of (pass, microbatch)."""
    buf = (zb_op * (3 * max(m, 1)))()
    n = C.c_int32(0)
    rc = lib.zb_schedule_order(p, stage, m, KIND[kind], buf, 3 * max(m, 1), C.byref(n))
    if rc != OK:
        raise ZbError(rc, "zb_schedule_order")
    return [(buf[i].pass_, buf[i].mb) for i in range(n.value)]


def schedule_stash_need(p: int, stage: int, m: int, kind: str) -> Tuple[int, int, int]:
    """zb_schedule_stash_need: (max pending-B, max pending-W, max in-flight)."""
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    rc = lib.zb_schedule_stash_need(p, stage, m, KIND[kind], C.byref(a), C.byref(b), C.byref(c))
    if rc != OK:
        raise ZbError(rc, "zb_schedule_stash_need")
    return a.value, b.value, c.value


def _pack_order(ops) -> "C.Array":
    buf = (zb_op * max(len(ops), 1))()
    for q, (c, k) in enumerate(ops):
        buf[q].pass_, buf[q].mb = int(c), int(k)
    return buf


def _pack_orders(orders) -> Tuple["C.Array", int, int]:
    p = len(orders)
    n = len(orders[0]) if p else 0
    if p == 0 or n == 0 or n % 3 or any(len(o) != n for o in orders):
        raise ZbError(EINVAL, "orders must be p lists of 3m (pass, microbatch) pairs")
    return _pack_order([op for o in orders for op in o]), p, n // 3


def _unpack_orders(buf, p: int, m: int) -> List[List[Tuple[int, int]]]:
    return [[(buf[i * 3 * m + q].pass_, buf[i * 3 * m + q].mb) for q in range(3 * m)] for i in range(p)]


def order_stash_need(ops) -> Tuple[int, int, int]:
    """zb_order_stash_need: (max pending-B, max pending-W, max in-flight) of an explicit stage order."""
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    rc = lib.zb_order_stash_need(_pack_order(ops), len(ops), C.byref(a), C.byref(b), C.byref(c))
    if rc != OK:
        raise ZbError(rc, "zb_order_stash_need")
    return a.value, b.value, c.value


def simulate_pipeline(orders, t_f: float, t_b: float, t_w: float, t_comm: float = 0.0,
                      fused_backward: bool = False) -> Tuple[float, float, List[float]]:
    """zb_simulate_pipeline: (cost, bubble rate, per-stage spans) of p stage orders."""
    buf, p, m = _pack_orders(orders)
    t = zb_pass_times(t_f, t_b, t_w, t_comm)
    cost, rate = C.c_double(0), C.c_double(0)
    spans = (C.c_double * p)()
    rc = lib.zb_simulate_pipeline(p, m, buf, C.byref(t), int(fused_backward), C.byref(cost), C.byref(rate), spans)
    if rc != OK:
        raise ZbError(rc, "zb_simulate_pipeline")
    return cost.value, rate.value, list(spans)


def auto_schedule(p: int, m: int, t_f: float, t_b: float, t_w: float, t_comm: float, m_limit: float,
                  m_b: float, m_w: float, extra_warmup_f: bool = False,
                  skip_f: bool = False) -> List[List[Tuple[int, int]]]:
    """zb_auto_schedule: the heuristic's p stage orders for one setting of its two options."""
    buf = (zb_op * max(3 * p * m, 1))()
    t = zb_pass_times(t_f, t_b, t_w, t_comm)
    mm = zb_memory_model(m_limit, m_b, m_w)
    rc = lib.zb_auto_schedule(p, m, C.byref(t), C.byref(mm), int(extra_warmup_f), int(skip_f), buf)
    if rc != OK:
        raise ZbError(rc, "zb_auto_schedule")
    return _unpack_orders(buf, p, m)


def auto_schedule_search(p: int, m: int, t_f: float, t_b: float, t_w: float, t_comm: float, m_limit: float,
                         m_b: float, m_w: float):
    """zb_auto_schedule_search: (orders, cost, bubble rate, (extra_warmup_f, skip_f))."""
    buf = (zb_op * max(3 * p * m, 1))()
    t = zb_pass_times(t_f, t_b, t_w, t_comm)
    mm = zb_memory_model(m_limit, m_b, m_w)
    cost, rate = C.c_double(0), C.c_double(0)
    ew, sk = C.c_int32(0), C.c_int32(0)
    rc = lib.zb_auto_schedule_search(p, m, C.byref(t), C.byref(mm), buf, C.byref(cost), C.byref(rate),
                                     C.byref(ew), C.byref(sk))
    if rc != OK:
        raise ZbError(rc, "zb_auto_schedule_search")
    return _unpack_orders(buf, p, m), cost.value, rate.value, (bool(ew.value), bool(sk.value))


def schedule_order_v(p: int, m: int) -> List[List[Tuple[int, int]]]:
    """zb_schedule_order_v: ZB-V orders of all p workers as (pass, virtual microbatch = chunk * m + mb)."""
    buf = (zb_op * max(6 * p * m, 1))()
    rc = lib.zb_schedule_order_v(p, m, buf)
    if rc != OK:
        raise ZbError(rc, "zb_schedule_order_v")
    return [[(buf[i * 6 * m + q].pass_, buf[i * 6 * m + q].mb) for q in range(6 * m)] for i in range(p)]


def simulate_pipeline_v(orders, m: int, t_f: float, t_b: float, t_w: float,
                        t_comm: float = 0.0) -> Tuple[float, float, List[float]]:
    """zb_simulate_pipeline_v: (cost, bubble rate, per-worker spans); times of one chunk's pass."""
    p = len(orders)
    buf = _pack_order([op for o in orders for op in o])
    t = zb_pass_times(t_f, t_b, t_w, t_comm)
    cost, rate = C.c_double(0), C.c_double(0)
    spans = (C.c_double * p)()
    rc = lib.zb_simulate_pipeline_v(p, m, buf, C.byref(t), C.byref(cost), C.byref(rate), spans)
    if rc != OK:
        raise ZbError(rc, "zb_simulate_pipeline_v")
    return cost.value, rate.value, list(spans)


def simulate_pipeline_w_runs(orders, t_f: float, t_b: float, t_w: float, t_comm: float,
                             t_w_next: float) -> Tuple[float, List[float]]:
    """zb_simulate_pipeline_w_runs: (cost, per-stage spans); a W right behind a W takes t_w_next."""
    buf, p, m = _pack_orders(orders)
    t = zb_pass_times(t_f, t_b, t_w, t_comm)
    cost = C.c_double(0)
    spans = (C.c_double * p)()
    rc = lib.zb_simulate_pipeline_w_runs(p, m, buf, C.byref(t), t_w_next, C.byref(cost), spans)
    if rc != OK:
        raise ZbError(rc, "zb_simulate_pipeline_w_runs")
    return cost.value, list(spans)


def order_group_w(ops, group: int) -> List[Tuple[int, int]]:
    """zb_order_group_w: the order with the W passes of its steady state run `group` at a time."""
    out = (zb_op * max(len(ops), 1))()
    rc = lib.zb_order_group_w(_pack_order(ops), len(ops), group, out)
    if rc != OK:
        raise ZbError(rc, "zb_order_group_w")
    return [(out[i].pass_, out[i].mb) for i in range(len(ops))]


def order_memory_peak(ops, m_b: float, m_w: float) -> float:
    """zb_order_memory_peak."""
    peak = C.c_double(0)
    rc = lib.zb_order_memory_peak(_pack_order(ops), len(ops), m_b, m_w, C.byref(peak))
    if rc != OK:
        raise ZbError(rc, "zb_order_memory_peak")
    return peak.value


GRAD_NORM_STATIC_MAX_FLOATS = 1 << 30


def grad_norm_static(grads_ptr: int, n: int, sq_out_ptr: int, nonfinite_out_ptr: int, stream_handle: int = 0):
    """zb_grad_norm_static: all three pointers are device addresses (ints), stream_handle a hipStream_t or 0."""
    rc = lib.zb_grad_norm_static(grads_ptr, n, sq_out_ptr, nonfinite_out_ptr, stream_handle or None)
    if rc != OK:
        raise ZbError(rc, "zb_grad_norm_static")


@dataclass
class StepReport:
    outcome: int
    stepped_optimistically: bool
    local_sq: float
    global_norm: float
    clip_coef: float
    t: int
    alg1_mismatch_elems: int

    @property
    def outcome_name(self) -> str:
        return OUTCOME_NAMES[self.outcome]


class Stage:
    """One pipeline stage living on the current CUDA/HIP device."""

    def __init__(self, *, layers, hidden, heads, ffn, seq, mb_size=1, dtype="bf16", max_microbatches,
                 max_pending_b, max_pending_w, max_inflight, journal=True, group_w=True, fuse_bw=False, chunks=1,
                 role="middle", vocab=0, ln_eps=1e-5, lr=1e-4, beta1=0.9,
                 beta2=0.95, adam_eps=1e-8, weight_decay=0.01, clip=1.0, device="cuda:0", stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the zero-bubble stage runs only on the device (no CPU fallback)")
        self._torch = torch
        self.device = torch.device(device)
        cfg = zb_config()
        lib.zb_config_defaults(C.byref(cfg))
        cfg.layers, cfg.hidden, cfg.heads, cfg.ffn, cfg.seq, cfg.mb_size = layers, hidden, heads, ffn, seq, mb_size
        cfg.max_microbatches, cfg.max_pending_b = max_microbatches, max_pending_b
        cfg.max_pending_w, cfg.max_inflight = max_pending_w, max_inflight
        cfg.dtype = BF16 if dtype == "bf16" else FP32
        cfg.journal = 1 if journal else 0
        cfg.group_w = 1 if group_w else 0
        cfg.fuse_bw = 1 if fuse_bw else 0
        cfg.chunks = chunks
        cfg.role, cfg.vocab = ROLE[role], vocab
        self.role, self.vocab, self.seq = role, vocab, seq
        cfg.ln_eps, cfg.lr, cfg.beta1, cfg.beta2 = ln_eps, lr, beta1, beta2
        cfg.adam_eps, cfg.weight_decay, cfg.clip = adam_eps, weight_decay, clip
        need = C.c_size_t(0)
        rc = lib.zb_stage_arena_bytes(C.byref(cfg), C.byref(need))
        if rc != OK:
            raise ZbError(rc, "zb_stage_arena_bytes: invalid configuration")
        self.arena_bytes = need.value
        with torch.cuda.device(self.device):
            self._arena = torch.empty(need.value + 256, dtype=torch.uint8, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        base = (self._arena.data_ptr() + 255) // 256 * 256
        cfg.arena, cfg.arena_bytes = base, need.value
        cfg.hip_stream = self.stream.cuda_stream
        self.cfg = cfg
        self.tokens, self.hidden = seq * mb_size, hidden
        h = C.c_void_p(None)
        with torch.cuda.device(self.device):
            rc = lib.zb_stage_init(C.byref(cfg), C.byref(h))
        if rc != OK or not h.value:
            raise ZbError(rc, "zb_stage_init")
        self._h = h
        n = C.c_size_t(0)
        lib.zb_stage_flat_count(self._h, C.byref(n))
        self.flat_count = n.value

    # -- helpers ------------------------------------------------------------------------
    def _call(self, fn, *args):
        with self._torch.cuda.device(self.device):
            rc = fn(self._h, *args)
        if rc != OK:
            raise ZbError(rc, lib.zb_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib.zb_stage_free(self._h)
            self._h = C.c_void_p(None)
            self._arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C entry points ---------------------------------------------------------------
    def begin_iteration(self, it: int, m: int):
        self._call(lib.zb_begin_iteration, it, m)

    def forward(self, mb: int):
        self._call(lib.zb_forward, mb)

    def backward_input(self, mb: int):
        self._call(lib.zb_backward_input, mb)

    def backward_weight(self, mb: int):
        self._call(lib.zb_backward_weight, mb)

    def backward_fused(self, mb: int):
        self._call(lib.zb_backward_fused, mb)

    def backward_weight_group(self, mbs):
        arr = (C.c_int32 * max(len(mbs), 1))(*[int(k) for k in mbs])
        self._call(lib.zb_backward_weight_group, arr, len(mbs))

    def run_schedule(self, p: int, stage: int, m: int, kind: str):
        self._call(lib.zb_run_schedule, p, stage, m, KIND[kind])

    def run_order(self, ops):
        self._call(lib.zb_run_order, _pack_order(ops), len(ops))

    def optimizer_step_validated(self, prev_sq=0.0, rest_sq=0.0, prev_nonfinite=False, rest_nonfinite=False,
                                 force_optimistic=False, want_report=True) -> Optional[StepReport]:
        gs = zb_global_state(prev_sq, rest_sq, int(prev_nonfinite), int(rest_nonfinite), int(force_optimistic))
        if not want_report:
            self._call(lib.zb_optimizer_step_validated, C.byref(gs), None)
            return None
        rep = zb_step_report()
        self._call(lib.zb_optimizer_step_validated, C.byref(gs), C.byref(rep))
        return StepReport(rep.outcome, bool(rep.stepped_optimistically), rep.local_sq, rep.global_norm,
                          rep.clip_coef, rep.t, rep.alg1_mismatch_elems)

    def stage_param_shape(self, index: int):
        h, v = self.cfg.hidden, self.vocab
        return [(v, h), (self.seq, h), (h,), (h,), (h, v)][index]

    def set_ids(self, what: int, mb: int, ids):
        """zb_set_tensor for T_INPUT_IDS / T_TARGET_IDS: int32 [tokens]."""
        v = np.ascontiguousarray(ids, np.int32)
        self._call(lib.zb_set_tensor, what, 0, mb, v.ctypes.data_as(C.c_void_p), v.nbytes)

    def get_ids(self, what: int, mb: int) -> np.ndarray:
        out = np.empty(self.tokens, np.int32)
        self._call(lib.zb_get_tensor, what, 0, mb, out.ctypes.data_as(C.c_void_p), out.nbytes)
        return out

    def get_loss(self, mb: int) -> float:
        out = np.empty(1, np.float32)
        self._call(lib.zb_get_tensor, T_LOSS, 0, mb, out.ctypes.data_as(C.c_void_p), out.nbytes)
        return float(out[0])

    def set_stage_params(self, extra):
        """extra: dict name -> fp32 array (emb_tok, emb_pos / lnf_g, lnf_b, w_head)."""
        for name, value in extra.items():
            self.set_tensor(T_STAGE_PARAM + STAGE_PARAM_INDEX[name], 0, 0, value)

    def get_stage_group(self, base: int):
        names = ("emb_tok", "emb_pos") if self.role == "first" else ("lnf_g", "lnf_b", "w_head")
        return {n: self.get_tensor(base + STAGE_PARAM_INDEX[n]) for n in names}

    def _count(self, what: int) -> int:
        if 96 <= what < 128:
            return int(np.prod(self.stage_param_shape((what - 96) % 8)))
        if what < 64:
            shp = self.param_shape(what % 16)
            return int(np.prod(shp))
        if what < 80:
            return self.tokens * self.hidden
        return self.flat_count

    def param_shape(self, index: int):
        h, f = self.cfg.hidden, self.cfg.ffn
        return [(h,), (h,), (h, 3 * h), (3 * h,), (h, h), (h,), (h,), (h,), (h, f), (f,), (f, h), (h,)][index]

    def get_tensor(self, what: int, layer: int = 0, mb: int = 0) -> np.ndarray:
        out = np.empty(self._count(what), np.float32)
        self._call(lib.zb_get_tensor, what, layer, mb, out.ctypes.data_as(C.c_void_p), out.nbytes)
        if 96 <= what < 128:
            return out.reshape(self.stage_param_shape((what - 96) % 8))
        if what < 64:
            return out.reshape(self.param_shape(what % 16))
        if what < 80:
            return out.reshape(self.tokens, self.hidden)
        return out

    def set_tensor(self, what: int, layer: int, mb: int, value: np.ndarray):
        v = np.ascontiguousarray(value, np.float32)
        self._call(lib.zb_set_tensor, what, layer, mb, v.ctypes.data_as(C.c_void_p), v.nbytes)

    def get_stash_columns(self, which: int, layer: int, mb: int, cols) -> np.ndarray:
        """zb_get_stash_columns: [tokens, len(cols)] fp32."""
        idx = (C.c_int32 * len(cols))(*[int(c) for c in cols])
        out = np.empty((self.tokens, len(cols)), np.float32)
        self._call(lib.zb_get_stash_columns, which, layer, mb, idx, len(cols), out.ctypes.data_as(C.c_void_p))
        return out

    def inject(self, what: int, mb: int, elem: int, value: float):
        self._call(lib.zb_inject, what, mb, elem, value)

    def synchronize(self):
        self._call(lib.zb_synchronize)

    def model_flops(self, m: int) -> float:
        out = C.c_double(0)
        self._call(lib.zb_stage_model_flops, m, C.byref(out))
        return out.value

    def stash_bytes(self) -> Tuple[float, float]:
        """zb_stage_stash_bytes: (bytes held per microbatch after F, after B)."""
        a, b = C.c_double(0), C.c_double(0)
        self._call(lib.zb_stage_stash_bytes, C.byref(a), C.byref(b))
        return a.value, b.value

    def profile_enable(self, on: bool):
        self._call(lib.zb_profile_enable, int(on))

    def profile_read(self):
        buf = (zb_kernel_stat * 32)()
        n = C.c_int32(0)
        self._call(lib.zb_profile_read, buf, 32, C.byref(n))
        return [dict(name=buf[i].name.decode(), launches=buf[i].launches, total_ms=buf[i].total_ms,
                     flops=buf[i].flops, bytes=buf[i].bytes) for i in range(n.value)]

    # -- convenience built only from the calls above ----------------------------------------
    def set_params(self, params):
        """params: list (one per layer) of dicts name -> fp32 array."""
        for l, P in enumerate(params):
            for name, idx in PARAM_INDEX.items():
                self.set_tensor(T_PARAM + idx, l, 0, P[name])

    def get_group(self, base: int):
        return [{name: self.get_tensor(base + idx, l, 0) for name, idx in PARAM_INDEX.items()}
                for l in range(self.cfg.layers)]
