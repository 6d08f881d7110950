"""ctypes binding of the QSAC C ABI (``include/qsac.h``): argument marshalling only.

Every step of the path runs in the HIP kernels of ``csrc/libqsac.so``.  There is no
fallback: ``load()`` raises if the library has not been built
(``python -m paper_2511_14510_amd.build``).  The functions carry the names of the C entry
points; ``Session`` is plumbing around them that owns the torch tensors (device memory,
pinned host memory, streams) a caller has to provide.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "csrc", "libqsac.so")
CALIB_LIB_PATH = os.path.join(HERE, "csrc", "libqsac_calib.so")

QSAC_F16, QSAC_BF16 = 0, 1
QSAC_OK, QSAC_EINVAL, QSAC_ENULL, QSAC_ERANGE = 0, -1, -2, -3
QSAC_EWORKSPACE, QSAC_EHIP, QSAC_ESTATE, QSAC_EALIGN, QSAC_ETIMEOUT = -4, -5, -6, -7, -8
QSAC_FLAG_DRY_RUN, QSAC_FLAG_SERIAL, QSAC_FLAG_SCORE_VALU, QSAC_FLAG_PROFILE, QSAC_FLAG_FILL_KERNEL = 1, 2, 4, 8, 16
QSAC_FLAG_PUSH_FILL, QSAC_FLAG_PUSH_HOLD, QSAC_FLAG_STAGGER = 32, 64, 128
QSAC_MAX_GROUP, QSAC_MAX_KV_HEADS, QSAC_HEAD_DIM = 8, 64, 128

EXPORTS = ("qsac_workspace_bytes", "qsac_workspace_layout", "qsac_init", "qsac_reset", "qsac_step",
           "qsac_get_stats", "qsac_free", "qsac_strerror", "qsac_last_hip_error", "qsac_num_stages",
           "qsac_stage_name", "qsac_get_stage_ms", "qsac_adaptive_thresholds", "qsac_reuse_difficulty",
           "qsac_graph_capture", "qsac_graph_launch", "qsac_graph_free", "qsac_step_static")
QSAC_STATIC_SCRATCH_BYTES = 32 << 20
CALIB_EXPORTS = ("qsac_calibration_copy", "qsac_calibration_read")


class qsac_config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("n_ctx", C.c_int64), ("k_max", C.c_int32), ("dtype", C.c_int32),
                ("q_head_importance", C.POINTER(C.c_float)), ("stream_main", C.c_void_p),
                ("stream_side", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("flags", C.c_int32), ("n_sink", C.c_int32), ("n_recent", C.c_int32), ("append_capacity", C.c_int32),
                ("push_threads", C.c_int32), ("push_wait_us", C.c_int32)]


class qsac_ws_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in
                ("valid", "set_sorted", "keys", "hist", "bm_new", "bm_eq", "bm_old", "miss_count", "miss_slot",
                 "miss_tok", "part_ml", "part_acc", "stats", "importance", "sel_r", "chunk_cnt", "fetch_tok", "push",
                 "total")] + \
               [("n_pad", C.c_int64), ("words", C.c_int32), ("max_splits", C.c_int32)]


class qsac_step_args(C.Structure):
    _fields_ = [("q", C.c_void_p), ("K_dev", C.c_void_p), ("K_src", C.c_void_p), ("V_src", C.c_void_p),
                ("K_slots", C.c_void_p), ("V_slots", C.c_void_p), ("slot_idx", C.c_void_p), ("prev_q", C.c_void_p),
                ("tau", C.POINTER(C.c_float)), ("n_tau", C.c_int32), ("k", C.c_int32), ("out", C.c_void_p),
                ("topk_idx", C.c_void_p), ("hit_mask", C.c_void_p), ("reuse_flags", C.c_void_p), ("sim", C.c_void_p),
                ("V_res", C.c_void_p), ("res_slot", C.POINTER(C.c_int8)), ("n_res", C.c_int32),
                ("K_app", C.c_void_p), ("V_app", C.c_void_p), ("n_app", C.c_int32), ("dev_params", C.c_void_p)]


class qsac_dev_params(C.Structure):
    _fields_ = [("tau", C.c_float * QSAC_MAX_KV_HEADS), ("n_app", C.c_int32), ("reserved", C.c_int32 * 3)]


class qsac_stats(C.Structure):
    _fields_ = [("steps", C.c_uint64), ("reuse_heads", C.c_uint64), ("miss_heads", C.c_uint64),
                ("slot_hits", C.c_uint64), ("slot_misses", C.c_uint64), ("bytes_filled_host", C.c_uint64),
                ("bytes_filled_dev", C.c_uint64), ("resident_rows", C.c_uint64), ("guided_selects", C.c_uint64),
                ("reserved", C.c_uint64 * 1)]


_lib = None
_calib = None


def load():
    """Loads the built library; raises if it is missing (there is no other implementation)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2511_14510_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.qsac_workspace_bytes.restype = C.c_size_t
        L.qsac_workspace_bytes.argtypes = [C.POINTER(qsac_config)]
        L.qsac_workspace_layout.argtypes = [C.POINTER(qsac_config), C.POINTER(qsac_ws_layout)]
        L.qsac_init.argtypes = [C.POINTER(qsac_config), C.POINTER(C.c_void_p)]
        L.qsac_reset.argtypes = [C.c_void_p]
        L.qsac_step.argtypes = [C.c_void_p, C.POINTER(qsac_step_args)]
        L.qsac_get_stats.argtypes = [C.c_void_p, C.POINTER(qsac_stats)]
        L.qsac_free.argtypes = [C.c_void_p]
        L.qsac_strerror.restype = C.c_char_p
        L.qsac_strerror.argtypes = [C.c_int]
        L.qsac_last_hip_error.restype = C.c_int
        L.qsac_num_stages.restype = C.c_int
        L.qsac_stage_name.restype = C.c_char_p
        L.qsac_stage_name.argtypes = [C.c_int]
        L.qsac_get_stage_ms.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
        L.qsac_graph_capture.argtypes = [C.c_void_p, C.POINTER(qsac_step_args), C.POINTER(C.c_void_p)]
        L.qsac_graph_launch.argtypes = [C.c_void_p]
        L.qsac_graph_free.argtypes = [C.c_void_p]
        L.qsac_step_static.argtypes = [C.POINTER(qsac_config), C.POINTER(qsac_step_args), C.c_int]
        fp = C.POINTER(C.c_float)
        L.qsac_adaptive_thresholds.argtypes = [fp, C.c_int32, C.c_float, C.c_float, fp]
        L.qsac_reuse_difficulty.argtypes = [fp, fp, C.c_int32, C.c_float, fp]
        _lib = L
    return _lib


def load_calib():
    """Loads the measurement-aid library (the copy and read-only kernels the benchmark is held against)."""
    global _calib
    if _calib is None:
        if not os.path.exists(CALIB_LIB_PATH):
            raise RuntimeError(f"{CALIB_LIB_PATH} is not built; run `python -m paper_2511_14510_amd.build`")
        L = C.CDLL(CALIB_LIB_PATH)
        L.qsac_calibration_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.qsac_calibration_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        _calib = L
    return _calib


class QsacError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {qsac_strerror(code)} ({code}), hip error {load().qsac_last_hip_error()}")


def qsac_strerror(code: int) -> str:
    return load().qsac_strerror(code).decode()


def qsac_workspace_bytes(cfg: qsac_config) -> int:
    return load().qsac_workspace_bytes(C.byref(cfg))


def qsac_workspace_layout(cfg: qsac_config) -> qsac_ws_layout:
    out = qsac_ws_layout()
    rc = load().qsac_workspace_layout(C.byref(cfg), C.byref(out))
    if rc:
        raise QsacError(rc, "qsac_workspace_layout")
    return out


def qsac_init(cfg: qsac_config) -> C.c_void_p:
    ctx = C.c_void_p()
    rc = load().qsac_init(C.byref(cfg), C.byref(ctx))
    if rc:
        raise QsacError(rc, "qsac_init")
    return ctx


def qsac_reset(ctx) -> None:
    rc = load().qsac_reset(ctx)
    if rc:
        raise QsacError(rc, "qsac_reset")


def qsac_step(ctx, args: qsac_step_args) -> None:
    rc = load().qsac_step(ctx, C.byref(args))
    if rc:
        raise QsacError(rc, "qsac_step")


def qsac_get_stats(ctx) -> dict:
    st = qsac_stats()
    rc = load().qsac_get_stats(ctx, C.byref(st))
    if rc:
        raise QsacError(rc, "qsac_get_stats")
    return {n: int(getattr(st, n)) for n in ("steps", "reuse_heads", "miss_heads", "slot_hits", "slot_misses",
                                             "bytes_filled_host", "bytes_filled_dev", "resident_rows",
                                             "guided_selects")}


def qsac_get_stage_ms(ctx):
    """(names, summed ms per stage, steps summed) of a context created with QSAC_FLAG_PROFILE."""
    L = load()
    n = L.qsac_num_stages()
    ms = (C.c_double * n)()
    steps = C.c_uint64()
    rc = L.qsac_get_stage_ms(ctx, ms, C.byref(steps))
    if rc:
        raise QsacError(rc, "qsac_get_stage_ms")
    return [L.qsac_stage_name(i).decode() for i in range(n)], list(ms), int(steps.value)


def qsac_calibration_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    rc = load_calib().qsac_calibration_copy(dst_ptr, src_ptr, nbytes, stream)
    if rc:
        raise QsacError(rc, "qsac_calibration_copy")


def qsac_calibration_read(src_ptr: int, nbytes: int, sink_ptr: int, stream: int = 0) -> None:
    rc = load_calib().qsac_calibration_read(src_ptr, nbytes, sink_ptr, stream)
    if rc:
        raise QsacError(rc, "qsac_calibration_read")


def qsac_graph_capture(ctx, args: qsac_step_args) -> C.c_void_p:
    g = C.c_void_p()
    rc = load().qsac_graph_capture(ctx, C.byref(args), C.byref(g))
    if rc:
        raise QsacError(rc, "qsac_graph_capture")
    return g


def qsac_graph_launch(graph) -> None:
    rc = load().qsac_graph_launch(graph)
    if rc:
        raise QsacError(rc, "qsac_graph_launch")


def qsac_graph_free(graph) -> None:
    rc = load().qsac_graph_free(graph)
    if rc:
        raise QsacError(rc, "qsac_graph_free")


def _floats(xs):
    return (C.c_float * len(xs))(*[float(x) for x in xs])


def qsac_adaptive_thresholds(importance, eta: float, p: float) -> list:
    """Eq. (3)-(5): per-head thresholds from head importance scores."""
    n = len(importance)
    out = (C.c_float * n)()
    rc = load().qsac_adaptive_thresholds(_floats(importance), n, eta, p, out)
    if rc:
        raise QsacError(rc, "qsac_adaptive_thresholds")
    return list(out)


def qsac_reuse_difficulty(tau, avg_sim, eps: float) -> list:
    """Section 4.4: D_i = tau_i - (avg_sim_i - eps)."""
    n = len(tau)
    out = (C.c_float * n)()
    rc = load().qsac_reuse_difficulty(_floats(tau), _floats(avg_sim), n, eps, out)
    if rc:
        raise QsacError(rc, "qsac_reuse_difficulty")
    return list(out)


def qsac_step_static(cfg: qsac_config, args: qsac_step_args, reset: bool) -> None:
    rc = load().qsac_step_static(C.byref(cfg), C.byref(args), int(bool(reset)))
    if rc:
        raise QsacError(rc, "qsac_step_static")


def qsac_free(ctx) -> None:
    rc = load().qsac_free(ctx)
    if rc:
        raise QsacError(rc, "qsac_free")


def make_config(B, Hq, Hkv, N, k_max, dtype, flags=0, importance=None, n_sink=0, n_recent=0,
                append_capacity=0, push_threads=0, push_wait_us=0) -> qsac_config:
    cfg = qsac_config()
    cfg.push_threads, cfg.push_wait_us = push_threads, push_wait_us
    cfg.n_sink, cfg.n_recent, cfg.append_capacity = n_sink, n_recent, append_capacity
    cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = B, Hq, Hkv, QSAC_HEAD_DIM
    cfg.n_ctx, cfg.k_max, cfg.dtype, cfg.flags = N, k_max, dtype, flags
    if importance is not None:
        arr = (C.c_float * len(importance))(*[float(x) for x in importance])
        cfg._keep = arr
        cfg.q_head_importance = C.cast(arr, C.POINTER(C.c_float))
    return cfg


class Session:
    """Owns the torch tensors of one layer's QSAC state and outputs and calls qsac_step on them.

    K_dev is the HBM copy read by the scoring pass; K_src / V_src are the fill sources (HBM
    tensors, or pinned host tensors, which HIP maps into the device address space).
    """

    def __init__(self, B, Hq, Hkv, N, k_max, dtype: str, K_dev, K_src, V_src, flags=0, importance=None,
                 side_stream=False, V_res=None, res_slot=None, n_sink=0, n_recent=0, K_app=None, V_app=None,
                 push_threads=0, push_wait_us=0):
        """V_res [B,n_res,N,128] (device) and res_slot [Hkv] make the KV heads with res_slot >= 0 resident."""
        import torch
        from .workload import DTYPE_CODES, TORCH_DTYPES
        assert torch.cuda.is_available(), "QSAC needs a GPU: there is no CPU path"
        self.torch = torch
        dev = torch.device("cuda:0")
        tdt = TORCH_DTYPES[dtype]
        P = B * Hkv
        self.B, self.Hq, self.Hkv, self.N, self.k_max, self.P = B, Hq, Hkv, N, k_max, P
        self.K_dev, self.K_src, self.V_src = K_dev, K_src, V_src
        self.V_res, self.res_slot = V_res, (None if res_slot is None else [int(x) for x in res_slot])
        if V_res is not None:
            assert V_res.is_cuda and V_res.is_contiguous() and V_res.dtype == tdt and len(self.res_slot) == Hkv
            assert V_res.shape == (B, V_res.shape[1], N, 128)
        for t in (K_dev, K_src, V_src):
            assert t.shape == (B, Hkv, N, 128) and t.dtype == tdt and t.is_contiguous()
        assert K_dev.is_cuda
        self.main = torch.cuda.Stream(device=dev)
        self.side = torch.cuda.Stream(device=dev) if side_stream else None
        self.K_app, self.V_app, self.n_app = K_app, V_app, 0
        cap = 0
        if K_app is not None:
            cap = K_app.shape[2]
            for t in (K_app, V_app):
                assert t.is_cuda and t.is_contiguous() and t.dtype == tdt and t.shape == (B, Hkv, cap, 128)
        cfg = make_config(B, Hq, Hkv, N, k_max, DTYPE_CODES[dtype], flags, importance, n_sink, n_recent, cap,
                          push_threads, push_wait_us)
        nbytes = qsac_workspace_bytes(cfg)
        if nbytes == 0:
            raise QsacError(QSAC_EINVAL, "qsac_workspace_bytes")
        self.layout = qsac_workspace_layout(cfg)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        cfg.workspace, cfg.workspace_bytes = self.workspace.data_ptr(), nbytes
        cfg.stream_main = self.main.cuda_stream
        cfg.stream_side = self.side.cuda_stream if self.side is not None else None
        self.cfg = cfg
        # cache state (caller-owned by the ABI)
        self.K_slots = torch.zeros((B, Hkv, k_max, 128), dtype=tdt, device=dev)
        self.V_slots = torch.zeros((B, Hkv, k_max, 128), dtype=tdt, device=dev)
        self.slot_idx = torch.full((B, Hkv, k_max), -1, dtype=torch.int32, device=dev)
        self.prev_q = torch.zeros((B, Hq, 128), dtype=tdt, device=dev)
        self.out = torch.zeros((B, Hq, 128), dtype=torch.float32, device=dev)
        self.reuse_flags = torch.zeros((B, Hkv), dtype=torch.uint8, device=dev)
        self.sim = torch.zeros((B, Hq), dtype=torch.float32, device=dev)
        self._k = None
        torch.cuda.synchronize()
        self.ctx = qsac_init(cfg)

    def _outputs_for(self, k):
        if self._k != k:
            t = self.torch
            self.topk_idx = t.zeros((self.B, self.Hkv, k), dtype=t.int32, device="cuda:0")
            self.hit_mask = t.zeros((self.B, self.Hkv, k), dtype=t.uint8, device="cuda:0")
            t.cuda.synchronize()  # the fills above run on torch's stream, the step on ours
            self._k = k

    def step(self, q, tau, k):
        """Enqueues one step on the session's main stream; q is a device tensor [B,Hq,128]."""
        qsac_step(self.ctx, self.step_args(q, tau, k))

    def step_args(self, q, tau, k, dev_params=None, n_app_bound=None):
        """The qsac_step_args of a step over this session's tensors.  With ``dev_params`` (a device tensor
        holding a qsac_dev_params) tau is ignored and n_app is the bound ``n_app_bound``."""
        self._outputs_for(k)
        a = qsac_step_args()
        if dev_params is None:
            taus = [float(tau)] if not hasattr(tau, "__len__") else [float(x) for x in tau]
            tau_arr = (C.c_float * len(taus))(*taus)
            a._keep_tau = tau_arr
            a.tau, a.n_tau = C.cast(tau_arr, C.POINTER(C.c_float)), len(taus)
        else:
            a.dev_params = dev_params.data_ptr()
        a.q, a.K_dev, a.K_src, a.V_src = q.data_ptr(), self.K_dev.data_ptr(), self.K_src.data_ptr(), self.V_src.data_ptr()
        a.K_slots, a.V_slots, a.slot_idx = self.K_slots.data_ptr(), self.V_slots.data_ptr(), self.slot_idx.data_ptr()
        a.prev_q, a.k = self.prev_q.data_ptr(), k
        a.out, a.topk_idx, a.hit_mask = self.out.data_ptr(), self.topk_idx.data_ptr(), self.hit_mask.data_ptr()
        a.reuse_flags, a.sim = self.reuse_flags.data_ptr(), self.sim.data_ptr()
        n_app = self.n_app if n_app_bound is None else n_app_bound
        if n_app:
            a.K_app, a.V_app, a.n_app = self.K_app.data_ptr(), self.V_app.data_ptr(), n_app
        if self.V_res is not None:
            rs = (C.c_int8 * self.Hkv)(*self.res_slot)
            a._keep_rs = rs
            a.V_res, a.res_slot, a.n_res = self.V_res.data_ptr(), C.cast(rs, C.POINTER(C.c_int8)), self.V_res.shape[1]
        self._last_q = q  # keep the tensor alive until the stream has consumed it
        return a

    def dev_params_table(self, taus, n_apps):
        """Device tensor [T, sizeof(qsac_dev_params)] (uint8) holding one qsac_dev_params per step: row t has the
        thresholds taus[t] (a scalar or one per KV head) and the append-buffer row count n_apps[t]."""
        t = self.torch
        size = C.sizeof(qsac_dev_params)
        host = t.zeros((len(taus), size), dtype=t.uint8)
        for i, (tau, n_app) in enumerate(zip(taus, n_apps)):
            tv = [float(tau)] * self.Hkv if not hasattr(tau, "__len__") else [float(x) for x in tau]
            host[i].view(t.float32)[:self.Hkv] = t.tensor(tv, dtype=t.float32)
            host[i].view(t.int32)[QSAC_MAX_KV_HEADS] = int(n_app)
        dev = host.cuda()
        t.cuda.synchronize()
        return dev

    def copy_on_main(self, dst, src):
        """dst <- src (device tensors) as an asynchronous copy ordered on the session's main stream."""
        with self.torch.cuda.stream(self.main):
            dst.copy_(src, non_blocking=True)

    def set_appended(self, n_app: int):
        """Number of valid rows of the append-only buffer from the next step on (the caller has written them)."""
        assert self.K_app is not None and 0 <= n_app <= self.K_app.shape[2]
        self.n_app = n_app

    def sync(self):
        self.main.synchronize()
        if self.side is not None:
            self.side.synchronize()

    def ws_view(self, name, dtype, shape):
        """A tensor view of one of the library's workspace arrays (for tests)."""
        t = self.torch
        off = getattr(self.layout, name)
        n = 1
        for s in shape:
            n *= s
        item = t.empty((), dtype=dtype).element_size()
        return self.workspace[off:off + n * item].view(dtype).view(*shape)

    def valid(self):
        return self.ws_view("valid", self.torch.int32, (self.P,))

    def reset(self):
        qsac_reset(self.ctx)

    def stats(self):
        return qsac_get_stats(self.ctx)

    def close(self):
        if self.ctx is not None:
            self.sync()
            qsac_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
