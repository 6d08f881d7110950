"""ctypes face of the QSAC oracle (``qsac_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.

All tensors cross this boundary as C-contiguous numpy arrays; 16-bit floats are
passed as their ``uint16`` bit patterns together with ``dtype`` (0 = IEEE
binary16, 1 = bfloat16).  Every function cites the passage of the paper
(LiteCache, arXiv 2511.14510) that its C counterpart follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

F16, BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qsac_oracle.c")
# QSAC_ORACLE_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer (host code only;
# the process then needs the sanitizer runtime preloaded, see tests/test_oracle_sanitized.py).
SANITIZE = os.environ.get("QSAC_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libqsac_oracle_san.so" if SANITIZE else "libqsac_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP over independent pairs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"] if SANITIZE else []
        subprocess.check_call(
            ["gcc", "-O1" if SANITIZE else "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-D_GNU_SOURCE"] + extra + ["-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Ext(C.Structure):
    _fields_ = [("n_sink", C.c_int32), ("n_recent", C.c_int32), ("n_app", C.c_int32), ("app_cap", C.c_int32),
                ("K_app", C.c_void_p), ("V_app", C.c_void_p)]


class _Dims(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("N", C.c_int64), ("k", C.c_int32), ("k_max", C.c_int32), ("dtype", C.c_int32)]


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.qo_widen.restype = C.c_double
        L.qo_widen.argtypes = [C.c_uint16, C.c_int]
        L.qo_cossim.restype = C.c_double
        L.qo_cossim.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        L.qo_aggregate.restype = C.c_double
        L.qo_aggregate.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.qo_adaptive_tau.restype = C.c_double
        L.qo_adaptive_tau.argtypes = [C.c_double, C.c_double, C.c_double]
        L.qo_reuse_difficulty.restype = C.c_double
        L.qo_reuse_difficulty.argtypes = [C.c_double, C.c_double, C.c_double]
        L.qo_scores.restype = None
        L.qo_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_void_p]
        L.qo_topk.restype = C.c_int
        L.qo_topk.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]
        L.qo_attention.restype = None
        L.qo_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                   C.c_void_p, C.c_void_p]
        L.qo_diff.restype = C.c_int
        L.qo_diff.argtypes = [C.c_int, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_void_p]
        L.qo_step.restype = C.c_int
        L.qo_step.argtypes = [C.POINTER(_Dims)] + [C.c_void_p] * 22 + [C.POINTER(_Ext)]
        L.qo_attention_hybrid.restype = None
        L.qo_attention_hybrid.argtypes = [C.c_void_p] * 3 + [C.c_int] + [C.c_void_p] * 2 + [C.c_int] * 3 + [C.c_void_p] * 2
        L.qo_num_threads.restype = C.c_int
        L.qo_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a, shape=None):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def widen(bits, dtype: int) -> np.ndarray:
    """16-bit patterns -> fp64, exactly (no arithmetic of the method)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    L = lib()
    return np.array([L.qo_widen(int(x), dtype) for x in b.ravel()], dtype=np.float64).reshape(b.shape)


def cossim(a, b, dtype: int) -> float:
    """CosSim of Section 3.1; zero-norm argument gives -1."""
    a, b = _u16(a), _u16(b)
    assert a.shape == b.shape and a.ndim == 1
    return lib().qo_cossim(_p(a), _p(b), a.shape[0], dtype)


def aggregate(sim, weights=None) -> float:
    """Eq. (2): importance-weighted harmonic aggregation over a query group."""
    s = np.ascontiguousarray(sim, dtype=np.float64)
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float64)
    return lib().qo_aggregate(_p(s), _p(w), s.shape[0])


def adaptive_tau(importance: float, eta: float, p: float) -> float:
    """Eq. (3)-(5): per-head reuse threshold from a head importance score."""
    return lib().qo_adaptive_tau(importance, eta, p)


def reuse_difficulty(tau: float, avg_sim: float, eps: float) -> float:
    """Section 4.4: D_i = tau_i - (s_hat_i - eps)."""
    return lib().qo_reuse_difficulty(tau, avg_sim, eps)


def scores(q, K, dtype: int) -> np.ndarray:
    """Eq. (1) over a query group: S[n] = max_g q_g . k_n.  q [G,D], K [N,D]."""
    q, K = _u16(q), _u16(K)
    G, D = q.shape
    N = K.shape[0]
    assert K.shape == (N, D)
    S = np.empty(N, dtype=np.float64)
    lib().qo_scores(_p(q), _p(K), G, N, D, dtype, _p(S))
    return S


def topk(S, k: int):
    """k best of S under (score desc, index asc); ascending indices and the k-th score."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    idx = np.empty(k, dtype=np.int32)
    kth = C.c_double(float("nan"))
    rc = lib().qo_topk(_p(S), S.shape[0], k, _p(idx), C.addressof(kth))
    if rc:
        raise ValueError(f"qo_topk failed ({rc})")
    return idx, kth.value


def attention(q, Kc, Vc, dtype: int):
    """softmax(q Kc^T / sqrt(D)) Vc over the given rows (Section 2.1); returns (out, weights)."""
    q, Kc, Vc = _u16(q), _u16(Kc), _u16(Vc)
    k, D = Kc.shape
    assert q.shape == (D,) and Vc.shape == (k, D)
    out = np.empty(D, dtype=np.float64)
    w = np.empty(k, dtype=np.float64)
    lib().qo_attention(_p(q), _p(Kc), _p(Vc), k, D, dtype, _p(out), _p(w))
    return out, w


def attention_hybrid(q, Kc, Vc, Ka, Va, dtype: int):
    """Attention over the cached rows followed by the appended rows (Section 6.2); returns (out, weights)."""
    q, Kc, Vc, Ka, Va = _u16(q), _u16(Kc), _u16(Vc), _u16(Ka), _u16(Va)
    k, D = Kc.shape
    na = Ka.shape[0]
    assert q.shape == (D,) and Vc.shape == (k, D) and Ka.shape == (na, D) and Va.shape == (na, D)
    out = np.empty(D, dtype=np.float64)
    w = np.empty(k + na, dtype=np.float64)
    lib().qo_attention_hybrid(_p(q), _p(Kc), _p(Vc), k, _p(Ka), _p(Va), na, D, dtype, _p(out), _p(w))
    return out, w


def diff(valid: bool, N: int, slot_idx, topk_idx):
    """Slot diff of Algorithm 1's transfer step.  Returns (slot_idx', hit_mask, miss_slot, miss_tok)."""
    sl = np.array(slot_idx, dtype=np.int32, copy=True)
    tk = np.ascontiguousarray(topk_idx, dtype=np.int32)
    k = tk.shape[0]
    hm = np.empty(k, dtype=np.uint8)
    ms = np.empty(k, dtype=np.int32)
    mt = np.empty(k, dtype=np.int32)
    m = lib().qo_diff(int(bool(valid)), N, k, _p(sl), _p(tk), _p(hm), _p(ms), _p(mt))
    if m < 0:
        raise ValueError(f"qo_diff failed ({m})")
    return sl, hm, ms[:m].copy(), mt[:m].copy()


@dataclass
class State:
    """Cache state of every (batch, KV head) pair: Algorithm 1's q_c, K_c, V_c plus slot bookkeeping."""
    valid: np.ndarray      # [P] u8
    prev_q: np.ndarray     # [B,Hq,D] u16
    slot_idx: np.ndarray   # [P,k_max] i32
    K_slots: np.ndarray    # [P,k_max,D] u16
    V_slots: np.ndarray    # [P,k_max,D] u16

    @staticmethod
    def empty(B, Hq, Hkv, D, k_max):
        P = B * Hkv
        return State(np.zeros(P, np.uint8), np.zeros((B, Hq, D), np.uint16),
                     np.full((P, k_max), -1, np.int32), np.zeros((P, k_max, D), np.uint16),
                     np.zeros((P, k_max, D), np.uint16))

    def copy(self):
        return State(*(a.copy() for a in (self.valid, self.prev_q, self.slot_idx, self.K_slots, self.V_slots)))


@dataclass
class StepResult:
    out: np.ndarray          # [B,Hq,D] f64
    topk_idx: np.ndarray     # [P,k] i32 ascending
    hit_mask: np.ndarray     # [P,k] u8
    reuse_flags: np.ndarray  # [P] u8
    sim: np.ndarray          # [B,Hq] f64
    s_agg: np.ndarray        # [P] f64
    kth_score: np.ndarray    # [P] f64 (NaN on reuse)
    n_filled: np.ndarray     # [P] i32
    scores: np.ndarray | None
    weights: np.ndarray | None


def step(state: State, q, K, K_src, V_src, tau, k: int, dtype: int, importance=None,
         want_scores=False, want_weights=False, pair_mask=None, n_sink=0, n_recent=0, K_app=None, V_app=None,
         n_app=0) -> StepResult:
    """One iteration of Algorithm 1 for every pair; ``state`` is updated in place.

    q [B,Hq,D], K/K_src/V_src [B,Hkv,N,D] as uint16 bit patterns; tau scalar or [Hkv].
    Pairs not marked in ``pair_mask`` are untouched (their outputs are undefined).
    ``n_sink`` / ``n_recent``: the first / last tokens of the context that every retrieved set contains
    (Section 7.1).  ``K_app`` / ``V_app`` [B,Hkv,cap,D] with ``n_app`` valid rows: the append-only buffer, attended
    in full next to the cached rows (Section 6.2).
    """
    q = _u16(q)
    B, Hq, D = q.shape
    K = _u16(K)
    Hkv, N = K.shape[1], K.shape[2]
    assert K.shape == (B, Hkv, N, D) and Hq % Hkv == 0 and Hq // Hkv <= 64
    K_src, V_src = _u16(K_src, K.shape), _u16(V_src, K.shape)
    P = B * Hkv
    k_max = state.slot_idx.shape[1]
    assert 1 <= k <= k_max and k <= N
    for a in (state.valid, state.prev_q, state.slot_idx, state.K_slots, state.V_slots):
        assert a.flags.c_contiguous
    tau_a = np.ascontiguousarray(np.broadcast_to(np.asarray(tau, dtype=np.float64), (Hkv,)))
    imp = None if importance is None else np.ascontiguousarray(importance, dtype=np.float64)
    out = np.zeros((B, Hq, D), np.float64)
    tk = np.zeros((P, k), np.int32)
    hm = np.zeros((P, k), np.uint8)
    rf = np.zeros(P, np.uint8)
    sim = np.zeros((B, Hq), np.float64)
    sa = np.zeros(P, np.float64)
    kth = np.full(P, np.nan, np.float64)
    nf = np.zeros(P, np.int32)
    sc = np.empty((P, N), np.float64) if want_scores else None
    wt = np.zeros((B, Hq, k + n_app), np.float64) if want_weights else None
    assert n_sink >= 0 and n_recent >= 0 and n_sink + n_recent <= k
    ext = _Ext(n_sink, n_recent, n_app, 0, None, None)
    if n_app:
        K_app, V_app = _u16(K_app), _u16(V_app)
        cap = K_app.shape[2]
        assert K_app.shape == (B, Hkv, cap, D) and V_app.shape == K_app.shape and 0 < n_app <= cap
        ext.app_cap, ext.K_app, ext.V_app = cap, K_app.ctypes.data, V_app.ctypes.data
    pm = None if pair_mask is None else np.ascontiguousarray(pair_mask, dtype=np.uint8)
    dm = _Dims(B, Hq, Hkv, D, N, k, k_max, dtype)
    rc = lib().qo_step(C.byref(dm), _p(q), _p(K), _p(K_src), _p(V_src), _p(state.valid),
                       _p(state.prev_q), _p(state.slot_idx), _p(state.K_slots), _p(state.V_slots),
                       _p(tau_a), _p(imp), _p(out), _p(tk), _p(hm), _p(rf), _p(sim), _p(sa), _p(kth),
                       _p(sc), _p(wt), _p(nf), _p(pm), C.byref(ext))
    if rc:
        raise ValueError(f"qo_step failed ({rc}): malformed cache state")
    return StepResult(out, tk, hm, rf, sim, sa, kth, nf, sc, wt)


def num_threads() -> int:
    return lib().qo_num_threads()


def set_num_threads(n: int) -> None:
    lib().qo_set_num_threads(int(n))
