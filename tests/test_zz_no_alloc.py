"""qsac_step_static(): the step for callers that cannot allocate device memory.  Its state and scratch live in
an array inside the library's device image instead of a caller-provided workspace.  Checked here, through the C
ABI, against qsac_step() on an ordinary context fed the same inputs (every output and every piece of cache state
bit for bit) and against the oracle, on two runs in a row of which the second is smaller, so that whatever the
first left in the array would show."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2511_14510_amd import binding as Q
from paper_2511_14510_amd import workload as W

FIELDS = ("out", "topk_idx", "hit_mask", "reuse_flags", "sim", "slot_idx", "K_slots", "V_slots", "prev_q")


def _run(H, B, Hq, Hkv, N, k, dtype, seed, steps, host_v, flags=0):
    print(f"static case B={B} Hq={Hq} Hkv={Hkv} N={N} k={k} {dtype} seed={seed} host_v={host_v} flags={flags}", flush=True)
    K, V = W.make_kv(B, Hkv, N, 128, dtype, seed)
    K_dev = K.cuda()
    V_src = V.pin_memory() if host_v else V.cuda()
    importance = [1.0 + 0.25 * (i % 3) for i in range(Hq)]
    ref = Q.Session(B, Hq, Hkv, N, k, dtype, K_dev, K_dev, V_src, flags=flags, importance=importance)
    # a second set of caller tensors; its context and workspace are never used for a step
    mine = Q.Session(B, Hq, Hkv, N, k, dtype, K_dev, K_dev, V_src, flags=flags, importance=importance)
    cfg = Q.make_config(B, Hq, Hkv, N, k, W.DTYPE_CODES[dtype], flags, importance)
    cfg.stream_main = mine.main.cuda_stream          # workspace stays NULL: the call must not need one
    state = {"first": True}

    def launch(q_dev, tau, kk):
        Q.qsac_step_static(cfg, mine.step_args(q_dev, tau, kk), reset=state["first"])
        state["first"] = False

    # the harness reads validity flags from a session's workspace view: point it at nothing it owns by comparing
    # against `ref` instead, and let the oracle follow `ref` (identical state is asserted every step)
    par = H.Parity(ref, dtype, W.bits(K), W.bits(K), W.bits(V), importance=importance)
    chain = W.QueryChain(B, Hq, 128, 0.95, seed)
    for t in range(steps):
        q64 = chain.next()
        par.step(q64, 0.9, k, label=f"static reference step {t}")
        launch(W.round_to(q64, dtype).cuda(), 0.9, k)
        mine.sync()
        for name in FIELDS:
            assert torch.equal(getattr(mine, name), getattr(ref, name)), f"step {t}: {name} differs from qsac_step"
    assert par.n_reuse > 0 and par.n_miss > B * Hkv
    # without a reset the configuration must be the one that was bound
    other = Q.make_config(B, Hq, Hkv, N - 1, k, W.DTYPE_CODES[dtype], flags)
    other.stream_main = mine.main.cuda_stream
    a = mine.step_args(W.round_to(chain.next(), dtype).cuda(), 0.9, k)
    assert Q.load().qsac_step_static(C.byref(other), C.byref(a), 0) == Q.QSAC_ESTATE
    ref.close()
    mine.close()


def test_static_entry_point_matches_qsac_step_twice_in_a_row():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    Q.load()
    import gpu_harness as H
    _run(H, B=2, Hq=8, Hkv=2, N=20000, k=600, dtype="bf16", seed=91, steps=8, host_v=True)
    _run(H, B=1, Hq=10, Hkv=2, N=3000, k=100, dtype="f16", seed=92, steps=8, host_v=False, flags=Q.QSAC_FLAG_FILL_KERNEL)
    # sizes beyond the array are turned down on the host
    big = Q.make_config(8, 32, 8, 1 << 20, 4096, Q.QSAC_BF16)
    assert Q.qsac_workspace_bytes(big) > Q.QSAC_STATIC_SCRATCH_BYTES
    a = Q.qsac_step_args()
    assert Q.load().qsac_step_static(C.byref(big), C.byref(a), 1) == Q.QSAC_EWORKSPACE
    side = Q.make_config(1, 8, 2, 4096, 256, Q.QSAC_F16)
    side.stream_side = 0x1234
    assert Q.load().qsac_step_static(C.byref(side), C.byref(a), 1) == Q.QSAC_EINVAL
