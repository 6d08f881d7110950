"""GPU tests of what sits around the step: replay from a captured graph with the per-step scalars in device
memory, checkpoint / resume of the cache state, the byte counters, a bounded seeded sweep over random valid
shapes, and the tiny workload at three seeds.  Every comparison with the oracle goes through
tests/gpu_harness.py (which states the bars)."""
import ctypes as C
import random

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2511_14510_amd import binding as Q
from paper_2511_14510_amd import workload as W


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    Q.load()
    import gpu_harness
    return gpu_harness


def _snapshot(sess):
    return [t.clone() for t in (sess.out, sess.topk_idx, sess.hit_mask, sess.reuse_flags, sess.slot_idx,
                                sess.K_slots, sess.V_slots, sess.prev_q, sess.sim)]


@pytest.mark.parametrize("N,k,flags,side", [(4096, 256, 0, False), (70001, 300, 0, False),
                                            (5000, 200, Q.QSAC_FLAG_FILL_KERNEL, True)])
def test_graph_replay_matches_eager_and_the_oracle(H, N, k, flags, side):
    """One step is captured once (Section 2.3, Section 5.2 of the paper: the decode step runs from a graph) and
    replayed for every later step while q, the per-head thresholds and the number of valid rows of the append-only
    buffer change: the replays are compared step by step with the oracle, and bit for bit with an eager session
    that takes the same inputs through qsac_step."""
    B, Hq, Hkv, cap, steps = 2, 8, 2, 48, 40 if N < 10000 else 12
    n_sink, n_recent = 4, 16
    print(f"graph case N={N} k={k} flags={flags} side={side}", flush=True)
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 61)
    Ka, Va = W.make_kv(B, Hkv, cap, 128, "bf16", 62)
    taus = [[0.9, 0.8] if t % 3 else [0.95, 0.85] for t in range(steps)]   # per KV head, changing between steps
    n_apps = [min(t + 1, cap) for t in range(steps)]
    chain = W.QueryChain(B, Hq, 128, 0.95, 61)
    qs = [chain.next() for _ in range(steps)]

    def session():
        return Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K.cuda(), V.cuda(), flags=flags, side_stream=side,
                         n_sink=n_sink, n_recent=n_recent, K_app=Ka.cuda(), V_app=Va.cuda())

    # eager reference run
    eager = session()
    ref = []
    for t in range(steps):
        eager.set_appended(n_apps[t])
        eager.step(W.round_to(qs[t], "bf16").cuda(), taus[t], k)
        eager.sync()
        ref.append(_snapshot(eager))
    eager_stats = eager.stats()
    eager.close()

    # graph run: q and the scalars live in fixed device buffers that are rewritten before each replay
    sess = session()
    q_buf = torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device="cuda:0")
    table = sess.dev_params_table(taus, n_apps)
    dp = torch.zeros(C.sizeof(Q.qsac_dev_params), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    graph = Q.qsac_graph_capture(sess.ctx, sess.step_args(q_buf, None, k, dev_params=dp, n_app_bound=cap))
    state = {"t": 0}

    def replay(q_dev, tau, kk):
        t = state["t"]
        sess.copy_on_main(q_buf, q_dev)
        sess.copy_on_main(dp, table[t])
        sess.n_app = n_apps[t]          # what the oracle is told; the kernels read it from the device block
        Q.qsac_graph_launch(graph)
        state["t"] = t + 1

    par = H.Parity(sess, "bf16", W.bits(K), W.bits(K), W.bits(V), n_sink=n_sink, n_recent=n_recent,
                   Kapp_b=W.bits(Ka), Vapp_b=W.bits(Va), launch=replay)
    for t in range(steps):
        par.step(qs[t], taus[t], k, label=f"graph replay {t}")
        for got, want in zip(_snapshot(sess), ref[t]):
            assert torch.equal(got, want), f"replay {t} differs from the eager step"
    assert par.n_reuse > 0 and par.n_miss > B * Hkv
    assert sess.stats() == eager_stats
    # replays and plain steps mix on one context
    sess.set_appended(cap)
    sess.step(W.round_to(chain.next(), "bf16").cuda(), 0.9, k)
    sess.copy_on_main(dp, table[steps - 1])
    Q.qsac_graph_launch(graph)
    sess.sync()
    assert sess.stats()["steps"] == steps + 2
    Q.qsac_graph_free(graph)
    sess.close()


@pytest.mark.parametrize("N,k,host,dtype", [(6000, 300, True, "bf16"), (33000, 1000, True, "f16"),
                                            (70001, 500, False, "bf16"), (140001, 400, True, "bf16")])
def test_staggered_schedule_matches_the_oracle(H, N, k, host, dtype):
    """QSAC_FLAG_STAGGER: the two halves of the batch (1 + 2 elements here) run on two streams, the second half
    scoring while the first fetches its rows; every select path, rows from pinned host memory or HBM."""
    B, Hq, Hkv = 3, 8, 2
    print(f"staggered case N={N} k={k} host={host} {dtype}", flush=True)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k + 5, dtype, 91, host, host, Q.QSAC_FLAG_STAGGER, None, True)
    par = H.Parity(sess, dtype, Kb, Ksb, Vsb)
    chain = W.QueryChain(B, Hq, 128, 0.95, 91)
    for t in range(10):
        par.step(chain.next(), 0.9, k, label=f"staggered step {t}")
    assert par.n_reuse > 0 and par.n_miss > B * Hkv
    st = sess.stats()
    assert st["reuse_heads"] == par.n_reuse and st["miss_heads"] == par.n_miss
    sess.close()


def test_staggered_schedule_with_resident_heads_sink_tokens_and_append_buffer(H):
    """Every optional tensor of the step is sliced with the batch: resident heads (their host rows poisoned, as
    in the resident-caching test), sink / recent tokens and an append-only buffer that grows by a row per step."""
    B, Hq, Hkv, N, k, cap = 3, 8, 4, 5000, 300, 12
    n_sink, n_recent = 4, 16
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 95)
    Ka, Va = W.make_kv(B, Hkv, cap, 128, "bf16", 96)
    res_slot = [-1, 0, -1, 1]
    K_bad, V_bad = K.clone(), V.clone()
    for h in (1, 3):
        K_bad[:, h] = 7.0
        V_bad[:, h] = -3.0
    V_res = torch.stack([V[:, 1], V[:, 3]], dim=1).contiguous().cuda()
    sess = Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K_bad.pin_memory(), V_bad.pin_memory(),
                     flags=Q.QSAC_FLAG_STAGGER, V_res=V_res, res_slot=res_slot, side_stream=True, n_sink=n_sink,
                     n_recent=n_recent, K_app=Ka.cuda(), V_app=Va.cuda())
    par = H.Parity(sess, "bf16", W.bits(K), W.bits(K), W.bits(V), n_sink=n_sink, n_recent=n_recent,
                   Kapp_b=W.bits(Ka), Vapp_b=W.bits(Va))
    chain = W.QueryChain(B, Hq, 128, 0.95, 95)
    for t in range(cap):
        sess.set_appended(t + 1)
        par.step(chain.next(), 0.9, k, label=f"staggered step {t} with every optional tensor")
    st = sess.stats()
    assert par.n_reuse > 0 and 0 < st["resident_rows"] < st["slot_misses"]
    sess.close()


def test_staggered_schedule_replays_from_a_graph(H):
    """The staggered step forks to stream_side and joins again inside one capture; replays equal eager steps."""
    B, Hq, Hkv, N, k, steps = 4, 8, 2, 9000, 256, 16
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 93)
    chain = W.QueryChain(B, Hq, 128, 0.95, 93)
    qs = [W.round_to(chain.next(), "bf16").cuda() for _ in range(steps)]
    taus = [[0.9, 0.85]] * steps

    def session():
        return Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K.cuda(), V.pin_memory(), flags=Q.QSAC_FLAG_STAGGER,
                         side_stream=True)

    eager = session()
    ref = []
    for t in range(steps):
        eager.step(qs[t], taus[t], k)
        eager.sync()
        ref.append(_snapshot(eager))
    eager.close()
    sess = session()
    q_buf = torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device="cuda:0")
    table = sess.dev_params_table(taus, [0] * steps)
    dp = torch.zeros(C.sizeof(Q.qsac_dev_params), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    graph = Q.qsac_graph_capture(sess.ctx, sess.step_args(q_buf, None, k, dev_params=dp, n_app_bound=0))
    for t in range(steps):
        sess.copy_on_main(q_buf, qs[t])
        sess.copy_on_main(dp, table[t])
        Q.qsac_graph_launch(graph)
        sess.sync()
        for got, want in zip(_snapshot(sess), ref[t]):
            assert torch.equal(got, want), f"replay {t} differs from the eager step"
    Q.qsac_graph_free(graph)
    sess.close()


def test_checkpoint_and_resume(H):
    """The cache state is the caller's slot tensors, slot table and labels plus the library's workspace
    (validity flags, the sorted set of every head): 64 steps in one go equal 32 steps, a copy of that state
    into a fresh context, and 32 more steps there, bit for bit."""
    B, Hq, Hkv, N, k = 2, 8, 2, 9001, 300
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 71)
    chain = W.QueryChain(B, Hq, 128, 0.95, 71)
    qs = [W.round_to(chain.next(), "bf16").cuda() for _ in range(64)]
    Kd, Vd = K.cuda(), V.cuda()
    torch.cuda.synchronize()

    def session():
        return Q.Session(B, Hq, Hkv, N, k, "bf16", Kd, Kd, Vd)

    full = session()
    outs = []
    for t in range(64):
        full.step(qs[t], 0.9, k)
        full.sync()
        outs.append(full.out.clone())
    want = _snapshot(full)
    want_stats = full.stats()
    full.close()

    first = session()
    for t in range(32):
        first.step(qs[t], 0.9, k)
    first.sync()
    saved = {name: getattr(first, name).cpu() for name in ("K_slots", "V_slots", "slot_idx", "prev_q")}
    saved["workspace"] = first.workspace.cpu()
    st32 = first.stats()
    first.close()
    del first

    second = session()          # a fresh context: every cache invalid
    second.sync()
    for name in ("K_slots", "V_slots", "slot_idx", "prev_q"):
        getattr(second, name).copy_(saved[name])
    second.workspace.copy_(saved["workspace"])      # the counters travel with it
    torch.cuda.synchronize()
    for t in range(32, 64):
        second.step(qs[t], 0.9, k)
        second.sync()
        assert torch.equal(second.out, outs[t]), f"step {t} after the restore"
    for got, ref in zip(_snapshot(second), want):
        assert torch.equal(got, ref)
    st = second.stats()
    for key in ("reuse_heads", "miss_heads", "slot_hits", "slot_misses", "bytes_filled_dev"):
        assert st[key] == want_stats[key], key
    assert st["steps"] == 32 and st32["steps"] == 32      # the host-side step counter belongs to the context
    second.close()


def test_byte_counters_follow_the_fill_sources(H):
    """bytes_filled_host / bytes_filled_dev: 512 bytes per filled row, split by where the K row and the V row
    came from; rows of resident heads always count as HBM."""
    B, Hq, Hkv, N, k = 1, 8, 2, 4000, 128
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 81)
    chain = W.QueryChain(B, Hq, 128, 0.95, 81)
    qs = [W.round_to(chain.next(), "bf16").cuda() for _ in range(6)]
    for host_k, host_v, per_row in ((False, False, 0), (False, True, 256), (True, True, 512)):
        sess, *_ = H.make_session(B, Hq, Hkv, N, k, "bf16", K=K, V=V, host_k=host_k, host_v=host_v, side_stream=False)
        for q in qs:
            sess.step(q, 2.0, k)
        st = sess.stats()
        assert st["slot_misses"] > 2 * k
        assert st["bytes_filled_host"] == per_row * st["slot_misses"]
        assert st["bytes_filled_host"] + st["bytes_filled_dev"] == 512 * st["slot_misses"]
        sess.close()
    V_res = V[:, 1:2].contiguous().cuda()
    sess = Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K.pin_memory(), V.pin_memory(), V_res=V_res, res_slot=[-1, 0])
    for q in qs:
        sess.step(q, 2.0, k)
    st = sess.stats()
    assert 0 < st["resident_rows"] < st["slot_misses"]
    assert st["bytes_filled_host"] == 512 * (st["slot_misses"] - st["resident_rows"])
    assert st["bytes_filled_dev"] == 512 * st["resident_rows"]
    sess.close()


def test_randomized_shapes_sweep(H):
    """A bounded, seeded sweep over random valid shapes on every select path (one-workgroup, grid-wide bitmaps,
    long-context lists), both dtypes, G = 1..8, every flag, host and HBM fill sources, sink / recent tokens:
    five steps each against the oracle; stops at the first failure."""
    rng = random.Random(20251114)
    Ns = [700, 4097, 8192, 16385, 20000, 32768, 32769, 50000, 65535, 65536, 65537, 100000, 262144, 262145, 300000]
    ks = [1, 16, 100, 333, 1000, 2048, 2300, 2731, 4096, 8000, 8192, 8193, 9000]
    for case in range(30):
        N = rng.choice(Ns)
        G = rng.choice([1, 2, 3, 4, 5, 8])
        Hkv = rng.choice([1, 2, 3])
        B = rng.choice([1, 2])
        k = min(rng.choice(ks), N)
        if N * B * Hkv * G > 1.2e6:
            B, Hkv = 1, 1          # keeps the oracle's share of a case to a second or two
        k_max = min(k + rng.choice([0, 0, 7]), N)
        dtype = rng.choice(["bf16", "f16"])
        flags = rng.choice([0, 0, 0, Q.QSAC_FLAG_FILL_KERNEL, Q.QSAC_FLAG_SCORE_VALU, Q.QSAC_FLAG_PROFILE])
        side = rng.choice([False, True])
        n_sink, n_recent = rng.choice([0, 0, 4]), rng.choice([0, 0, 9])
        if n_sink + n_recent > k:
            n_sink = n_recent = 0
        tau = rng.choice([0.9, 0.93, 2.0])
        host_v = rng.choice([False, True]) and N <= 70000
        seed = rng.randrange(1000)
        print(f"sweep case {case}: B={B} Hkv={Hkv} G={G} N={N} k={k} k_max={k_max} {dtype} flags={flags} side={side} "
              f"sink={n_sink} recent={n_recent} tau={tau} host_v={host_v} seed={seed}", flush=True)
        K, V = W.make_kv(B, Hkv, N, 128, dtype, seed)
        sess = Q.Session(B, Hkv * G, Hkv, N, k_max, dtype, K.cuda(), K.cuda(), V.pin_memory() if host_v else V.cuda(),
                         flags=flags, side_stream=side, n_sink=n_sink, n_recent=n_recent)
        par = H.Parity(sess, dtype, W.bits(K), W.bits(K), W.bits(V), n_sink=n_sink, n_recent=n_recent)
        chain = W.QueryChain(B, Hkv * G, 128, 0.95, seed)
        for t in range(5):
            par.step(chain.next(), tau, k, label=f"sweep case {case} step {t}")
        sess.close()
        del sess, K, V


@pytest.mark.parametrize("seed", [W.DEFAULT_SEED + 1, W.DEFAULT_SEED + 2, 7])
def test_tiny_config_other_seeds(H, seed):
    """The tiny workload at three more seeds (the default seed runs in test_gpu_parity.py)."""
    w = W.CONFIGS["tiny"]
    sess, Kb, Ksb, Vsb = H.make_session(w.B, w.Hq, w.Hkv, w.N, w.k, w.dtype, seed)
    par = H.Parity(sess, w.dtype, Kb, Ksb, Vsb)
    chain = W.QueryChain(w.B, w.Hq, 128, w.rho, seed)
    for t in range(32):
        par.step(chain.next(), w.tau, w.k, label=f"tiny seed {seed} step {t}")
    assert par.n_reuse > 0 and par.n_miss > w.P
    sess.close()
