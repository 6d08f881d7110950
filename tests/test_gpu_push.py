"""Push-mode transfer (Section 5.2 GPU-centric synchronization, Section 6.2 zero-copy transfer engine of the
paper): the GPU publishes the miss lists and Flag1, host transfer threads copy the rows into the cache slots and
set Flag2, a polling kernel with a bounded wait gates the attention.  Same parity bars as the pull mode."""
import ctypes as C

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


def _session(K, V, B, Hq, Hkv, N, k_max, dtype, flags, **kw):
    return Q.Session(B, Hq, Hkv, N, k_max, dtype, K.cuda(), K.pin_memory(), V.pin_memory(), flags=flags, **kw)


@pytest.mark.parametrize("N,k,k_max,threads,flags", [(6000, 384, 400, 0, 0), (6000, 384, 384, 1, Q.QSAC_FLAG_PROFILE),
                                                     (70001, 300, 300, 7, 0), (300000, 1000, 1000, 3, Q.QSAC_FLAG_SCORE_VALU)])
def test_push_mode_parity(H, N, k, k_max, threads, flags):
    B, Hq, Hkv, dtype = 2, 8, 2, "bf16"
    if N > 100000:
        B = 1
    print(f"push case N={N} k={k} k_max={k_max} threads={threads} flags={flags}", flush=True)
    K, V = W.make_kv(B, Hkv, N, 128, dtype, 101)
    sess = _session(K, V, B, Hq, Hkv, N, k_max, dtype, Q.QSAC_FLAG_PUSH_FILL | flags, push_threads=threads)
    par = H.Parity(sess, dtype, W.bits(K), W.bits(K), W.bits(V))
    chain = W.QueryChain(B, Hq, 128, 0.95, 101)
    for t in range(12):
        par.step(chain.next(), 0.9, k, label=f"push step {t}")
    st = sess.stats()
    assert par.n_reuse > 0 and par.n_miss > B * Hkv
    assert st["bytes_filled_host"] == 512 * st["slot_misses"] == 512 * par.filled
    sess.close()


def test_push_and_pull_end_in_the_same_state(H):
    """The same chain through the GPU-pull fill and through the push mode, steps enqueued back to back without
    host synchronisation: identical outputs, slot tables and slot rows."""
    B, Hq, Hkv, N, k = 2, 8, 2, 9001, 300
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 102)
    chain = W.QueryChain(B, Hq, 128, 0.95, 102)
    qs = [W.round_to(chain.next(), "bf16").cuda() for _ in range(24)]
    torch.cuda.synchronize()
    res = []
    for flags in (0, Q.QSAC_FLAG_PUSH_FILL):
        sess = _session(K, V, B, Hq, Hkv, N, k, "bf16", flags)
        for q in qs:
            sess.step(q, 0.9, k)
        sess.sync()
        res.append([t.clone() for t in (sess.out, sess.topk_idx, sess.hit_mask, sess.slot_idx, sess.K_slots, sess.V_slots)]
                   + [sess.stats()])
        sess.close()
    for x, y in zip(res[0][:-1], res[1][:-1]):
        assert torch.equal(x, y)
    assert res[0][-1] == res[1][-1]


def test_push_mode_replayed_from_a_graph(H):
    B, Hq, Hkv, N, k, steps = 1, 8, 2, 5000, 200, 10
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 103)
    sess = _session(K, V, B, Hq, Hkv, N, k, "bf16", Q.QSAC_FLAG_PUSH_FILL)
    q_buf = torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device="cuda:0")
    table = sess.dev_params_table([0.9] * steps, [0] * steps)
    dp = table[0].clone()
    torch.cuda.synchronize()
    graph = Q.qsac_graph_capture(sess.ctx, sess.step_args(q_buf, None, k, dev_params=dp))

    def replay(q_dev, tau, kk):
        sess.copy_on_main(q_buf, q_dev)
        Q.qsac_graph_launch(graph)

    par = H.Parity(sess, "bf16", W.bits(K), W.bits(K), W.bits(V), launch=replay)
    chain = W.QueryChain(B, Hq, 128, 0.95, 103)
    for t in range(steps):
        par.step(chain.next(), 0.9, k, label=f"push graph replay {t}")
    assert par.n_reuse > 0 and par.n_miss > B * Hkv
    Q.qsac_graph_free(graph)
    sess.close()


def test_polling_kernel_gives_up_when_the_host_does_not_answer(H):
    """With the transfer threads told to ignore every request the polling kernel runs into its bound (2 ms here),
    records that and exits: the stream drains, the library reports QSAC_ETIMEOUT and refuses further steps until
    a reset."""
    B, Hq, Hkv, N, k = 1, 8, 2, 3000, 100
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 104)
    sess = _session(K, V, B, Hq, Hkv, N, k, "bf16", Q.QSAC_FLAG_PUSH_FILL | Q.QSAC_FLAG_PUSH_HOLD, push_wait_us=2000)
    q = W.round_to(W.QueryChain(B, Hq, 128, 0.95, 104).next(), "bf16").cuda()
    sess.step(q, 0.9, k)
    sess.sync()                                   # returns: the polling kernel ended by itself
    with pytest.raises(Q.QsacError) as e:
        sess.stats()
    assert e.value.code == Q.QSAC_ETIMEOUT
    with pytest.raises(Q.QsacError) as e:
        sess.step(q, 0.9, k)
    assert e.value.code in (Q.QSAC_ETIMEOUT, Q.QSAC_ESTATE)
    sess.reset()                                  # clears the condition; the threads still hold, so it comes back
    sess.step(q, 0.9, k)
    sess.sync()
    with pytest.raises(Q.QsacError) as e:
        sess.stats()
    assert e.value.code == Q.QSAC_ETIMEOUT
    sess.close()


def test_push_mode_needs_host_sources(H):
    B, Hq, Hkv, N, k = 1, 8, 2, 3000, 100
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 105)
    sess = Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K.cuda(), V.pin_memory(), flags=Q.QSAC_FLAG_PUSH_FILL)
    q = W.round_to(W.QueryChain(B, Hq, 128, 0.95, 105).next(), "bf16").cuda()
    with pytest.raises(Q.QsacError) as e:
        sess.step(q, 0.9, k)
    assert e.value.code == Q.QSAC_EINVAL
    sess.close()


def test_qwen_shaped_offload_full_size_in_push_mode(H):
    w = W.CONFIGS["qwen25_14b_128k_offload"]
    sess, Kb, Ksb, Vsb = H.make_session_on_gpu(w, Q.QSAC_FLAG_PUSH_FILL, False)
    par = H.Parity(sess, w.dtype, Kb, Ksb, Vsb)
    chain = W.chain_for(w)
    rng = np.random.default_rng(5)
    for t in range(4):
        pairs = range(w.P) if t in (0, 3) else rng.choice(w.P, size=8, replace=False)
        par.step(chain.next(), w.tau, w.k, label=f"qwen push step {t}", pairs=pairs)
        print(f"  step {t}: ok, reuse {par.n_reuse}, miss {par.n_miss}, max err {par.max_err:.2e}", flush=True)
    assert par.n_reuse > 0 and par.n_miss > w.P
    sess.close()
    torch.cuda.empty_cache()
