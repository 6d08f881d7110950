"""GPU parity: every case drives the HIP kernels through the C ABI and checks each step against
the oracle (tests/gpu_harness.py states the bars)."""
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


def run_chain(H, B, Hq, Hkv, N, k, k_max, dtype, steps, tau=0.9, rho=0.95, seed=3, flags=0, importance=None,
              host_k=False, host_v=False, q_norm=1.0, side_stream=True, expect_both=True):
    print(f"case B={B} Hq={Hq} Hkv={Hkv} N={N} k={k} k_max={k_max} {dtype} steps={steps} tau={tau} rho={rho} "
          f"seed={seed} flags={flags} host=({host_k},{host_v}) q_norm={q_norm}", flush=True)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k_max, dtype, seed, host_k, host_v, flags, importance, side_stream)
    par = H.Parity(sess, dtype, Kb, Ksb, Vsb, importance)
    chain = W.QueryChain(B, Hq, 128, rho, seed, q_norm=q_norm)
    for t in range(steps):
        par.step(chain.next(), tau, k, label=f"step {t}")
    st = sess.stats()
    assert st["steps"] == steps
    assert st["reuse_heads"] == par.n_reuse and st["miss_heads"] == par.n_miss
    assert st["slot_misses"] == par.filled and st["slot_hits"] == par.n_miss * k - par.filled
    if expect_both:
        assert par.n_reuse > 0 and par.n_miss > B * Hkv
    sess.close()
    return par


def test_tiny_config_full_run(H):
    """The tiny workload in full: 1 x 8q/2kv, N=4096, k=256, fp16, tau=0.9, 64 steps."""
    w = W.CONFIGS["tiny"]
    par = run_chain(H, w.B, w.Hq, w.Hkv, w.N, w.k, w.k, w.dtype, w.steps, w.tau, w.rho, w.seed)
    assert 0.3 < par.n_reuse / (par.n_reuse + par.n_miss) < 0.95


@pytest.mark.parametrize("flags", [0, Q.QSAC_FLAG_SCORE_VALU, Q.QSAC_FLAG_PROFILE, Q.QSAC_FLAG_FILL_KERNEL,
                                   Q.QSAC_FLAG_FILL_KERNEL | Q.QSAC_FLAG_SERIAL, Q.QSAC_FLAG_FILL_KERNEL | Q.QSAC_FLAG_PROFILE])
def test_ragged_shapes_gqa5_bf16(H, flags):
    """N, k and k_max off every tile size (1024-key score tiles, 8192-key select chunks, 64-row
    fill and attention tiles), G = 5 as in the Qwen2.5-14B shape."""
    run_chain(H, B=2, Hq=10, Hkv=2, N=9001, k=300, k_max=333, dtype="bf16", steps=16, flags=flags)


@pytest.mark.parametrize("G,dtype", [(1, "f16"), (2, "bf16"), (3, "f16"), (4, "bf16"), (6, "bf16"), (7, "f16"), (8, "bf16")])
@pytest.mark.parametrize("flags", [0, Q.QSAC_FLAG_SCORE_VALU])
def test_group_sizes(H, G, dtype, flags):
    run_chain(H, B=1, Hq=2 * G, Hkv=2, N=2500, k=130, k_max=130, dtype=dtype, steps=10, flags=flags, seed=10 + G,
              side_stream=False)


@pytest.mark.parametrize("N,k", [(1, 1), (3, 3), (17, 1), (64, 64), (100, 99), (1024, 1), (1025, 1025)])
def test_degenerate_sizes(H, N, k):
    run_chain(H, B=1, Hq=4, Hkv=1, N=N, k=k, k_max=k, dtype="bf16", steps=6, tau=0.97, expect_both=False)


def test_tau_above_one_refreshes_every_step(H):
    par = run_chain(H, B=1, Hq=8, Hkv=2, N=3000, k=200, k_max=200, dtype="bf16", steps=8, tau=2.0, expect_both=False)
    assert par.n_reuse == 0


def test_tau_minus_one_keeps_the_first_set(H):
    par = run_chain(H, B=1, Hq=8, Hkv=2, N=3000, k=200, k_max=200, dtype="f16", steps=8, tau=-1.0, rho=0.2,
                    expect_both=False)
    assert par.n_miss == 2 and par.n_reuse == 14


def test_k_equals_N_matches_dense_attention(H):
    """With k = N the sparse step is dense attention; after the first step nothing is ever fetched."""
    par = run_chain(H, B=1, Hq=8, Hkv=2, N=777, k=777, k_max=777, dtype="bf16", steps=8, tau=0.93)
    assert par.filled == 2 * 777


def test_peaked_softmax_and_outlier_values(H):
    """||q|| = 2 sqrt(D): logits spread over hundreds of units, the online rescaling is exercised."""
    run_chain(H, B=1, Hq=8, Hkv=2, N=4000, k=512, k_max=512, dtype="bf16", steps=10, q_norm=2 * np.sqrt(128.0))


@pytest.mark.parametrize("flags", [0, Q.QSAC_FLAG_FILL_KERNEL])
def test_fill_from_pinned_host_memory(H, flags):
    run_chain(H, B=2, Hq=8, Hkv=2, N=6000, k=384, k_max=400, dtype="bf16", steps=12, host_k=True, host_v=True, flags=flags)
    run_chain(H, B=1, Hq=8, Hkv=2, N=6000, k=384, k_max=384, dtype="f16", steps=8, host_v=True, side_stream=False,
              flags=flags)


@pytest.mark.parametrize("flags", [0, Q.QSAC_FLAG_FILL_KERNEL])
def test_resident_heads_never_touch_their_host_rows(H, flags):
    """Resident caching (Section 4.4): KV heads 1 and 3 keep their full V in HBM (V_res) and take K rows from
    K_dev.  Their regions of the host-side fill sources are overwritten with other values, so any read from
    there would show up as wrong slot rows or outputs; the results must equal those of the oracle on the true K, V."""
    B, Hq, Hkv, N, k = 2, 8, 4, 5000, 300
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 31)
    res_slot = [-1, 0, -1, 1]
    K_bad, V_bad = K.clone(), V.clone()
    for h in (1, 3):
        K_bad[:, h] = 7.0
        V_bad[:, h] = -3.0
    V_res = torch.stack([V[:, 1], V[:, 3]], dim=1).contiguous().cuda()
    sess = Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K_bad.pin_memory(), V_bad.pin_memory(), flags=flags,
                     V_res=V_res, res_slot=res_slot, side_stream=bool(flags))
    par = H.Parity(sess, "bf16", W.bits(K), W.bits(K), W.bits(V))
    chain = W.QueryChain(B, Hq, 128, 0.95, 31)
    for t in range(10):
        par.step(chain.next(), 0.9, k, label=f"resident step {t}")
    st = sess.stats()
    assert par.n_reuse > 0 and 0 < st["resident_rows"] < st["slot_misses"]
    sess.close()


@pytest.mark.parametrize("flags,N", [(0, 6000), (Q.QSAC_FLAG_SCORE_VALU, 6000), (0, 70001)])
def test_sink_recent_tokens_and_append_buffer(H, flags, N):
    """Section 7.1 / 6.2: 4 sink and 64 recent tokens are members of every retrieved set, and the attention
    runs over the k cached rows plus the append-only buffer, which grows by one generated token per step."""
    B, Hq, Hkv, k, cap = 2, 8, 2, 200, 40
    n_sink, n_recent = 4, 64
    K, V = W.make_kv(B, Hkv, N, 128, "bf16", 41)
    Ka, Va = W.make_kv(B, Hkv, cap, 128, "bf16", 42)
    sess = Q.Session(B, Hq, Hkv, N, k, "bf16", K.cuda(), K.cuda(), V.cuda(), flags=flags, n_sink=n_sink,
                     n_recent=n_recent, K_app=Ka.cuda(), V_app=Va.cuda())
    par = H.Parity(sess, "bf16", W.bits(K), W.bits(K), W.bits(V), n_sink=n_sink, n_recent=n_recent,
                   Kapp_b=W.bits(Ka), Vapp_b=W.bits(Va))
    chain = W.QueryChain(B, Hq, 128, 0.95, 41)
    forced = set(range(n_sink)) | set(range(N - n_recent, N))
    for t in range(cap):
        sess.set_appended(t + 1)
        par.step(chain.next(), 0.9, k, label=f"append step {t}")
        for p in range(B * Hkv):
            assert forced <= set(sess.topk_idx.view(B * Hkv, k)[p].tolist())
    assert par.n_reuse > 0 and par.n_miss > B * Hkv
    sess.close()


def test_only_persistent_tokens_fit(H):
    """k = n_sink + n_recent: the retrieved set is exactly the persistent tokens, whatever the scores."""
    N, k = 3000, 68
    sess, Kb, Ksb, Vsb = H.make_session(1, 4, 1, N, k, "bf16", seed=43)
    sess.close()
    K, V = W.make_kv(1, 1, N, 128, "bf16", 43)
    sess = Q.Session(1, 4, 1, N, k, "bf16", K.cuda(), K.cuda(), V.cuda(), n_sink=4, n_recent=64)
    par = H.Parity(sess, "bf16", W.bits(K), W.bits(K), W.bits(V), n_sink=4, n_recent=64)
    chain = W.QueryChain(1, 4, 128, 0.5, 43)
    for t in range(3):
        par.step(chain.next(), 2.0, k, label=f"persistent only step {t}")
        assert sess.topk_idx.view(-1).tolist() == list(range(4)) + list(range(N - 64, N))
    sess.close()


def test_per_head_tau_and_importance(H):
    imp = [0.2, 1.0, 3.0, 0.7, 1.0, 1.0, 0.1, 2.5]
    par = run_chain(H, B=2, Hq=8, Hkv=2, N=2000, k=100, k_max=100, dtype="bf16", steps=16, tau=[0.95, 0.8],
                    importance=imp)
    assert par.n_reuse > 0


@pytest.mark.parametrize("flags", [0, Q.QSAC_FLAG_FILL_KERNEL])
def test_many_pairs_long_rows(H, flags):
    """More pairs than compute-unit waves in flight, and an N that spans several select chunks."""
    run_chain(H, B=8, Hq=16, Hkv=4, N=20000, k=640, k_max=640, dtype="bf16", steps=6, flags=flags)


def test_attention_with_several_tiles_per_wave(H):
    """k large enough that a workgroup takes 512 slots: eight tiles per wave through the two-buffer pipeline."""
    run_chain(H, B=4, Hq=8, Hkv=2, N=40000, k=3000, k_max=3000, dtype="bf16", steps=5, tau=0.93, expect_both=False)


@pytest.mark.parametrize("flags,N,k", [(0, 140001, 700), (Q.QSAC_FLAG_SCORE_VALU, 140001, 700), (0, 270001, 700),
                                         (0, 270001, 8200), (Q.QSAC_FLAG_FILL_KERNEL, 270001, 333)])
def test_large_n_path(H, flags, N, k):
    """N above 65536 takes the grid-wide select (histogram fused into scoring, refine, mark, diff on bitmaps);
    above 262144 keys the set is emitted as a token list by the whole grid and diffed from LDS, unless k is
    above 8192: then the bitmap diff runs with 32 words per lane instead of 8."""
    run_chain(H, B=1, Hq=8, Hkv=2, N=N, k=k, k_max=k, dtype="bf16", steps=6, flags=flags, tau=0.93)


def test_adaptive_thresholds_drive_the_gate(H):
    """Eq. (3)-(5): thresholds from synthetic KV-head importance scores (eta = 0.8, p = 3 as in the paper's
    setup) feed the per-head tau input; the unimportant head reuses far more often than the important one."""
    tau = Q.qsac_adaptive_thresholds([1.0, 0.97, 0.6, 0.0], 0.8, 3.0)
    assert tau[0] == pytest.approx(0.8, abs=1e-6) and tau[3] == pytest.approx(-1.0, abs=1e-6) and tau[0] > tau[1] > tau[2] > tau[3]
    sess, Kb, Ksb, Vsb = H.make_session(1, 8, 4, 3000, 128, "bf16", seed=9)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    chain = W.QueryChain(1, 8, 128, 0.9, 9)
    reuse = np.zeros(4)
    for t in range(24):
        par.step(chain.next(), tau, 128, label=f"adaptive step {t}")
        reuse += sess.reuse_flags.cpu().numpy().reshape(-1)
    assert reuse[3] == 23 and reuse[0] < reuse[2] <= reuse[3]
    sess.close()


@pytest.mark.parametrize("N", [65536, 65537])
def test_both_sides_of_the_select_switch(H, N):
    run_chain(H, B=1, Hq=5, Hkv=1, N=N, k=1000, k_max=1000, dtype="bf16", steps=4, tau=0.93, expect_both=False)


def test_ties_across_many_waves_of_the_bitmap(H):
    """Half the keys are one repeated row: thousands of keys equal the k-th key, spread over every wave's
    share of the bitmap, so the ranked tie resolution (not the all-ties-belong shortcut) decides the set."""
    B, Hq, Hkv, N = 1, 4, 1, 70000
    g = torch.Generator().manual_seed(5)
    K = torch.randn((B, Hkv, N, 128), generator=g)
    K[:, :, 1::2] = K[0, 0, 1]
    K = K.to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, 128), generator=g).to(torch.bfloat16)
    # (large-N diff on bitmaps, one-workgroup select, large-N diff on lists)
    for n_ctx, k in ((N, 30000), (40000, 15000), (N, 5000)):
        sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, n_ctx, k, "bf16", K=K[:, :, :n_ctx].contiguous(),
                                            V=V[:, :, :n_ctx].contiguous())
        par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
        # queries along the repeated row: its score is positive and in the upper half, so the
        # k-th score is that of the repeated row itself
        base = K[0, 0, 1].double().numpy()
        rng = np.random.default_rng(3)
        for t in range(3):
            q = np.tile(base / np.linalg.norm(base), (B, Hq, 1)) + 0.02 * rng.standard_normal((B, Hq, 128))
            r = par.step(q, 2.0, k, label=f"mass ties N={n_ctx} step {t}")
            assert (r.scores[0] == r.kth_score[0]).sum() > 1000
        assert par.n_band == 0
        sess.close()


def test_ties_on_the_long_context_path(H):
    """Above 262144 keys the set is emitted as a token list by the whole grid: thousands of keys equal the
    k-th key, in every chunk, and only the first r of them (by index) may be taken."""
    B, Hq, Hkv, N, k = 1, 4, 1, 270000, 6000
    g = torch.Generator().manual_seed(6)
    K = torch.randn((B, Hkv, N, 128), generator=g)
    K[:, :, 1::2] = K[0, 0, 1]
    K = K.to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, 128), generator=g).to(torch.bfloat16)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "bf16", K=K, V=V)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    base = K[0, 0, 1].double().numpy()
    rng = np.random.default_rng(4)
    for t in range(3):
        q = np.tile(base / np.linalg.norm(base), (B, Hq, 1)) + 0.02 * rng.standard_normal((B, Hq, 128))
        r = par.step(q, 2.0, k, label=f"long-context ties step {t}")
        assert (r.scores[0] == r.kth_score[0]).sum() > 1000
    assert par.n_band == 0
    sess.close()


def exact_tie_case(H, flags, N=5000, k=257):
    """K entries in {-1, 0, 1} and queries with a few small-integer entries: every score is a small
    integer, exact in fp32 and fp64 alike, with hundreds of exact ties across the k-th score - the
    index sets must match exactly under the lowest-index tie-break."""
    B, Hq, Hkv = 1, 4, 2
    rng = np.random.default_rng(99)
    K = torch.from_numpy(rng.integers(-1, 2, (B, Hkv, N, 128)).astype(np.float32)).to(torch.bfloat16)
    V = torch.from_numpy(rng.standard_normal((B, Hkv, N, 128)).astype(np.float32)).to(torch.bfloat16)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "bf16", flags=flags, K=K, V=V)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    for t in range(6):
        q = np.zeros((B, Hq, 128))
        for hq in range(Hq):
            pos = rng.choice(128, 6, replace=False)
            q[0, hq, pos] = rng.integers(-2, 3, 6)
            q[0, hq, pos[0]] = 1
        r = par.step(q, 2.0, k, label=f"ties step {t}")
        for p in range(2):
            kth = r.kth_score[p]
            assert (r.scores[p] == kth).sum() > 20          # the k-th score really is tied
    assert par.n_band == 0
    st = sess.stats()
    sess.close()
    return st


@pytest.mark.parametrize("flags", [0, Q.QSAC_FLAG_SCORE_VALU])
def test_exact_ties_take_the_lowest_index(H, flags):
    exact_tie_case(H, flags)


def test_exact_ties_inside_the_candidate_list(H):
    """The same integer scores at a size where the one-workgroup select works on its candidate list: the bin
    of the k-th key holds hundreds of equal keys (more than one wave can rank directly), of which only the first
    few by index belong to the set."""
    st = exact_tie_case(H, 0, N=20000, k=1000)
    print("guided selects", st["guided_selects"], "of", st["miss_heads"], flush=True)
    assert st["guided_selects"] > 0


def test_all_keys_equal_selects_the_first_k(H):
    B, Hq, Hkv, N, k = 1, 4, 1, 9000, 100
    row = torch.randn(128, generator=torch.Generator().manual_seed(1))
    K = row.expand(B, Hkv, N, 128).contiguous().to(torch.float16)
    V = torch.randn((B, Hkv, N, 128), generator=torch.Generator().manual_seed(2)).to(torch.float16)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "f16", K=K, V=V)
    par = H.Parity(sess, "f16", Kb, Ksb, Vsb)
    chain = W.QueryChain(B, Hq, 128, 0.5, 4)
    for t in range(3):
        par.step(chain.next(), 2.0, k, label=f"equal keys step {t}")
        assert sess.topk_idx.cpu().numpy().reshape(-1).tolist() == list(range(k))
    sess.close()


def test_gate_equality_reuses(H):
    """cos = 1/2 exactly against tau = 1/2 reuses ("at or above")."""
    sess, Kb, Ksb, Vsb = H.make_session(1, 1, 1, 500, 16, "bf16")
    a = np.zeros((1, 1, 128)); a[0, 0, :4] = 1
    b = np.zeros((1, 1, 128)); b[0, 0, 0] = 1
    dev = lambda x: W.round_to(x, "bf16").cuda()
    sess.step(dev(a), 0.5, 16); sess.sync()
    sess.step(dev(b), 0.5, 16); sess.sync()
    assert sess.reuse_flags.item() == 1 and sess.sim.item() == 0.5
    sess.reset()
    sess.step(dev(a), 0.5, 16); sess.sync()
    sess.step(dev(b), float(np.float32(0.5) + np.float32(2 ** -24) * 2), 16); sess.sync()
    assert sess.reuse_flags.item() == 0
    sess.close()


def test_reset_and_rerun_are_bit_identical(H):
    """Two runs of the same chain (with a reset between them) give identical outputs: integer
    atomics only, no order-dependent floating-point accumulation anywhere on the path."""
    sess, Kb, Ksb, Vsb = H.make_session(2, 8, 2, 7000, 256, "bf16")
    outs = []
    for rep in range(2):
        chain = W.QueryChain(2, 8, 128, 0.95, 21)
        rec = []
        for t in range(12):
            sess.step(W.round_to(chain.next(), "bf16").cuda(), 0.9, 256)
            sess.sync()
            rec.append((sess.out.clone(), sess.topk_idx.clone(), sess.hit_mask.clone(), sess.reuse_flags.clone(),
                        sess.slot_idx.clone()))
        outs.append(rec)
        sess.reset()
    for a, b in zip(*outs):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
    sess.close()


def test_back_to_back_steps_without_host_sync(H):
    """Steps enqueued without synchronising in between (the way bench.py drives them) end in the
    same state as the same steps taken one at a time."""
    res = []
    for sync_each in (True, False):
        sess, *_ = H.make_session(2, 8, 2, 7000, 256, "bf16", host_v=True, flags=Q.QSAC_FLAG_FILL_KERNEL)
        chain = W.QueryChain(2, 8, 128, 0.95, 22)
        qs = [W.round_to(chain.next(), "bf16").cuda() for _ in range(16)]
        torch.cuda.synchronize()
        for q in qs:
            sess.step(q, 0.9, 256)
            if sync_each:
                sess.sync()
        sess.sync()
        res.append((sess.out.clone(), sess.topk_idx.clone(), sess.slot_idx.clone(), sess.K_slots.clone(),
                    sess.V_slots.clone(), sess.stats()))
        sess.close()
    for x, y in zip(res[0][:5], res[1][:5]):
        assert torch.equal(x, y)
    assert res[0][5] == res[1][5]


@pytest.mark.parametrize("N,k,k_max", [(9001, 300, 333), (40000, 1111, 1200), (65536, 2048, 2048), (700, 700, 700),
                                       (3000, 16, 16), (65536, 5000, 5000)])
def test_guided_select(H, N, k, k_max):
    """The one-workgroup select takes its top-k from the keys above a sampled bound when it can, and from all
    keys when it cannot (k = N, k too large for the candidate list): sets, masks and slots against the oracle."""
    par = run_chain(H, B=3, Hq=8, Hkv=2, N=N, k=k, k_max=k_max, dtype="bf16", steps=12, seed=77, side_stream=False)


def outstanding_rows_case(H, N, k, special, scale):
    """Keys at `special` score `scale` times what the others do (all along one direction d, queries along d)."""
    B, Hq, Hkv = 1, 4, 1
    g = torch.Generator().manual_seed(21)
    K = torch.randn((B, Hkv, N, 128), generator=g)
    d = torch.randn(128, generator=g)
    d = d / d.norm()
    K[0, 0, special] = scale * d + 0.05 * torch.randn((len(special), 128), generator=g)
    K = K.to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, 128), generator=g).to(torch.bfloat16)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "bf16", K=K, V=V, side_stream=False)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    rng = np.random.default_rng(22)
    for t in range(4):
        q = np.tile(d.double().numpy(), (B, Hq, 1)) + 0.05 * rng.standard_normal((B, Hq, 128))
        par.step(q, 2.0, k, label=f"outstanding rows step {t}")
    st = sess.stats()
    sess.close()
    return st


def test_guided_select_with_the_kth_key_far_above_the_bound(H):
    """1500 keys score a hundred times what the rest do, none of them where the select samples, and k = 512:
    the sampled bound lies among the ordinary keys, the k-th key octaves above it, beyond what the candidates'
    histogram resolves, so the radix levels over the candidate list decide."""
    N, k = 32768, 512
    unsampled = np.setdiff1d(np.arange(N), 4 * np.arange(N // 4))
    special = np.random.default_rng(5).choice(unsampled, 1500, replace=False)
    st = outstanding_rows_case(H, N, k, special, 100.0)
    assert st["miss_heads"] == 4 and st["guided_selects"] == 4


def test_guided_select_when_one_wave_holds_too_many_candidates(H):
    """768 outstanding keys in the three 256-token stripes that one wave of the select reads (tokens 0..255 of
    every 4096): that wave's part of the candidate list overflows and the full radix path takes over."""
    N, k = 32768, 2048
    special = np.concatenate([np.arange(4096 * j, 4096 * j + 256) for j in range(3)])
    st = outstanding_rows_case(H, N, k, special, 40.0)
    assert st["miss_heads"] == 4 and st["guided_selects"] == 0


@pytest.mark.parametrize("N", [32768, 100000])
def test_partial_ties_among_the_candidates(H, N):
    """200 identical key rows score highest and k = 100: the k-th key's fine bin holds more equal keys than a wave
    ranks directly, and only the first 100 of them by index belong to the set (one-workgroup select at 32768,
    list-building select at 100000)."""
    B, Hq, Hkv, k = 1, 4, 1, 100
    g = torch.Generator().manual_seed(31)
    K = torch.randn((B, Hkv, N, 128), generator=g)
    row = 3.0 * torch.randn(128, generator=g)
    twins = np.sort(np.random.default_rng(32).choice(N, 200, replace=False))
    K[0, 0, twins] = row
    K = K.to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, 128), generator=g).to(torch.bfloat16)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "bf16", K=K, V=V, side_stream=False)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    rng = np.random.default_rng(33)
    base = K[0, 0, twins[0]].double().numpy()
    for t in range(3):
        q = np.tile(base / np.linalg.norm(base), (B, Hq, 1)) + 0.01 * rng.standard_normal((B, Hq, 128))
        r = par.step(q, 2.0, k, label=f"partial ties N={N} step {t}")
        assert (r.scores[0] == r.kth_score[0]).sum() == 200
        assert sess.topk_idx.cpu().numpy().reshape(-1).tolist() == twins[:k].tolist()
    assert par.n_band == 0 and sess.stats()["guided_selects"] == 3
    sess.close()


@pytest.mark.parametrize("N,k", [(100000, 20000), (131072, 40000), (70000, 9000)])
def test_list_building_select_with_large_k(H, N, k):
    """More keys at or above the k-th key's level-0 bin than the pairs' lists hold: one workgroup streams the
    keys, descends a radix level and compacts what is left into LDS (or, at 9000, stays with the list)."""
    run_chain(H, B=1, Hq=4, Hkv=1, N=N, k=k, k_max=k, dtype="bf16", steps=3, tau=2.0, expect_both=False, seed=41)


def test_calibration_kernels_run(H):
    """The two measurement aids: the copy moves the bytes, the read-only kernel leaves its sink alone."""
    src = torch.arange(1 << 18, dtype=torch.int32, device="cuda:0")
    dst = torch.zeros_like(src)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    Q.qsac_calibration_copy(dst.data_ptr(), src.data_ptr(), src.numel() * 4)
    Q.qsac_calibration_read(src.data_ptr(), src.numel() * 4, sink.data_ptr())
    Q.qsac_calibration_read(src.data_ptr() + 16, 4096 + 16, sink.data_ptr())      # a ragged span
    torch.cuda.synchronize()
    assert torch.equal(dst, src) and int(sink.item()) == 0


def test_guided_select_falls_back_when_its_sample_misleads(H):
    """1000 keys with outstanding scores sit exactly where the one-workgroup select samples (N = 32768: the
    first key of key vectors 0..1023, 2048..3071, ...), so the sampled bound lands among them, fewer than k keys
    pass it, and the full radix path has to take over: same sets as the oracle, and the counters say so."""
    B, Hq, Hkv, N, k = 1, 4, 1, 32768, 2048
    g = torch.Generator().manual_seed(12)
    K = torch.randn((B, Hkv, N, 128), generator=g)
    d = torch.randn(128, generator=g)
    d = d / d.norm()
    sampled = np.concatenate([4 * np.arange(2048 * j, 2048 * j + 1024) for j in range(4)])
    special = sampled[np.random.default_rng(1).choice(sampled.size, 1000, replace=False)]
    K[0, 0, special] = 40.0 * d + 0.05 * torch.randn((1000, 128), generator=g)
    K = K.to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, 128), generator=g).to(torch.bfloat16)
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "bf16", K=K, V=V, side_stream=False)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    rng = np.random.default_rng(2)
    for t in range(4):
        q = np.tile(d.double().numpy(), (B, Hq, 1)) + 0.05 * rng.standard_normal((B, Hq, 128))
        par.step(q, 2.0, k, label=f"misleading sample step {t}")
    st = sess.stats()
    assert st["miss_heads"] == 4 and st["guided_selects"] == 0
    sess.close()
    # the same shape with ordinary keys takes the guided path
    sess, Kb, Ksb, Vsb = H.make_session(B, Hq, Hkv, N, k, "bf16", seed=12, side_stream=False)
    par = H.Parity(sess, "bf16", Kb, Ksb, Vsb)
    chain = W.QueryChain(B, Hq, 128, 0.95, 12)
    for t in range(4):
        par.step(chain.next(), 2.0, k, label=f"ordinary keys step {t}")
    st = sess.stats()
    assert st["miss_heads"] == 4 and st["guided_selects"] == 4
    sess.close()
