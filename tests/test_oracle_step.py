"""Pins for the oracle's whole step (Algorithm 1): the limiting cases the method fixes, and a
set-based restatement of Algorithm 1 (whole-head Gather, no slots) run beside it on small inputs."""
import numpy as np
import pytest
import torch

from paper_2511_14510_amd import workload as W

F16, BF16 = 0, 1


def widen_lib(b, dtype):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float64)
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def sdpa(q, K, V):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    return torch.nn.functional.scaled_dot_product_attention(t(q)[None, None, None, :], t(K)[None, None], t(V)[None, None])[0, 0, 0].numpy()


def make_case(B=2, Hq=8, Hkv=2, N=300, dtype="bf16", seed=7, steps=8, rho=0.95, **chain_kw):
    K, V = W.make_kv(B, Hkv, N, 128, dtype, seed)
    chain = W.QueryChain(B, Hq, 128, rho, seed, **chain_kw)
    qs = [W.bits(W.round_to(chain.next(), dtype)) for _ in range(steps)]
    return W.bits(K), W.bits(V), qs, W.DTYPE_CODES[dtype]


def run(oracle, Kb, Vb, qs, code, k, tau, k_max=None, importance=None):
    B, Hkv = Kb.shape[:2]
    Hq = qs[0].shape[1]
    st = oracle.State.empty(B, Hq, Hkv, 128, k_max or k)
    res = []
    for q in qs:
        before = st.copy()
        r = oracle.step(st, q, Kb, Kb, Vb, tau, k, code, importance=importance, want_weights=True)
        res.append((r, before, st.copy()))
    return res


def brute_set(qg, Kp, k):
    """Top-k set of one pair by a full Python sort under (score desc, index asc)."""
    S = (Kp @ qg.T).max(axis=1)
    order = sorted(range(len(S)), key=lambda n: (-(0.0 if S[n] == 0 else S[n]), n))
    return sorted(order[:k])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_k_equals_N_is_dense_attention(oracle, dtype):
    Kb, Vb, qs, code = make_case(N=96, dtype=dtype, steps=5)
    Kd, Vd = widen_lib(Kb, code), widen_lib(Vb, code)
    # every step, every head: sparse attention over all N slots == dense attention (torch SDPA)
    for tau in (0.9, 2.0):
        results = run(oracle, Kb, Vb, qs, code, k=96, tau=tau)
        for t, (r, _, st) in enumerate(results):
            qd = widen_lib(qs[t], code)
            for b in range(2):
                for hq in range(8):
                    ref = sdpa(qd[b, hq], Kd[b, hq // 4], Vd[b, hq // 4])
                    assert np.allclose(r.out[b, hq], ref, atol=1e-12)
            assert np.array_equal(r.topk_idx, np.tile(np.arange(96, dtype=np.int32), (4, 1)))
            if t > 0:  # nothing can be missing from a cache that holds everything
                assert r.hit_mask.all() and (r.n_filled == 0).all()


def test_tau_above_one_refreshes_every_step(oracle):
    Kb, Vb, qs, code = make_case()
    Kd = widen_lib(Kb, code)
    for t, (r, _, st) in enumerate(run(oracle, Kb, Vb, qs, code, k=24, tau=2.0)):
        assert not r.reuse_flags.any()
        qd = widen_lib(qs[t], code)
        for p in range(4):
            b, h = divmod(p, 2)
            assert r.topk_idx[p].tolist() == brute_set(qd[b, 4 * h:4 * h + 4], Kd[b, h], 24)
        assert np.array_equal(st.prev_q, qs[t])


def test_tau_minus_one_never_changes_the_set(oracle):
    Kb, Vb, qs, code = make_case(rho=0.3)
    results = run(oracle, Kb, Vb, qs, code, k=24, tau=-1.0)
    first = results[0][0]
    assert not first.reuse_flags.any() and not first.hit_mask.any()
    assert (first.n_filled == 24).all()
    for t, (r, before, st) in enumerate(results[1:], 1):
        assert r.reuse_flags.all() and r.hit_mask.all() and (r.n_filled == 0).all()
        assert np.array_equal(r.topk_idx, first.topk_idx)
        assert np.array_equal(st.prev_q, qs[0])          # the label is rewritten only on a miss
        for a, b in zip((before.slot_idx, before.K_slots, before.V_slots), (st.slot_idx, st.K_slots, st.V_slots)):
            assert np.array_equal(a, b)                   # a reuse step leaves the cache untouched


@pytest.mark.parametrize("dtype,G", [("bf16", 4), ("f16", 5), ("bf16", 1)])
def test_against_set_based_algorithm_1(oracle, dtype, G):
    """Algorithm 1 written with the cache as a set of tokens (K_c, V_c = Gather(K, V, index) on every
    miss, no slots, no diff) and library pieces: numpy dot products, Python sort, torch SDPA."""
    Hkv, B, N, k, tau = 2, 2, 257, 19, 0.9
    Hq = Hkv * G
    Kb, Vb, qs, code = make_case(B=B, Hq=Hq, Hkv=Hkv, N=N, dtype=dtype, steps=24, seed=11)
    Kd, Vd = widen_lib(Kb, code), widen_lib(Vb, code)
    results = run(oracle, Kb, Vb, qs, code, k=k, tau=tau, k_max=k + 3)
    label = {}
    cached = {}
    n_reuse = 0
    for t, (r, before, st) in enumerate(results):
        qd = widen_lib(qs[t], code)
        for p in range(B * Hkv):
            b, h = divmod(p, Hkv)
            qg = qd[b, h * G:(h + 1) * G]
            reuse = False
            if p in label:
                sims = [float(a @ c) / (np.linalg.norm(a) * np.linalg.norm(c)) for a, c in zip(qg, label[p])]
                assert np.allclose(r.sim[b, h * G:(h + 1) * G], sims, atol=1e-13)
                s = -1.0 if min(sims) <= 0 else len(sims) / sum(1.0 / x for x in sims)
                assert abs(s - tau) > 1e-9
                reuse = s >= tau
            assert bool(r.reuse_flags[p]) == reuse
            if not reuse:
                new = brute_set(qg, Kd[b, h], k)
                old = cached.get(p, [])
                assert r.hit_mask[p].tolist() == [int(n in old) for n in new]
                assert r.n_filled[p] == len(set(new) - set(old))
                cached[p] = new
                label[p] = qg.copy()
            n_reuse += reuse
            assert r.topk_idx[p].tolist() == cached[p]
            # the slots hold exactly the gathered rows, bit for bit, in some order
            sl = st.slot_idx[p, :k]
            assert sorted(sl.tolist()) == cached[p]
            assert np.array_equal(st.K_slots[p, :k], Kb[b, h][sl])
            assert np.array_equal(st.V_slots[p, :k], Vb[b, h][sl])
            for g in range(G):
                ref = sdpa(qg[g], Kd[b, h][cached[p]], Vd[b, h][cached[p]])
                assert np.allclose(r.out[b, h * G + g], ref, atol=1e-12)
                assert r.weights[b, h * G + g].sum() == pytest.approx(1.0, abs=1e-13)
    total = len(results) * B * Hkv
    assert 0.2 < n_reuse / total < 0.95   # both branches are exercised


def test_importance_weights_enter_the_gate(oracle):
    Kb, Vb, qs, code = make_case(B=1, Hq=4, Hkv=1, N=64, steps=2)
    # step 2: replace head 0's query by one at cosine ~0.5 with its label, keep the others
    q1 = widen_lib(qs[0], code)
    rng = np.random.default_rng(0)
    e = rng.standard_normal(128); e -= (e @ q1[0, 0]) * q1[0, 0] / (q1[0, 0] @ q1[0, 0]); e /= np.linalg.norm(e)
    q2 = q1.copy(); q2[0, 0] = 0.5 * q1[0, 0] / np.linalg.norm(q1[0, 0]) + np.sqrt(0.75) * e
    q2b = W.bits(W.round_to(q2, "bf16"))
    for imp, want_reuse in (([1e-3, 1, 1, 1], True), ([5, 1, 1, 1], False)):
        st = oracle.State.empty(1, 4, 1, 128, 8)
        oracle.step(st, qs[0], Kb, Kb, Vb, 0.8, 8, code, importance=imp)
        r = oracle.step(st, q2b, Kb, Kb, Vb, 0.8, 8, code, importance=imp)
        sims = r.sim[0]
        w = np.asarray(imp, dtype=np.float64)
        assert r.s_agg[0] == pytest.approx(w.sum() / (w / sims).sum(), abs=1e-14)
        assert bool(r.reuse_flags[0]) == want_reuse


def test_pair_mask_limits_the_work(oracle):
    Kb, Vb, qs, code = make_case(steps=3)
    full = run(oracle, Kb, Vb, qs, code, k=16, tau=0.9)
    st = oracle.State.empty(2, 8, 2, 128, 16)
    mask = np.array([0, 1, 0, 1], np.uint8)
    for t, q in enumerate(qs):
        r = oracle.step(st, q, Kb, Kb, Vb, 0.9, 16, code, pair_mask=mask)
        for p in (1, 3):
            assert np.array_equal(r.topk_idx[p], full[t][0].topk_idx[p])
            assert r.reuse_flags[p] == full[t][0].reuse_flags[p]
        assert st.valid.tolist() == [0, 1, 0, 1]
        assert (st.slot_idx[[0, 2]] == -1).all()


def test_query_chain_recipe():
    """The synthetic queries behave as the recipe says: unit norm, adjacent cosine near rho,
    exactly rho in the exact variant, and a reuse rate in the range the paper's Table 3 spans."""
    ch = W.QueryChain(2, 8, 128, 0.95, 3)
    qs = [ch.next() for _ in range(200)]
    cs = np.array([(a * b).sum(-1) for a, b in zip(qs, qs[1:])])
    assert np.allclose(np.linalg.norm(qs[5], axis=-1), 1.0, atol=1e-12)
    assert 0.93 < cs.mean() < 0.97 and cs.std() < 0.03
    ch = W.QueryChain(1, 4, 128, np.array([0.3, 0.6, 0.9, 0.99]), 3, exact=True)
    a = ch.next(); b = ch.next()
    assert np.allclose((a * b).sum(-1)[0], [0.3, 0.6, 0.9, 0.99], atol=1e-12)
    ch = W.QueryChain(1, 4, 128, 0.95, 3, q_norm=5.0)
    assert np.allclose(np.linalg.norm(ch.next(), axis=-1), 5.0)


def test_kv_recipe_has_outlier_channels():
    K, V = W.make_kv(1, 2, 4096, 128, "bf16", 5)
    ch = W.outlier_channels(2, 128, 5)
    for T in (K, V):
        sd = T.float().std(dim=2)[0]           # [Hkv, D]
        for h in range(2):
            mask = np.zeros(128, bool); mask[ch[h]] = True
            assert len(set(ch[h].tolist())) == 4
            assert (sd[h][torch.from_numpy(mask)] > 7).all() and (sd[h][torch.from_numpy(~mask)] < 1.2).all()
    K2, _ = W.make_kv(1, 2, 4096, 128, "bf16", 5)
    assert torch.equal(K, K2)


def test_gate_reuses_on_equality(oracle):
    """cos = 1/2 exactly against tau = 1/2: "at or above" reuses; just above tau misses."""
    Kb, Vb, _, code = make_case(B=1, Hq=1, Hkv=1, N=64, steps=1)
    a = np.zeros((1, 1, 128)); a[0, 0, :4] = 1
    b = np.zeros((1, 1, 128)); b[0, 0, 0] = 1
    qa, qb = W.bits(W.round_to(a, "bf16")), W.bits(W.round_to(b, "bf16"))
    for tau, want in ((0.5, 1), (np.nextafter(0.5, 1.0), 0), (0.25, 1)):
        st = oracle.State.empty(1, 1, 1, 128, 8)
        oracle.step(st, qa, Kb, Kb, Vb, tau, 8, code)
        r = oracle.step(st, qb, Kb, Kb, Vb, tau, 8, code)
        assert r.sim[0, 0] == 0.5 and r.reuse_flags[0] == want


def test_hybrid_attention_is_attention_over_the_concatenation(oracle):
    """Section 6.2: the attention reads the cached rows and the append-only buffer as one set."""
    rng = np.random.default_rng(12)
    bits = lambda x: W.bits(W.round_to(x, "bf16"))
    for k, na in ((5, 1), (40, 17), (1, 64)):
        q = bits(rng.standard_normal(128))
        Kc, Vc = bits(rng.standard_normal((k, 128))), bits(rng.standard_normal((k, 128)))
        Ka, Va = bits(rng.standard_normal((na, 128)) * 2), bits(rng.standard_normal((na, 128)))
        out, w = oracle.attention_hybrid(q, Kc, Vc, Ka, Va, BF16)
        ref = sdpa(widen_lib(q, BF16), np.concatenate([widen_lib(Kc, BF16), widen_lib(Ka, BF16)]),
                   np.concatenate([widen_lib(Vc, BF16), widen_lib(Va, BF16)]))
        assert np.allclose(out, ref, atol=1e-12)
        assert w.shape == (k + na,) and w.sum() == pytest.approx(1.0, abs=1e-13)


def test_sink_and_recent_tokens_are_always_retrieved(oracle):
    """Section 7.1: 4 sink and 64 recent tokens stay in the cache.  The first n_sink and the last n_recent
    tokens belong to every retrieved set; the other slots go to the best of the remaining tokens."""
    Kb, Vb, qs, code = make_case(B=1, Hq=4, Hkv=1, N=400, steps=6)
    Kd = widen_lib(Kb, code)
    n_sink, n_recent, k = 4, 64, 100
    st = oracle.State.empty(1, 4, 1, 128, k)
    forced = list(range(n_sink)) + list(range(400 - n_recent, 400))
    for t, q in enumerate(qs):
        r = oracle.step(st, q, Kb, Kb, Vb, 2.0, k, code, n_sink=n_sink, n_recent=n_recent)
        got = r.topk_idx[0].tolist()
        assert set(forced) <= set(got)
        qd = widen_lib(q, code)[0]
        S = (Kd[0, 0] @ qd.T).max(axis=1)
        middle = [n for n in range(400) if n not in forced]
        best = sorted(middle, key=lambda n: (-S[n], n))[:k - len(forced)]
        assert got == sorted(forced + best)
    # with no room for anything else the set is exactly the forced tokens
    st = oracle.State.empty(1, 4, 1, 128, 68)
    r = oracle.step(st, qs[0], Kb, Kb, Vb, 2.0, 68, code, n_sink=4, n_recent=64)
    assert r.topk_idx[0].tolist() == forced


def test_step_with_append_buffer_and_k_equals_N_is_dense_over_everything(oracle):
    Kb, Vb, qs, code = make_case(B=2, Hq=8, Hkv=2, N=80, steps=5)
    rng = np.random.default_rng(13)
    cap = 12
    Ka = W.bits(W.round_to(rng.standard_normal((2, 2, cap, 128)), "bf16"))
    Va = W.bits(W.round_to(rng.standard_normal((2, 2, cap, 128)), "bf16"))
    st = oracle.State.empty(2, 8, 2, 128, 80)
    for t, q in enumerate(qs):
        n_app = t + 1                       # one generated token joins the buffer per step
        r = oracle.step(st, q, Kb, Kb, Vb, 0.9, 80, code, K_app=Ka, V_app=Va, n_app=n_app, want_weights=True)
        qd = widen_lib(q, code)
        for b in range(2):
            for hq in range(8):
                h = hq // 4
                Kall = np.concatenate([widen_lib(Kb, code)[b, h], widen_lib(Ka, code)[b, h, :n_app]])
                Vall = np.concatenate([widen_lib(Vb, code)[b, h], widen_lib(Va, code)[b, h, :n_app]])
                assert np.allclose(r.out[b, hq], sdpa(qd[b, hq], Kall, Vall), atol=1e-12)
        assert r.weights.shape == (2, 8, 80 + n_app)
