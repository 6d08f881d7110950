"""Pins for the oracle's building blocks: each function in ``oracle/`` is tied to something
other than itself - a closed form, a hand-worked value (tests/golden/), a library routine
(numpy / torch / Python's sorted), or brute force on tiny inputs."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")
F16, BF16 = 0, 1


def f16_bits(x):
    return np.asarray(x, dtype=np.float16).view(np.uint16)


def bf16_bits(x):
    return torch.tensor(np.asarray(x, dtype=np.float64)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def to_bits(x, dtype):
    return f16_bits(x) if dtype == F16 else bf16_bits(x)


def widen_lib(b, dtype):
    """16-bit patterns -> float64 through numpy / torch conversions (library routines)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float64)
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


# ---------------------------------------------------------------- widening

def test_widen_every_f16_pattern_matches_numpy(oracle):
    pats = np.arange(65536, dtype=np.uint16)
    ref = pats.view(np.float16).astype(np.float64)
    got = oracle.widen(pats, F16)
    keep = ~np.isnan(ref)
    assert np.array_equal(got[keep], ref[keep])
    assert np.isnan(got[~keep]).all()
    assert np.array_equal(np.signbit(got[keep]), np.signbit(ref[keep]))


def test_widen_every_bf16_pattern_matches_torch(oracle):
    pats = np.arange(65536, dtype=np.uint16)
    ref = widen_lib(pats, BF16)
    got = oracle.widen(pats, BF16)
    keep = ~np.isnan(ref)
    assert np.array_equal(got[keep], ref[keep])
    assert np.isnan(got[~keep]).all()


# ---------------------------------------------------------------- CosSim (Section 3.1)

@pytest.mark.parametrize("dtype", [F16, BF16])
def test_cossim_closed_forms(oracle, dtype):
    D = 128
    rng = np.random.default_rng(1)
    q = to_bits(rng.standard_normal(D), dtype)
    qv = widen_lib(q, dtype)
    assert oracle.cossim(q, q, dtype) == pytest.approx(1.0, abs=1e-15)
    assert oracle.cossim(q, to_bits(-qv, dtype), dtype) == pytest.approx(-1.0, abs=1e-15)
    # positive scaling of either argument (powers of two are exact in 16 bits)
    other = to_bits(rng.standard_normal(D), dtype)
    base = oracle.cossim(q, other, dtype)
    assert oracle.cossim(to_bits(4 * qv, dtype), other, dtype) == pytest.approx(base, abs=1e-15)
    assert oracle.cossim(q, to_bits(0.25 * widen_lib(other, dtype), dtype), dtype) == pytest.approx(base, abs=1e-15)
    # orthogonal, 3-4-5 and an asymmetric pair
    a = np.zeros(D); a[0], a[1] = 3, 4
    b = np.zeros(D); b[0] = 1
    c = np.zeros(D); c[1] = 7
    d = np.zeros(D); d[0], d[1] = 4, 3
    e = np.zeros(D); e[5] = 2
    assert oracle.cossim(to_bits(a, dtype), to_bits(b, dtype), dtype) == pytest.approx(0.6, abs=1e-15)
    assert oracle.cossim(to_bits(a, dtype), to_bits(c, dtype), dtype) == pytest.approx(0.8, abs=1e-15)
    assert oracle.cossim(to_bits(a, dtype), to_bits(d, dtype), dtype) == pytest.approx(24 / 25, abs=1e-15)
    assert oracle.cossim(to_bits(a, dtype), to_bits(e, dtype), dtype) == 0.0
    # zero-norm argument: the reading taken is -1
    z = to_bits(np.zeros(D), dtype)
    assert oracle.cossim(z, q, dtype) == -1.0
    assert oracle.cossim(q, z, dtype) == -1.0


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_cossim_matches_numpy_on_random_pairs(oracle, dtype):
    rng = np.random.default_rng(2)
    for _ in range(20):
        a = to_bits(rng.standard_normal(128), dtype)
        b = to_bits(rng.standard_normal(128) * 3, dtype)
        av, bv = widen_lib(a, dtype), widen_lib(b, dtype)
        ref = float(av @ bv) / (np.linalg.norm(av) * np.linalg.norm(bv))
        assert oracle.cossim(a, b, dtype) == pytest.approx(ref, abs=1e-14)


# ---------------------------------------------------------------- Eq. (2)

def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [c.strip() for c in line.split(";")]


def test_eq2_hand_worked_values(oracle):
    n = 0
    for w, sims, want in _rows("eq2_aggregation.txt"):
        w = [float(x) for x in w.split(",")]
        sims = [float(x) for x in sims.split(",")]
        assert oracle.aggregate(sims, w) == pytest.approx(float(Fraction(want)), abs=1e-15)
        n += 1
    assert n == 6


def test_eq2_properties(oracle):
    rng = np.random.default_rng(3)
    for _ in range(50):
        m = int(rng.integers(1, 9))
        sims = rng.uniform(0.05, 1.0, m)
        w = rng.uniform(0.1, 2.0, m)
        s = oracle.aggregate(sims, w)
        assert sims.min() - 1e-15 <= s <= float((w * sims).sum() / w.sum()) + 1e-15
        assert oracle.aggregate(sims, None) == pytest.approx(oracle.aggregate(sims, np.ones(m)), abs=0)
        # rule 2 of Section 4.2: more importance on the lowest similarity pulls the aggregate down
        w2 = w.copy(); w2[np.argmin(sims)] *= 4
        assert oracle.aggregate(sims, w2) <= s + 1e-15
    # a non-positive similarity in the group: the reading taken is -1
    assert oracle.aggregate([0.9, 0.0, 0.9], None) == -1.0
    assert oracle.aggregate([0.9, -0.2], [1.0, 1.0]) == -1.0


# ---------------------------------------------------------------- Eq. (3)-(5), D_i

def test_eq345_closed_forms(oracle):
    n = 0
    for s, eta, p, want, _why in _rows("eq345_thresholds.txt"):
        assert oracle.adaptive_tau(float(s), float(eta), float(p)) == pytest.approx(float(want), abs=1e-12)
        n += 1
    assert n == 8
    # monotone: a more important head gets a larger threshold, bounded by eta
    taus = [oracle.adaptive_tau(s, 0.8, 3) for s in np.linspace(0, 1, 21)]
    assert all(b >= a for a, b in zip(taus, taus[1:]))
    assert taus[0] == pytest.approx(-1.0) and taus[-1] == pytest.approx(0.8)


def test_reuse_difficulty(oracle):
    assert oracle.reuse_difficulty(0.8, 0.9, 0.1) == pytest.approx(0.0, abs=1e-15)
    assert oracle.reuse_difficulty(0.8, 0.6, 0.05) == pytest.approx(0.25, abs=1e-15)


# ---------------------------------------------------------------- Eq. (1) scores

@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("G", [1, 4, 5])
def test_scores_match_numpy_matmul(oracle, dtype, G):
    rng = np.random.default_rng(4 + G)
    N, D = 97, 128
    q = to_bits(rng.standard_normal((G, D)), dtype)
    K = to_bits(rng.standard_normal((N, D)) * 2, dtype)
    ref = (widen_lib(K, dtype) @ widen_lib(q, dtype).T).max(axis=1)
    got = oracle.scores(q, K, dtype)
    assert np.allclose(got, ref, rtol=0, atol=1e-12)


def test_scores_are_not_symmetric_in_head_and_key_index(oracle):
    # a transposed operand or a min-instead-of-max would fail here
    D = 8
    q = np.zeros((2, D)); q[0, 0] = 1; q[1, 1] = 1
    K = np.zeros((3, D)); K[0, 0] = 5; K[0, 1] = -7; K[1, 0] = -2; K[1, 1] = 3; K[2, 0] = -1; K[2, 1] = -4
    got = oracle.scores(f16_bits(q), f16_bits(K), F16)
    assert got.tolist() == [5.0, 3.0, -1.0]


# ---------------------------------------------------------------- top-k

def brute_topk(S, k):
    S = [0.0 if s == 0 else float(s) for s in S]
    order = sorted(range(len(S)), key=lambda n: (-S[n], n))
    return sorted(order[:k]), S[order[k - 1]]


def test_topk_brute_force_tiny(oracle):
    rng = np.random.default_rng(5)
    for trial in range(200):
        N = int(rng.integers(1, 65))
        k = int(rng.integers(1, N + 1))
        # few distinct values -> many ties
        S = rng.integers(-3, 4, N).astype(np.float64) if trial % 2 else rng.standard_normal(N)
        idx, kth = oracle.topk(S, k)
        want, wkth = brute_topk(S, k)
        assert idx.tolist() == want
        assert kth == wkth


def test_topk_matches_torch_topk_on_distinct_scores(oracle):
    rng = np.random.default_rng(6)
    S = rng.permutation(5000).astype(np.float64) * 0.37 - 800
    idx, kth = oracle.topk(S, 300)
    tv, ti = torch.topk(torch.from_numpy(S), 300)
    assert idx.tolist() == sorted(ti.tolist())
    assert kth == float(tv[-1])


def test_topk_ties_take_lowest_index_and_signed_zero(oracle):
    idx, _ = oracle.topk(np.full(40, 1.25), 7)
    assert idx.tolist() == list(range(7))
    S = np.array([-1.0, -0.0, 0.0, -0.0, 0.0, -2.0])
    idx, kth = oracle.topk(S, 2)
    assert idx.tolist() == [1, 2] and kth == 0.0
    S = np.array([3.0, 1.0, 3.0, 1.0, 3.0, 1.0])
    assert oracle.topk(S, 4)[0].tolist() == [0, 1, 2, 4]
    with pytest.raises(ValueError):
        oracle.topk(S, 7)


def test_topk_invariant_under_positive_query_scaling(oracle):
    # Section 3.1: the ordering of qkscores does not depend on ||q||
    rng = np.random.default_rng(7)
    q = rng.standard_normal((4, 128))
    K = f16_bits(rng.standard_normal((300, 128)))
    a = oracle.topk(oracle.scores(f16_bits(q), K, F16), 30)[0]
    b = oracle.topk(oracle.scores(f16_bits(widen_lib(f16_bits(q), F16) * 8), K, F16), 30)[0]
    assert a.tolist() == b.tolist()


def test_topk_selects_planted_keys(oracle):
    rng = np.random.default_rng(8)
    q = rng.standard_normal((1, 128)); q /= np.linalg.norm(q)
    K = rng.standard_normal((500, 128))
    planted = [3, 77, 499]
    for n in planted:
        K[n] = 40 * q[0]
    idx, _ = oracle.topk(oracle.scores(bf16_bits(q), bf16_bits(K), BF16), 3)
    assert idx.tolist() == planted


# ---------------------------------------------------------------- slot diff

def test_diff_worked_example(oracle):
    g = {}
    with open(os.path.join(GOLD, "diff_worked_example.txt")) as f:
        for line in f:
            if not line.startswith("#") and ":" in line:
                key, v = line.split(":")
                g[key.strip()] = [int(x) for x in v.split()]
    sl, hm, ms, mt = oracle.diff(True, 12, g["old_slots"], g["new_set"])
    assert sl.tolist() == g["new_slots"]
    assert hm.tolist() == g["hit_mask"]
    assert ms.tolist() == g["miss_slot"] and mt.tolist() == g["miss_tok"]


def test_diff_invariants_random(oracle):
    rng = np.random.default_rng(9)
    for _ in range(200):
        N = int(rng.integers(2, 200))
        k = int(rng.integers(1, N + 1))
        old = rng.permutation(N)[:k].astype(np.int32)
        new = np.sort(rng.permutation(N)[:k]).astype(np.int32)
        valid = bool(rng.integers(0, 2))
        sl, hm, ms, mt = oracle.diff(valid, N, old, new)
        assert sorted(sl.tolist()) == new.tolist()
        if valid:
            inter = set(old.tolist()) & set(new.tolist())
            assert int(hm.sum()) == len(inter)
            assert [int(t) for t, h in zip(new, hm) if h] == sorted(inter)
            # rows that stay keep their slot
            for j in range(k):
                if old[j] in inter:
                    assert sl[j] == old[j]
            assert len(ms) == k - len(inter)
        else:
            assert hm.sum() == 0 and ms.tolist() == list(range(k)) and mt.tolist() == new.tolist()
        assert (np.diff(ms) > 0).all() and (np.diff(mt) > 0).all()
        assert sl[ms].tolist() == mt.tolist()


def test_diff_rejects_malformed_state(oracle):
    with pytest.raises(ValueError):
        oracle.diff(True, 10, [1, 1, 2], [0, 1, 2])
    with pytest.raises(ValueError):
        oracle.diff(True, 10, [1, 11, 2], [0, 1, 2])


# ---------------------------------------------------------------- attention (Section 2.1)

def sdpa(q, K, V):
    """torch's scaled_dot_product_attention in fp64 (default scale 1/sqrt(D))."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    return torch.nn.functional.scaled_dot_product_attention(t(q)[None, None, None, :], t(K)[None, None], t(V)[None, None])[0, 0, 0].numpy()


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_attention_matches_torch_sdpa(oracle, dtype):
    rng = np.random.default_rng(10)
    for k in (1, 2, 37, 256):
        q = to_bits(rng.standard_normal(128) * 2, dtype)
        K = to_bits(rng.standard_normal((k, 128)), dtype)
        V = to_bits(rng.standard_normal((k, 128)) * 3, dtype)
        out, w = oracle.attention(q, K, V, dtype)
        ref = sdpa(widen_lib(q, dtype), widen_lib(K, dtype), widen_lib(V, dtype))
        assert np.allclose(out, ref, rtol=0, atol=1e-12)
        assert (w >= 0).all() and w.sum() == pytest.approx(1.0, abs=1e-13)


def test_attention_special_cases(oracle):
    rng = np.random.default_rng(11)
    D, k = 128, 50
    q = f16_bits(rng.standard_normal(D))
    V = f16_bits(rng.standard_normal((k, D)))
    # all keys equal -> uniform weights -> mean of the V rows
    K = f16_bits(np.tile(rng.standard_normal(D), (k, 1)))
    out, w = oracle.attention(q, K, V, F16)
    assert np.allclose(w, 1.0 / k, atol=1e-15)
    assert np.allclose(out, widen_lib(V, F16).mean(axis=0), atol=1e-13)
    # permuting the slots leaves the output unchanged
    K = f16_bits(rng.standard_normal((k, D)))
    perm = rng.permutation(k)
    a, _ = oracle.attention(q, K, V, F16)
    b, _ = oracle.attention(q, K[perm], V[perm], F16)
    assert np.allclose(a, b, atol=1e-13)
    # one dominant key -> its V row
    qv = widen_lib(q, F16)
    Kd = widen_lib(K, F16); Kd[17] = 30 * qv
    out, w = oracle.attention(q, f16_bits(Kd), V, F16)
    assert w[17] > 1 - 1e-12
    assert np.allclose(out, widen_lib(V, F16)[17], atol=1e-9)
    # the 1/sqrt(D) scale is there: two keys with q.k = +-sqrt(D) ln(3)/2 weigh 3:1
    q2 = np.zeros(D); q2[0] = 1
    K2 = np.zeros((2, D)); K2[0, 0] = 1; K2[1, 0] = -1
    V2 = np.zeros((2, D)); V2[0, 1] = 1; V2[1, 2] = 1
    _, w = oracle.attention(f16_bits(q2 * 8), f16_bits(K2), f16_bits(V2), F16)
    x = 8 / math.sqrt(D)
    assert w[0] / w[1] == pytest.approx(math.exp(2 * x), rel=1e-13)


def test_attention_survives_huge_logits(oracle):
    # logits of +-1448 would overflow exp() without the max subtraction; the softmax is still a
    # two-way split between the two best keys
    D = 128
    q = np.zeros(D); q[0] = 256
    K = np.zeros((3, D)); K[0, 0] = 64; K[1, 0] = 64; K[2, 0] = -64
    V = np.zeros((3, D)); V[0, 1] = 2; V[1, 2] = 4; V[2, 3] = 8
    out, w = oracle.attention(bf16_bits(q), bf16_bits(K), bf16_bits(V), BF16)
    assert w.tolist() == [0.5, 0.5, 0.0]
    assert out[1] == 1.0 and out[2] == 2.0 and out[3] == 0.0
