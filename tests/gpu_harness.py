"""Step-by-step comparison of the HIP path (through the C ABI) with the oracle.

At every step the oracle starts from the GPU's own cache state (label, slot table, slot rows,
validity) read back before the step, so a tolerated near-tie difference in one step's index
set cannot cascade into the next.  Bars (from the benchmark spec):
  reuse flags, hit masks, index sets   bit-exact; an index-set difference is accepted only for
                                       tokens whose ORACLE score lies within 1e-4 relative of
                                       the oracle's k-th score
  attention output                     max-abs error <= 2e-3
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2511_14510_amd import binding as Q
from paper_2511_14510_amd import workload as W

OUT_TOL = 2e-3
BAND = 1e-4
GATE_MARGIN = 1e-9


def host_state(sess: Q.Session) -> oracle.State:
    return oracle.State(
        valid=(sess.valid().cpu().numpy() != 0).astype(np.uint8),
        prev_q=W.bits(sess.prev_q),
        slot_idx=sess.slot_idx.cpu().numpy().reshape(sess.P, sess.k_max).copy(),
        K_slots=W.bits(sess.K_slots).reshape(sess.P, sess.k_max, 128).copy(),
        V_slots=W.bits(sess.V_slots).reshape(sess.P, sess.k_max, 128).copy())


class Parity:
    """Runs steps on a Session and checks each against the oracle."""

    def __init__(self, sess: Q.Session, dtype: str, Kb, Ksrc_b, Vsrc_b, importance=None, pair_mask=None,
                 n_sink=0, n_recent=0, Kapp_b=None, Vapp_b=None, launch=None):
        """``launch(q_dev, tau, k)`` replaces ``sess.step`` as the way a step reaches the GPU (a graph replay,
        the allocation-free entry point); it must leave the results in the session's tensors."""
        self.s, self.dtype, self.code = sess, dtype, W.DTYPE_CODES[dtype]
        self.Kb, self.Ksb, self.Vsb = Kb, Ksrc_b, Vsrc_b
        self.importance = importance
        self.n_sink, self.n_recent, self.Kapp_b, self.Vapp_b = n_sink, n_recent, Kapp_b, Vapp_b
        self.launch = launch if launch is not None else sess.step
        self.pair_mask = None if pair_mask is None else np.asarray(pair_mask, np.uint8)
        self.pairs = list(range(sess.P)) if pair_mask is None else [p for p in range(sess.P) if pair_mask[p]]
        self.n_reuse = self.n_miss = self.n_band = 0
        self.max_err = 0.0
        self.min_margin = np.inf
        self.filled = 0

    def step(self, q_np64, tau, k, label="", pairs=None):
        """One step on the GPU and in the oracle; ``pairs`` limits the comparison (and the oracle's work)
        to those pairs for this step."""
        if pairs is not None:
            self.pairs = sorted(int(p) for p in pairs)
            self.pair_mask = np.zeros(self.s.P, np.uint8)
            self.pair_mask[self.pairs] = 1
        s = self.s
        G = s.Hq // s.Hkv
        qt = W.round_to(q_np64, self.dtype)
        qb = W.bits(qt)
        before = host_state(s)
        st = before.copy()
        self.launch(qt.cuda(), tau, k)
        s.sync()
        r = oracle.step(st, qb, self.Kb, self.Ksb, self.Vsb, tau, k, self.code, importance=self.importance,
                        want_scores=True, pair_mask=self.pair_mask, n_sink=self.n_sink, n_recent=self.n_recent,
                        K_app=self.Kapp_b, V_app=self.Vapp_b, n_app=s.n_app)
        after = host_state(s)
        g_reuse = s.reuse_flags.cpu().numpy().reshape(-1)
        g_topk = s.topk_idx.cpu().numpy().reshape(s.P, k)
        g_hit = s.hit_mask.cpu().numpy().reshape(s.P, k)
        g_out = s.out.cpu().numpy().astype(np.float64)
        g_sim = s.sim.cpu().numpy().astype(np.float64)
        tau_h = np.broadcast_to(np.asarray(tau, dtype=np.float64), (s.Hkv,))
        mc = s.ws_view("miss_count", torch.int32, (s.P,)).cpu().numpy()
        for p in self.pairs:
            b, h = divmod(p, s.Hkv)
            where = f"{label} pair {p}"
            heads = slice(h * G, (h + 1) * G)
            if before.valid[p]:
                if r.s_agg[p] != -1.0:   # -1 is set exactly (a non-positive cosine in the group), not computed
                    self.min_margin = min(self.min_margin, abs(r.s_agg[p] - tau_h[h]))
                    assert abs(r.s_agg[p] - tau_h[h]) > GATE_MARGIN, f"{where}: gate too close to tau to compare"
                assert np.allclose(g_sim[b, heads], r.sim[b, heads], atol=2e-6), where
            assert g_reuse[p] == r.reuse_flags[p], f"{where}: reuse flag {g_reuse[p]} != {r.reuse_flags[p]}"
            assert after.valid[p] == 1, where
            same_set = np.array_equal(g_topk[p], r.topk_idx[p])
            if not same_set:
                # only keys the oracle itself ranks within the band of its k-th score may differ
                assert not r.reuse_flags[p], f"{where}: reused set differs"
                kth = r.kth_score[p]
                diff = np.setxor1d(g_topk[p], r.topk_idx[p])
                sc = r.scores[p][diff]
                assert np.isfinite(kth) and np.all(np.abs(sc - kth) <= BAND * abs(kth)), \
                    f"{where}: index sets differ outside the band"
                assert np.all(np.diff(g_topk[p]) > 0), where
                self.n_band += 1
            if r.reuse_flags[p]:
                self.n_reuse += 1
                assert g_hit[p].all(), where
                assert mc[p] == 0, where
                assert np.array_equal(after.prev_q[b, heads], before.prev_q[b, heads]), f"{where}: label rewritten on reuse"
                assert np.array_equal(after.slot_idx[p], before.slot_idx[p]), where
                assert np.array_equal(after.K_slots[p], before.K_slots[p]), where
                assert np.array_equal(after.V_slots[p], before.V_slots[p]), where
            else:
                self.n_miss += 1
                want_hit = (np.isin(g_topk[p], before.slot_idx[p, :k]).astype(np.uint8) if before.valid[p]
                            else np.zeros(k, np.uint8))
                assert np.array_equal(g_hit[p], want_hit), f"{where}: hit mask"
                if same_set:
                    assert np.array_equal(g_hit[p], r.hit_mask[p]), where
                    assert mc[p] == r.n_filled[p], where
                    assert np.array_equal(after.slot_idx[p, :k], st.slot_idx[p, :k]), f"{where}: slot placement"
                assert mc[p] == k - int(want_hit.sum()), where
                self.filled += int(mc[p])
                assert np.array_equal(after.prev_q[b, heads], qb[b, heads]), f"{where}: label not updated on miss"
                # rows that were cached and stay cached keep their slot
                if before.valid[p]:
                    stay = np.isin(before.slot_idx[p, :k], g_topk[p])
                    assert np.array_equal(after.slot_idx[p, :k][stay], before.slot_idx[p, :k][stay]), where
            sl = after.slot_idx[p, :k]
            assert np.array_equal(np.sort(sl), g_topk[p]), f"{where}: slots do not hold the reported set"
            assert np.array_equal(after.K_slots[p, :k], self.Ksb[b, h][sl]), f"{where}: K rows"
            assert np.array_equal(after.V_slots[p, :k], self.Vsb[b, h][sl]), f"{where}: V rows"
            for g in range(G):
                hq = h * G + g
                if same_set:
                    ref = r.out[b, hq]
                else:
                    if s.n_app:
                        ref, _ = oracle.attention_hybrid(qb[b, hq], after.K_slots[p, :k], after.V_slots[p, :k],
                                                         self.Kapp_b[b, h, :s.n_app], self.Vapp_b[b, h, :s.n_app], self.code)
                    else:
                        ref, _ = oracle.attention(qb[b, hq], after.K_slots[p, :k], after.V_slots[p, :k], self.code)
                err = float(np.abs(g_out[b, hq] - ref).max())
                self.max_err = max(self.max_err, err)
                assert err <= OUT_TOL, f"{where} head {hq}: attention max-abs error {err:.3e}"
        return r


def make_session_on_gpu(w, flags=0, side_stream=False):
    """A full-size benchmark workload: K, V drawn on the GPU, copied once to pinned host memory (which
    is both the fill source of the offload workloads and what the oracle reads)."""
    K_dev, V_dev = W.make_kv(w.B, w.Hkv, w.N, w.D, w.dtype, w.seed, device="cuda:0")
    K_host = torch.empty(K_dev.shape, dtype=K_dev.dtype, pin_memory=True).copy_(K_dev)
    V_host = torch.empty(V_dev.shape, dtype=V_dev.dtype, pin_memory=True).copy_(V_dev)
    torch.cuda.synchronize()
    K_src = K_host if w.host_k else K_dev
    V_src = V_host if w.host_v else V_dev
    if w.host_v:
        del V_dev
    sess = Q.Session(w.B, w.Hq, w.Hkv, w.N, w.k, w.dtype, K_dev, K_src, V_src, flags=flags, side_stream=side_stream)
    Kb = K_host.view(torch.int16).numpy().view(np.uint16)
    Vb = V_host.view(torch.int16).numpy().view(np.uint16)
    return sess, Kb, Kb, Vb


def make_session(B, Hq, Hkv, N, k_max, dtype, seed=W.DEFAULT_SEED, host_k=False, host_v=False, flags=0,
                 importance=None, side_stream=True, K=None, V=None):
    """Synthetic K, V (or the given ones), a Session over them and the bit views the oracle needs."""
    if K is None:
        K, V = W.make_kv(B, Hkv, N, 128, dtype, seed)
    K_dev = K.cuda()
    K_src = K.pin_memory() if host_k else K_dev
    V_src = V.pin_memory() if host_v else V.cuda()
    sess = Q.Session(B, Hq, Hkv, N, k_max, dtype, K_dev, K_src, V_src, flags=flags, importance=importance,
                     side_stream=side_stream)
    return sess, W.bits(K), W.bits(K), W.bits(V)
