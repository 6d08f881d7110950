"""Parity at the full sizes of the five benchmark workloads, through the same Session / launch configuration
bench.py times.  The oracle follows every (batch, KV head) pair on the first and on the last step and a seeded
sample of pairs on the steps between, starting each step from the GPU's own cache state."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2511_14510_amd import binding as Q
from paper_2511_14510_amd import workload as W


def run_full(name, steps, n_sample, flags=0, side_stream=False, taus=None, all_first=True, all_last=True):
    """Runs ``steps`` steps per threshold in ``taus`` (default: the workload's own) on one session, with a reset
    and a fresh query chain between thresholds.  Returns one (Parity, stats) per threshold."""
    import gpu_harness as H
    w = W.CONFIGS[name]
    taus = [w.tau] if taus is None else list(taus)
    print(f"full-size case {name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} N={w.N} k={w.k} {w.dtype} taus={taus} steps={steps} "
          f"flags={flags} side_stream={side_stream}", flush=True)
    sess, Kb, Ksb, Vsb = H.make_session_on_gpu(w, flags, side_stream)
    rng = np.random.default_rng(w.seed)
    results = []
    for tau in taus:
        sess.reset()
        par = H.Parity(sess, w.dtype, Kb, Ksb, Vsb)
        chain = W.chain_for(w)
        for t in range(steps):
            if (t == 0 and all_first) or (t == steps - 1 and all_last):
                pairs = range(w.P)
            else:
                pairs = rng.choice(w.P, size=min(n_sample, w.P), replace=False)
            par.step(chain.next(), tau, w.k, label=f"{name} tau {tau} step {t}", pairs=pairs)
            print(f"  tau {tau} step {t}: ok on {len(par.pairs)} pairs, reuse so far {par.n_reuse}, miss {par.n_miss}, "
                  f"band {par.n_band}, max err {par.max_err:.2e}", flush=True)
        results.append((par, sess.stats()))
    sess.close()
    del sess, Kb, Ksb, Vsb
    torch.cuda.empty_cache()
    return results, w


def test_llama3_8b_32k_full_size():
    [(par, st)], w = run_full("llama3_8b_32k", steps=8, n_sample=12)
    assert par.n_reuse > 0 and par.n_miss > w.P
    assert 0.3 < st["reuse_heads"] / (st["reuse_heads"] + st["miss_heads"]) < 0.9
    assert st["bytes_filled_host"] == 0 and st["bytes_filled_dev"] == 512 * st["slot_misses"]


def test_llama3_8b_32k_full_size_fill_kernel_on_side_stream():
    run_full("llama3_8b_32k", steps=4, n_sample=8, flags=Q.QSAC_FLAG_FILL_KERNEL, side_stream=True, all_first=False)


def test_qwen25_14b_128k_offload_full_size():
    [(par, st)], w = run_full("qwen25_14b_128k_offload", steps=5, n_sample=8)
    assert par.n_miss > w.P and par.n_reuse > 0
    assert st["bytes_filled_host"] == 512 * st["slot_misses"]


def test_qwen25_offload_full_size_fill_kernel_on_side_stream():
    run_full("qwen25_14b_128k_offload", steps=3, n_sample=6, flags=Q.QSAC_FLAG_FILL_KERNEL, side_stream=True,
             all_first=False, all_last=False)


def test_long_1m_full_size():
    [(par, st)], w = run_full("long_1m", steps=4, n_sample=8)
    assert par.n_miss >= w.P
    assert st["bytes_filled_host"] == 256 * st["slot_misses"]          # only the V rows live on the host


def test_low_sim_stress_full_size():
    """All 256 pairs on the first and last step of each threshold of the sweep; the correlation differs from KV
    head to KV head, so both branches of the gate are taken at every threshold and the reuse rate falls as the
    threshold rises."""
    results, w = run_full("low_sim_stress", steps=4, n_sample=16, taus=(0.8, 0.9, 0.95))
    rates = []
    for par, st in results:
        assert par.n_reuse > 0 and par.n_miss > w.P
        rates.append(st["reuse_heads"] / (st["reuse_heads"] + st["miss_heads"]))
        assert st["bytes_filled_host"] == 512 * st["slot_misses"]
    assert rates[0] > rates[1] >= rates[2] > 0, rates     # four steps tell 0.9 from 0.95 only by a few pairs


def test_low_sim_stress_full_size_staggered_schedule():
    """The largest workload under QSAC_FLAG_STAGGER (what bench.py's headline line runs): four slices of eight
    batch elements on two streams; every pair on the first step, a sample afterwards."""
    [(par, st)], w = run_full("low_sim_stress", steps=3, n_sample=16, flags=Q.QSAC_FLAG_STAGGER, side_stream=True,
                              all_last=False)
    assert par.n_reuse > 0 and par.n_miss > w.P
    assert st["bytes_filled_host"] == 512 * st["slot_misses"]
