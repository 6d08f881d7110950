"""Parity at the full sizes of the five benchmark workloads, through the same Session / launch configuration
bench.py times.  The oracle follows a seeded sample of (batch, KV head) pairs every step (all pairs on
the first step, where every head misses), starting each step from the GPU's own cache state."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2511_14510_amd import binding as Q
from paper_2511_14510_amd import workload as W


def run_full(name, steps, n_sample, flags=0, side_stream=False, tau=None, all_first=True):
    import gpu_harness as H
    w = W.CONFIGS[name]
    tau = w.tau if tau is None else tau
    print(f"full-size case {name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} N={w.N} k={w.k} {w.dtype} tau={tau} steps={steps} "
          f"flags={flags} side_stream={side_stream}", flush=True)
    sess, Kb, Ksb, Vsb = H.make_session_on_gpu(w, flags, side_stream)
    par = H.Parity(sess, w.dtype, Kb, Ksb, Vsb)
    chain = W.chain_for(w)
    rng = np.random.default_rng(w.seed)
    for t in range(steps):
        if t == 0 and all_first:
            pairs = range(w.P)
        else:
            pairs = rng.choice(w.P, size=min(n_sample, w.P), replace=False)
        par.step(chain.next(), tau, w.k, label=f"{name} step {t}", pairs=pairs)
        print(f"  step {t}: ok, reuse so far {par.n_reuse}, miss {par.n_miss}, band {par.n_band}, "
              f"max err {par.max_err:.2e}", flush=True)
    st = sess.stats()
    sess.close()
    del sess, Kb, Ksb, Vsb
    torch.cuda.empty_cache()
    return par, st, w


def test_llama3_8b_32k_full_size():
    par, st, w = run_full("llama3_8b_32k", steps=8, n_sample=12)
    assert par.n_reuse > 0 and par.n_miss > w.P
    assert 0.3 < st["reuse_heads"] / (st["reuse_heads"] + st["miss_heads"]) < 0.9


def test_llama3_8b_32k_full_size_fill_kernel_on_side_stream():
    run_full("llama3_8b_32k", steps=4, n_sample=8, flags=Q.QSAC_FLAG_FILL_KERNEL, side_stream=True, all_first=False)


def test_qwen25_14b_128k_offload_full_size():
    par, st, w = run_full("qwen25_14b_128k_offload", steps=5, n_sample=8)
    assert par.n_miss > w.P


def test_qwen25_offload_full_size_fill_kernel_on_side_stream():
    run_full("qwen25_14b_128k_offload", steps=3, n_sample=6, flags=Q.QSAC_FLAG_FILL_KERNEL, side_stream=True,
             all_first=False)


def test_long_1m_full_size():
    par, st, w = run_full("long_1m", steps=3, n_sample=8)
    assert par.n_miss >= w.P


def test_low_sim_stress_full_size():
    par, st, w = run_full("low_sim_stress", steps=3, n_sample=10, all_first=False, tau=0.9)
    assert par.n_miss > 0
