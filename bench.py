#!/usr/bin/env python3
"""Benchmark of the QSAC decode step on one MI355X.

A step is one qsac_step() over the whole batch of one attention layer (gate, scoring of the
missing heads, top-k select, slot diff, miss fill, sparse attention).  Inputs are synthetic
(see paper_2511_14510_amd/workload.py) and resident in HBM (and, for the offload workloads,
in pinned host memory) before the timed region starts.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tau T]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes the scoring kernel moves per missing pair, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (profiles/qsac_step_kernels__llama3_8b_32k_all_miss__pmc_{fetch,write}_size.txt): per launch of 64 missing
# pairs FETCH_SIZE = 262431.7 units of 2.000 KiB and WRITE_SIZE = 8242.8 units of 1.000 KiB (units calibrated
# against the 256-MiB qsac_copy_kernel of the same runs).  bench.py cannot collect counters itself.
PMC_SCORE_BYTES_PER_MISSING_PAIR = {"llama3_8b_32k": (262431.7 * 2.000 + 8242.8 * 1.000) * 1024 / 64}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="llama3_8b_32k")
    ap.add_argument("--tau", type=float, default=None, help="override the workload's threshold")
    ap.add_argument("--flags", type=int, default=0, help="extra qsac_config.flags (e.g. 4 = ALU scoring)")
    ap.add_argument("--decode-buffers", action="store_true",
                    help="4 sink + 64 recent tokens kept in every set, and an append-only buffer that grows by one "
                         "generated token per step (Sections 6.1, 6.2, 7.1)")
    ap.add_argument("--resident", type=int, default=0,
                    help="keep this many KV heads resident in HBM (Section 4.4), chosen by reuse difficulty")
    ap.add_argument("--side-stream", action="store_true",
                    help="give the library a second stream (attention of reused heads, or the fill kernel, runs on it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="skip the stage-timing passes")
    ap.add_argument("--k-fill-from-hbm", action="store_true",
                    help="not the workload as specified: take the missing K rows from the HBM copy of K that scoring "
                         "reads (K_src = K_dev), so that only V rows cross PCIe")
    ap.add_argument("--calibration-reads", type=int, default=0,
                    help="after the run, launch this many read-only kernels (qsac_calibration_read) of the attention "
                         "launch's and of the all-miss scoring launch's size: what a launch of that size can reach")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="launch this many plain 256 MiB copies first (qsac_copy_kernel), to scale profiler counters")
    ap.add_argument("--cpu-steps", type=int, default=0, help="oracle steps to time (0 = sized to ~15 s)")
    return ap.parse_args()


def make_queries(w, W, n_steps):
    import torch
    chain = W.chain_for(w)
    qs = [W.round_to(chain.next(), w.dtype) for _ in range(n_steps)]
    return torch.stack(qs)


def run_steps(sess, q_dev, tau, k, lo, hi):
    for t in range(lo, hi):
        if sess.K_app is not None:
            sess.set_appended(t + 1)   # the token generated at step t has joined the append-only buffer
        sess.step(q_dev[t], tau, k)


def h2d_peak_gbs(torch):
    """Pinned host -> device copy rate of a 1 GiB buffer: the PCIe figure the fill is held against."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    return 3 * n / (time.perf_counter() - t0) / 1e9


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the QSAC step has no inter-GPU part); use --gpus 1",
              file=sys.stderr)
        return 2
    import numpy as np
    import torch
    from paper_2511_14510_amd import binding as Q
    from paper_2511_14510_amd import workload as W

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU path)"
    Q.load()
    w = W.CONFIGS[a.workload]
    if a.k_fill_from_hbm:
        import dataclasses
        w = dataclasses.replace(w, host_k=False)
    tau = w.tau if a.tau is None else a.tau
    K_steps, W_steps = a.steps, a.warmup
    total = K_steps + W_steps

    if a.calibration_copies:
        n = 256 << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(a.calibration_copies):
            Q.qsac_calibration_copy(dst.data_ptr(), src.data_ptr(), n)
        torch.cuda.synchronize()
        del src, dst

    # ---- inputs, resident before any timing
    K_dev, V_dev = W.make_kv(w.B, w.Hkv, w.N, w.D, w.dtype, w.seed, device="cuda:0")
    K_host = V_host = None
    if w.host_k or w.host_v or not a.no_cpu_baseline:
        K_host = torch.empty(K_dev.shape, dtype=K_dev.dtype, pin_memory=True).copy_(K_dev)
        V_host = torch.empty(V_dev.shape, dtype=V_dev.dtype, pin_memory=True).copy_(V_dev)
    K_src = K_host if w.host_k else K_dev
    V_src = V_host if w.host_v else V_dev
    q_all = make_queries(w, W, total)
    V_res = res_slot = None
    if a.resident:
        # reuse difficulty D_i = tau_i - (s_hat_i - eps) from the adjacent-query cosines of the chain itself
        # (the paper profiles s_hat offline on sample sequences); the hardest heads become resident
        qf = q_all.double()
        cos = (qf[1:] * qf[:-1]).sum(-1) / (qf[1:].norm(dim=-1) * qf[:-1].norm(dim=-1))     # [T-1,B,Hq]
        cos = cos.reshape(total - 1, w.B, w.Hkv, w.G).clamp_min(1e-6)
        s_hat = (w.G / (1.0 / cos).sum(-1)).mean(dim=(0, 1))                                 # Eq. (2), then mean
        D = Q.qsac_reuse_difficulty([tau] * w.Hkv, s_hat.tolist(), 0.1)
        hard = sorted(range(w.Hkv), key=lambda h: -D[h])[:a.resident]
        res_slot = [-1] * w.Hkv
        for i, h in enumerate(sorted(hard)):
            res_slot[h] = i
        V_res = torch.stack([V_dev[:, h] for h in sorted(hard)], dim=1).contiguous()
    if w.host_v:
        V_dev = None  # the offload workloads keep V on the host only (and in V_res for resident heads)
    q_dev = q_all.cuda()
    K_app = V_app = None
    n_sink = n_recent = 0
    if a.decode_buffers:
        # the generated tokens' KV are synthetic too and resident beforehand; a step only raises the valid count
        n_sink, n_recent = 4, 64
        K_app, V_app = W.make_kv(w.B, w.Hkv, total, w.D, w.dtype, w.seed + 7, device="cuda:0")
    torch.cuda.synchronize()

    def session(flags):
        return Q.Session(w.B, w.Hq, w.Hkv, w.N, w.k, w.dtype, K_dev, K_src, V_src, flags=flags | a.flags,
                         side_stream=bool(a.side_stream), V_res=V_res, res_slot=res_slot, n_sink=n_sink,
                         n_recent=n_recent, K_app=K_app, V_app=V_app)

    # ---- timed run: K steps after W warmup steps, overlapped fill, no events inside
    sess = session(0)
    run_steps(sess, q_dev, tau, w.k, 0, W_steps)
    sess.sync()
    torch.cuda.synchronize()
    s0 = sess.stats()
    t0 = time.perf_counter()
    run_steps(sess, q_dev, tau, w.k, W_steps, total)
    sess.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    s1 = sess.stats()
    sess.close()
    d = {key: s1[key] - s0[key] for key in s1}
    pairs = w.P * K_steps
    reuse_rate = d["reuse_heads"] / pairs
    fresh_rows = d["slot_hits"] + d["slot_misses"]
    slot_hit_rate = d["slot_hits"] / fresh_rows if fresh_rows else None

    result = {
        "metric": "QSAC decode steps/s per layer", "value": K_steps / elapsed, "unit": "steps/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W_steps, "ms_per_step": 1e3 * elapsed / K_steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "n_q_heads": w.Hq, "n_kv_heads": w.Hkv, "head_dim": w.D,
                   "n_ctx": w.N, "k": w.k, "tau": tau, "rho": list(w.rho_range) if w.rho_range else w.rho,
                   "K_fill_source": "pinned host" if w.host_k else "HBM",
                   "V_fill_source": "pinned host" if w.host_v else "HBM",
                   "scoring": "alu" if (a.flags & Q.QSAC_FLAG_SCORE_VALU) else "mfma",
                   "fill": "own kernel on a side stream" if (a.flags & Q.QSAC_FLAG_FILL_KERNEL) else "folded into attention loads",
                   "side_stream": (("fill kernel" if (a.flags & Q.QSAC_FLAG_FILL_KERNEL) else "attention of reused heads")
                                   if a.side_stream else None)},
        "reuse_rate": reuse_rate, "slot_hit_rate": slot_hit_rate,
        "guided_select_rate": d["guided_selects"] / d["miss_heads"] if d["miss_heads"] else None,
        "rows_filled_per_step": d["slot_misses"] / K_steps,
        "rows_filled_from_host_per_step": ((d["slot_misses"] - d["resident_rows"]) / K_steps
                                           if (w.host_k or w.host_v) else 0.0),
    }
    if a.decode_buffers:
        result["config"].update({"n_sink": n_sink, "n_recent": n_recent, "append_rows_at_end": total})
    if a.resident:
        result["config"]["resident_kv_heads"] = sorted(hard)
        result["config"]["reuse_difficulty"] = [round(x, 4) for x in D]

    # ---- stage timing (HIP events on the stream the kernels run on), same steps, fill not overlapped
    if not a.no_profile:
        def profile(tau_p, n_warm, n_steps, extra=0):
            ps = session(Q.QSAC_FLAG_PROFILE | extra)
            run_steps(ps, q_dev, tau_p, w.k, 0, n_warm)
            ps.sync()
            _, ms0, c0 = Q.qsac_get_stage_ms(ps.ctx)
            st0 = ps.stats()
            run_steps(ps, q_dev, tau_p, w.k, n_warm, n_warm + n_steps)
            ps.sync()
            names, ms1, c1 = Q.qsac_get_stage_ms(ps.ctx)
            st1 = ps.stats()
            ps.close()
            assert c1 - c0 == n_steps
            us = [1e3 * (y - x) / n_steps for x, y in zip(ms0, ms1)]
            return names, us, {key: st1[key] - st0[key] for key in st1}

        def roof(us, dd, n_steps):
            miss_per_launch = dd["miss_heads"] / n_steps
            score_bytes = 256.0 * w.N * miss_per_launch          # K bytes one scoring launch has to read
            attn_bytes = 512.0 * w.k * w.P                        # slot bytes one attention launch has to read
            return {
                "score": {"bound": "hbm", "achieved": score_bytes / (us[1] * 1e-6) / 1e9 if miss_per_launch else 0.0,
                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "bytes_per_launch": score_bytes,
                          "us_per_launch": us[1], "missing_pairs_per_launch": miss_per_launch},
                "attn": {"bound": "hbm", "achieved": attn_bytes / (us[4] * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "bytes_per_launch": attn_bytes, "us_per_launch": us[4]},
            }

        names, us, dd = profile(tau, W_steps, K_steps)
        r = roof(us, dd, K_steps)
        sc = r["score"]
        result["roofline"] = {"bound": "hbm", "kernel": names[1], "achieved": sc["achieved"], "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": sc["achieved"] / HBM_PEAK_GBS,
                              "traffic": (PMC_SCORE_BYTES_PER_MISSING_PAIR[w.name] * sc["missing_pairs_per_launch"]
                                          if w.name in PMC_SCORE_BYTES_PER_MISSING_PAIR and not a.flags else None),
                              "bytes_per_launch": sc["bytes_per_launch"], "us_per_launch": sc["us_per_launch"],
                              "missing_pairs_per_launch": sc["missing_pairs_per_launch"]}
        result["stage_us"] = dict(zip(names, [round(x, 2) for x in us]))
        result["attn_roofline"] = {**r["attn"], "frac": r["attn"]["achieved"] / HBM_PEAK_GBS}
        # every pair misses every step: each scoring launch reads all of K
        n_all = min(K_steps, 32)
        names, us2, dd2 = profile(2.0, 2, n_all)
        r2 = roof(us2, dd2, n_all)
        result["all_miss"] = {"tau": 2.0, "steps": n_all, "stage_us": dict(zip(names, [round(x, 2) for x in us2])),
                              "score_GBps": r2["score"]["achieved"], "score_frac": r2["score"]["achieved"] / HBM_PEAK_GBS,
                              "attn_GBps": r2["attn"]["achieved"], "attn_frac": r2["attn"]["achieved"] / HBM_PEAK_GBS,
                              "rows_filled_per_step": dd2["slot_misses"] / n_all}
        if w.host_k or w.host_v:
            # the miss fill as a kernel of its own (not folded into the attention loads), so that the PCIe
            # rate of the GPU-issued row fetches can be read off its duration
            peak = h2d_peak_gbs(torch)
            per_row = 256 * (int(w.host_k) + int(w.host_v))
            for tag, tau_f, nw, ns in (("fill", tau, W_steps, K_steps), ("fill_all_miss", 2.0, 2, n_all)):
                _, uf, df = profile(tau_f, nw, ns, extra=Q.QSAC_FLAG_FILL_KERNEL)
                by = per_row * df["slot_misses"] / ns
                gbs = by / (uf[3] * 1e-6) / 1e9 if by else 0.0
                result[tag] = {"bound": "pcie", "kernel": "qsac_fill_kernel", "bytes_per_launch": by,
                               "us_per_launch": uf[3], "achieved": gbs, "peak": peak, "unit": "GB/s",
                               "frac": gbs / peak, "peak_kind": "measured hipMemcpyAsync pinned H2D, 1 GiB"}

    # ---- read-only launches of the sizes of the two HBM-bound kernels (a yardstick, not part of the step)
    if a.calibration_reads:
        pool = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        result["read_only_launch"] = {}
        for name, nbytes in (("attn", 512 * w.k * w.P), ("score_all_miss", 256 * w.N * w.P)):
            nbytes = min(nbytes, 512 << 20) // 16 * 16
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            us = []
            for r in range(a.calibration_reads + 2):
                off = (r * nbytes) % ((1 << 30) - nbytes + 256) // 256 * 256     # rotate: nothing stays in a cache
                ev[0].record()
                Q.qsac_calibration_read(pool.data_ptr() + off, nbytes, sink.data_ptr())   # on the null stream, as the events
                ev[1].record()
                ev[1].synchronize()
                if r >= 2:
                    us.append(1e3 * ev[0].elapsed_time(ev[1]))
            result["read_only_launch"][name] = {"bytes": nbytes, "us_by_events": sum(us) / len(us),
                                                "GBps_by_events": nbytes / (sum(us) / len(us) * 1e-6) / 1e9}
        del pool

    # ---- the oracle on the host cores of this machine, a bounded sample of the same workload
    if not a.no_cpu_baseline:
        import oracle
        Kb, Vb = W.bits(K_host), W.bits(V_host)
        qb = W.bits(q_dev.cpu())
        st = oracle.State.empty(w.B, w.Hq, w.Hkv, w.D, w.k)
        code = W.DTYPE_CODES[w.dtype]
        t0 = time.perf_counter()
        oracle.step(st, qb[0], Kb, Kb, Vb, tau, w.k, code)      # first step: every pair misses
        first = time.perf_counter() - t0
        n_cpu = a.cpu_steps or max(2, min(K_steps + W_steps - 1, int(15.0 / max(first * 0.5, 1e-3))))
        t0 = time.perf_counter()
        for t in range(1, 1 + n_cpu):
            oracle.step(st, qb[t], Kb, Kb, Vb, tau, w.k, code)
        cpu_t = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n_cpu / cpu_t, "unit": "steps/s", "cores": oracle.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"steps 2..{n_cpu + 1} of the same query chain on the full batch "
                                            f"({w.P} pairs, OpenMP over pairs), after an untimed all-miss first step "
                                            f"({first:.2f} s)"}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
