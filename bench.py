#!/usr/bin/env python3
"""Benchmark of the QSAC decode step on one MI355X.

A step is one qsac_step() over the whole batch of one attention layer (gate, scoring of the
missing heads, top-k select, slot diff, miss fill, sparse attention).  Inputs are synthetic
(see paper_2511_14510_amd/workload.py) and resident in HBM (and, for the offload workloads,
in pinned host memory) before the timed region starts.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]          all five workloads; headline = the largest
  python bench.py --workload NAME [--tau T] [--flags F] ...    one workload in detail (what the profiles run)

With no --workload every workload of the benchmark is timed in one run: the headline fields (value,
ms_per_step, config, roofline, cpu_baseline) are those of the largest one, low_sim_stress, whose step is bound
by the PCIe fetch of the missing rows; the other four are summarised under "workloads".
"""
import argparse
import ctypes
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
HEADLINE = "low_sim_stress"
ORDER = ("tiny", "llama3_8b_32k", "qwen25_14b_128k_offload", "long_1m", "low_sim_stress")
STAGES = ("gate", "score", "select", "fill", "attn", "combine")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default=None, help="time only this workload, in detail")
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
    ap.add_argument("--no-profile", action="store_true", help="skip the stage-timing passes and the extra legs")
    ap.add_argument("--k-fill-from-hbm", action="store_true",
                    help="not the workload as specified: take the missing K rows from the HBM copy of K that scoring "
                         "reads (K_src = K_dev), so that only V rows cross PCIe")
    ap.add_argument("--calibration-reads", type=int, default=0,
                    help="after the run, launch this many read-only kernels (qsac_calibration_read) of the attention "
                         "launch's and of the all-miss scoring launch's size: what a launch of that size can reach")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="launch this many plain 256 MiB copies first (qsac_copy_kernel), to scale profiler counters")
    ap.add_argument("--cpu-seconds", type=float, default=0.0, help="oracle time budget (0 = 15 s headline, 4 s others)")
    return ap.parse_args()


def r4(x):
    """Four significant digits: keeps the line short."""
    if x is None:
        return None
    return float(f"{x:.4g}")


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


# ---- recorded profiler figures (bench.py cannot collect counters itself): read from the tracked summaries

def recorded_counter(workload, kernel_substr):
    """HBM bytes per launch of a kernel from the tracked rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries of this
    script on `workload` (a workload name, or name + "_all_miss" for the run with tau = 2), scaled by what the
    same counters read for the 256-MiB qsac_copy_kernel of the same runs.  Returns (bytes or None, source files)."""
    total, files = 0.0, []
    for counter in ("fetch_size", "write_size"):
        path = os.path.join(ROOT, "profiles", f"qsac_step_kernels__{workload}__pmc_{counter}.txt")
        if not os.path.exists(path):
            return None, []
        rows = {}
        for line in open(path):
            f = line.split()
            if len(f) >= 6 and f[1] in ("FETCH_SIZE", "WRITE_SIZE"):
                rows[f[0]] = float(f[3])
        copy = [v for name, v in rows.items() if "qsac_copy_kernel" in name]
        kern = [v for name, v in rows.items() if kernel_substr in name]
        if not copy or not kern:
            return None, []
        unit = (256 << 20) / copy[0]                 # bytes per counter unit
        total += kern[0] * unit
        files.append(os.path.relpath(path, ROOT))
    return total, files


def recorded_trace_us(workload, kernel_substr):
    """Average duration of a kernel in the tracked rocprofv3 --kernel-trace summary of this script on `workload`."""
    path = os.path.join(ROOT, "profiles", f"qsac_step_kernels__{workload}__kernel_trace.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        f = line.split()
        if len(f) >= 6 and kernel_substr in f[0] and re.fullmatch(r"\d+", f[1]):
            return float(f[2]), os.path.relpath(path, ROOT)
    return None, None


class Bench:
    def __init__(self, a):
        import torch
        from paper_2511_14510_amd import binding as Q
        from paper_2511_14510_amd import workload as W
        assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU path)"
        Q.load()
        self.a, self.torch, self.Q, self.W = a, torch, Q, W
        self._h2d = None

    def h2d(self):
        if self._h2d is None:
            self._h2d = h2d_peak_gbs(self.torch)
            self.torch.cuda.empty_cache()
        return self._h2d

    # ------------------------------------------------------------------ one workload
    def run(self, name, K_steps, W_steps, detail, cpu_seconds):
        """Times one workload.  detail: 'headline' | 'single' (every leg) or 'brief' (what the summary needs)."""
        a, torch, Q, W = self.a, self.torch, self.Q, self.W
        w = W.CONFIGS[name]
        if a.k_fill_from_hbm:
            import dataclasses
            w = dataclasses.replace(w, host_k=False)
        tau = w.tau if (a.tau is None or detail == "brief") else a.tau
        total = K_steps + W_steps
        single = detail == "single"
        want_cpu = cpu_seconds > 0

        # ---- inputs, resident before any timing
        K_dev, V_dev = W.make_kv(w.B, w.Hkv, w.N, w.D, w.dtype, w.seed, device="cuda:0")
        K_host = V_host = None
        if w.host_k or want_cpu:
            K_host = torch.empty(K_dev.shape, dtype=K_dev.dtype, pin_memory=w.host_k).copy_(K_dev)
        if w.host_v or want_cpu:
            V_host = torch.empty(V_dev.shape, dtype=V_dev.dtype, pin_memory=w.host_v).copy_(V_dev)
        for t in (K_host, V_host):
            if t is not None and t.is_pinned():
                # The store was filled by a device copy: the host's own page-table entries for it do not exist yet, and
                # the first host access to each page would fault them in (tens of microseconds per 64 KiB here).  A
                # host KV store written by the host has them; touch every page once so the push-mode transfer
                # threads, which read it from the host, are not timed on page faults.
                t.view(-1)[::2048].float().sum().item()
        K_src = K_host if w.host_k else K_dev
        V_src = V_host if w.host_v else V_dev
        chain = W.chain_for(w)
        q_all = torch.stack([W.round_to(chain.next(), w.dtype) for _ in range(total)])
        V_res = res_slot = None
        hard, D = [], []
        if single and a.resident:
            # reuse difficulty D_i = tau_i - (s_hat_i - eps) from the adjacent-query cosines of the chain itself
            # (the paper profiles s_hat offline on sample sequences); the hardest heads become resident
            qf = q_all.double()
            cos = (qf[1:] * qf[:-1]).sum(-1) / (qf[1:].norm(dim=-1) * qf[:-1].norm(dim=-1))     # [T-1,B,Hq]
            cos = cos.reshape(total - 1, w.B, w.Hkv, w.G).clamp_min(1e-6)
            s_hat = (w.G / (1.0 / cos).sum(-1)).mean(dim=(0, 1))                                 # Eq. (2), then mean
            D = Q.qsac_reuse_difficulty([tau] * w.Hkv, s_hat.tolist(), 0.1)
            hard = sorted(sorted(range(w.Hkv), key=lambda h: -D[h])[:a.resident])
            res_slot = [-1] * w.Hkv
            for i, h in enumerate(hard):
                res_slot[h] = i
            V_res = torch.stack([V_dev[:, h] for h in hard], dim=1).contiguous()
        if w.host_v:
            V_dev = None  # the offload workloads keep V on the host only (and in V_res for resident heads)
        q_dev = q_all.cuda()
        K_app = V_app = None
        n_sink = n_recent = 0
        if single and a.decode_buffers:
            # the generated tokens' KV are synthetic too and resident beforehand; a step only raises the valid count
            n_sink, n_recent = 4, 64
            K_app, V_app = W.make_kv(w.B, w.Hkv, total, w.D, w.dtype, w.seed + 7, device="cuda:0")
        torch.cuda.synchronize()
        user_flags = a.flags if single else 0

        def session(flags, side=False):
            return Q.Session(w.B, w.Hq, w.Hkv, w.N, w.k, w.dtype, K_dev, K_src, V_src, flags=flags | user_flags,
                             side_stream=side or (single and a.side_stream), V_res=V_res, res_slot=res_slot,
                             n_sink=n_sink, n_recent=n_recent, K_app=K_app, V_app=V_app)

        def run_steps(sess, tau_r, lo, hi):
            for t in range(lo, hi):
                if sess.K_app is not None:
                    sess.set_appended(t + 1)   # the token generated at step t has joined the append-only buffer
                sess.step(q_dev[t], tau_r, w.k)

        def timed(flags=0, side=False, tau_r=None):
            """(seconds for K steps after W warm-up steps, counter deltas over the K steps)."""
            tau_r = tau if tau_r is None else tau_r
            sess = session(flags, side)
            run_steps(sess, tau_r, 0, W_steps)
            sess.sync()
            torch.cuda.synchronize()
            s0 = sess.stats()
            t0 = time.perf_counter()
            run_steps(sess, tau_r, W_steps, total)
            sess.sync()
            torch.cuda.synchronize()
            el = time.perf_counter() - t0
            s1 = sess.stats()
            sess.close()
            return el, {key: s1[key] - s0[key] for key in s1}

        # ---- the timed run: K steps after W warm-up steps, no events inside
        elapsed, d = timed()
        pairs = w.P * K_steps
        fresh_rows = d["slot_hits"] + d["slot_misses"]
        res = {
            "steps_per_s": K_steps / elapsed, "ms_per_step": 1e3 * elapsed / K_steps,
            "reuse_rate": d["reuse_heads"] / pairs,
            "slot_hit_rate": d["slot_hits"] / fresh_rows if fresh_rows else None,
            "guided_select_rate": d["guided_selects"] / d["miss_heads"] if d["miss_heads"] else None,
            "rows_filled_per_step": d["slot_misses"] / K_steps,
            "host_bytes_per_step": d["bytes_filled_host"] / K_steps,
        }
        res["_w"], res["_tau"] = w, tau
        if not single and (w.host_k or w.host_v) and w.B >= 2 and (detail == "headline" or name == "qwen25_14b_128k_offload"):
            # the same steps under the staggered schedule: batch slices pipelined over two streams, a slice is scored
            # (HBM) while the rows of the slice before it are fetched (PCIe)
            t_st, d_st = timed(Q.QSAC_FLAG_STAGGER, side=True)
            res["staggered"] = {"steps_per_s": K_steps / t_st, "ms_per_step": 1e3 * t_st / K_steps,
                                "plain_ms_per_step": res["ms_per_step"], "slices": stagger_slices(w.B),
                                "host_GBps_over_the_step": d_st["bytes_filled_host"] / t_st / 1e9}
        if single:
            res["_cfg_extra"] = {}
            if a.decode_buffers:
                res["_cfg_extra"].update({"n_sink": n_sink, "n_recent": n_recent, "append_rows_at_end": total})
            if a.resident:
                res["_cfg_extra"].update({"resident_kv_heads": hard, "reuse_difficulty": [round(x, 4) for x in D]})

        # ---- stage timing (HIP events on the stream the kernels run on), same steps
        if not a.no_profile:
            def profile(tau_p, n_warm, n_steps, extra=0):
                ps = session(Q.QSAC_FLAG_PROFILE | extra)
                run_steps(ps, tau_p, 0, n_warm)
                ps.sync()
                _, ms0, c0 = Q.qsac_get_stage_ms(ps.ctx)
                st0 = ps.stats()
                run_steps(ps, tau_p, n_warm, n_warm + n_steps)
                ps.sync()
                names, ms1, c1 = Q.qsac_get_stage_ms(ps.ctx)
                st1 = ps.stats()
                ps.close()
                assert c1 - c0 == n_steps and tuple(names) == STAGES
                us = dict(zip(names, [1e3 * (y - x) / n_steps for x, y in zip(ms0, ms1)]))
                return us, {key: (st1[key] - st0[key]) / n_steps for key in st1}

            def hbm(us, dd):
                """Algorithmic bytes per launch over the event-timed duration of the two HBM-bound kernels."""
                score_bytes = 256.0 * w.N * dd["miss_heads"]       # K bytes one scoring launch has to read
                attn_bytes = 512.0 * w.k * w.P                      # slot bytes one attention launch has to read
                return {"score_us": us["score"], "score_bytes": score_bytes,
                        "score_GBps": score_bytes / us["score"] / 1e3 if score_bytes else None,
                        "attn_us": us["attn"], "attn_bytes": attn_bytes, "attn_GBps": attn_bytes / us["attn"] / 1e3,
                        "missing_pairs": dd["miss_heads"]}

            us, dd = profile(tau, W_steps, K_steps)
            res["stage_us"] = us
            res["hbm"] = hbm(us, dd)
            n_all = min(K_steps, 16)
            us2, dd2 = profile(2.0, 2, n_all)          # every pair misses every step: each launch reads all of K
            res["all_miss"] = {"stage_us": us2, **hbm(us2, dd2), "rows_filled": dd2["slot_misses"]}
            if w.host_k or w.host_v:
                peak = self.h2d()
                # fill on read (the default): the host bytes a step fetches over the attention kernel's duration
                res["pcie"] = {"peak_GBps": peak, "peak_kind": "hipMemcpyAsync pinned H2D of 1 GiB, measured in this run",
                               "fill_on_read_GBps": dd["bytes_filled_host"] / us["attn"] / 1e3,
                               "fill_on_read_all_miss_GBps": dd2["bytes_filled_host"] / us2["attn"] / 1e3}
                if detail != "brief" or name == "qwen25_14b_128k_offload":
                    # the fill as a kernel of its own, so that the rate of the GPU-issued row fetches alone shows
                    uf, df = profile(tau, W_steps, K_steps, extra=Q.QSAC_FLAG_FILL_KERNEL)
                    res["pcie"]["fill_kernel_GBps"] = df["bytes_filled_host"] / uf["fill"] / 1e3
                    res["pcie"]["fill_kernel_us"] = uf["fill"]
                    # overlap efficiency of the side stream: (serial - overlapped) / fill time
                    t_ser, _ = timed(Q.QSAC_FLAG_FILL_KERNEL, side=False)
                    t_ovl, _ = timed(Q.QSAC_FLAG_FILL_KERNEL, side=True)
                    res["overlap"] = {"serial_us": 1e6 * t_ser / K_steps, "side_stream_us": 1e6 * t_ovl / K_steps,
                                      "fill_us": uf["fill"],
                                      "efficiency": (t_ser - t_ovl) / K_steps * 1e6 / uf["fill"] if uf["fill"] else None}
                    if w.host_k and w.host_v and not (single and a.resident):
                        # the paper's push mode as the A/B: host threads write the rows into the slots, the GPU polls
                        t_push, dpush = timed(Q.QSAC_FLAG_PUSH_FILL)
                        up, dp_ = profile(tau, W_steps, K_steps, extra=Q.QSAC_FLAG_PUSH_FILL)
                        res["push"] = {"steps_per_s": K_steps / t_push, "us_per_step": 1e6 * t_push / K_steps,
                                       "transfer_us": up["fill"], "GBps": dp_["bytes_filled_host"] / up["fill"] / 1e3,
                                       "frac": dp_["bytes_filled_host"] / up["fill"] / 1e3 / peak,
                                       "pull_us_per_step": res["ms_per_step"] * 1e3, "threads": 4}
            if (detail != "brief" or name in ("tiny", "llama3_8b_32k")) and not (single and (a.decode_buffers or a.resident)):
                res["graph"] = self.graph_leg(session, q_dev, tau, w, K_steps, W_steps)

        # ---- read-only launches of the sizes of the two HBM-bound kernels (a yardstick, not part of the step)
        if single and a.calibration_reads:
            pool = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
            sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
            res["read_only_launch"] = {}
            for tag, nbytes in (("attn", 512 * w.k * w.P), ("score_all_miss", 256 * w.N * w.P)):
                nbytes = min(nbytes, 512 << 20) // 16 * 16
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                us_l = []
                for r in range(a.calibration_reads + 2):
                    off = (r * nbytes) % ((1 << 30) - nbytes + 256) // 256 * 256     # rotate: nothing stays in a cache
                    ev[0].record()
                    Q.qsac_calibration_read(pool.data_ptr() + off, nbytes, sink.data_ptr())   # null stream, as the events
                    ev[1].record()
                    ev[1].synchronize()
                    if r >= 2:
                        us_l.append(1e3 * ev[0].elapsed_time(ev[1]))
                res["read_only_launch"][tag] = {"bytes": nbytes, "us_by_events": sum(us_l) / len(us_l),
                                                "GBps_by_events": nbytes / (sum(us_l) / len(us_l) * 1e-6) / 1e9}
            del pool

        # ---- the oracle on the host cores of this machine, a bounded sample of the same workload
        if want_cpu:
            res["cpu_baseline"] = self.cpu_leg(w, tau, K_host, V_host, q_all, cpu_seconds)
        del K_dev, V_dev, K_host, V_host, K_src, V_src, q_dev, V_res, K_app, V_app
        torch.cuda.empty_cache()
        return res

    # ------------------------------------------------------------------ eager launches against graph replay
    def graph_leg(self, session, q_dev, tau, w, K_steps, W_steps):
        """The same steps launched kernel by kernel and replayed from one captured graph (Section 2.3 of the
        paper: launch overhead of short steps).  Both sides copy the step's query into the fixed buffer the
        graph is bound to, so the difference is the launch mechanism alone."""
        torch, Q = self.torch, self.Q
        total = K_steps + W_steps
        out = {}
        for mode in ("eager", "replay"):
            sess = session(0)
            q_buf = torch.zeros_like(q_dev[0])
            table = sess.dev_params_table([tau] * 1, [0])
            dp = table[0].clone()
            torch.cuda.synchronize()
            graph = Q.qsac_graph_capture(sess.ctx, sess.step_args(q_buf, None, w.k, dev_params=dp)) if mode == "replay" else None
            args = sess.step_args(q_buf, tau, w.k)

            def go(lo, hi):
                for t in range(lo, hi):
                    sess.copy_on_main(q_buf, q_dev[t])
                    if graph is not None:
                        Q.qsac_graph_launch(graph)
                    else:
                        Q.qsac_step(sess.ctx, args)
            go(0, W_steps)
            sess.sync()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            go(W_steps, total)
            sess.sync()
            torch.cuda.synchronize()
            out[mode + "_us"] = 1e6 * (time.perf_counter() - t0) / K_steps
            if graph is not None:
                Q.qsac_graph_free(graph)
            sess.close()
        return out

    # ------------------------------------------------------------------ the oracle, timed
    def cpu_leg(self, w, tau, K_host, V_host, q_all, seconds):
        import numpy as np
        import oracle
        W = self.W
        cores = oracle.num_threads()
        Kb, Vb = W.bits(K_host), W.bits(V_host)
        qb = W.bits(q_all)
        code = W.DTYPE_CODES[w.dtype]
        n_steps_max = len(qb) - 1

        def sample_mask(n_pairs):
            mask = np.zeros(w.P, np.uint8)
            mask[np.linspace(0, w.P - 1, n_pairs).round().astype(int)] = 1     # spread over batch and heads
            return mask

        def first_step(mask):
            st = oracle.State.empty(w.B, w.Hq, w.Hkv, w.D, w.k)
            t0 = time.perf_counter()
            oracle.step(st, qb[0], Kb, Kb, Vb, tau, w.k, code, pair_mask=mask)      # first step: every pair misses
            return st, time.perf_counter() - t0

        # one pair per thread first (pairs are independent); if the query chain at hand would not fill the time
        # budget with that many pairs, the sample grows in whole rounds of `cores` pairs
        mask = sample_mask(min(w.P, cores))
        st, first = first_step(mask)
        rounds = int(seconds / max(first * 0.6 * n_steps_max, 1e-3))
        if rounds >= 2 and w.P > cores:
            mask = sample_mask(min(w.P, cores * rounds))
            st, first = first_step(mask)
        n_pairs = int(mask.sum())
        n_cpu = max(2, min(n_steps_max, int(seconds / max(first * 0.6, 1e-3))))
        t0 = time.perf_counter()
        for t in range(1, 1 + n_cpu):
            oracle.step(st, qb[t], Kb, Kb, Vb, tau, w.k, code, pair_mask=mask)
        cpu_t = time.perf_counter() - t0
        scale = n_pairs / w.P                            # linear in the number of pairs
        return {"value": n_cpu / cpu_t * scale, "unit": "steps/s", "cores": cores, "kind": "oracle",
                "sample": f"steps 2..{n_cpu + 1} of the same query chain on {n_pairs} of the {w.P} pairs (OpenMP over "
                          f"pairs, rate scaled by {n_pairs}/{w.P}), after an untimed all-miss first step ({first:.2f} s)"}


def stagger_slices(B):
    """Batch elements per slice of the library's staggered schedule (enqueue_step in csrc/qsac.hip): B / 12 first,
    then each twice the one before; a small rest joins the last slice."""
    sizes, at, size = [], 0, max(B // 12, 1)
    while at < B:
        nxt = B if (len(sizes) + 1 == 8 or B - at - size < size // 2) else at + size
        sizes.append(nxt - at)
        at, size = nxt, size * 2
    return sizes


def config_of(res, Q, a):
    w, tau = res["_w"], res["_tau"]
    cfg = {"workload": w.name, "batch": w.B, "n_q_heads": w.Hq, "n_kv_heads": w.Hkv, "head_dim": w.D,
           "n_ctx": w.N, "k": w.k, "tau": tau,
           "rho": ("one per KV head, quantiles of U[%g, %g]" % w.rho_range) if w.rho_range else w.rho,
           "K_fill_source": "pinned host" if w.host_k else "HBM", "V_fill_source": "pinned host" if w.host_v else "HBM",
           "fill": "folded into attention loads"}
    if a.workload:
        cfg["scoring"] = "alu" if (a.flags & Q.QSAC_FLAG_SCORE_VALU) else "mfma"
        if a.flags & Q.QSAC_FLAG_FILL_KERNEL:
            cfg["fill"] = "own kernel"
        if a.side_stream:
            cfg["side_stream"] = ("staggered batch slices" if (a.flags & Q.QSAC_FLAG_STAGGER) else
                                  "fill kernel" if (a.flags & Q.QSAC_FLAG_FILL_KERNEL) else "attention of reused heads")
        cfg.update(res.get("_cfg_extra", {}))
    return cfg


def rooflines(res):
    """The roofline objects of a workload: the dominant kernel's, and the HBM-bound scoring kernel's beside it."""
    w = res["_w"]
    h = res["hbm"]
    out = {}
    traffic, files = recorded_counter(w.name + "_all_miss", "qsac_score")
    trace_us, trace_file = recorded_trace_us(w.name + "_all_miss", "qsac_score")
    score = {"bound": "hbm", "kernel": "qsac_score_mfma_kernel", "achieved": r4(h["score_GBps"]), "peak": HBM_PEAK_GBS,
             "unit": "GB/s", "frac": r4(h["score_GBps"] / HBM_PEAK_GBS) if h["score_GBps"] else None,
             "bytes_per_launch": r4(h["score_bytes"]), "us_per_launch": r4(h["score_us"]), "timed_by": "HIP events",
             "missing_pairs_per_launch": r4(h["missing_pairs"]),
             "all_miss_frac": r4(res["all_miss"]["score_GBps"] / HBM_PEAK_GBS),
             # recorded with rocprofv3 on the same command, not measured in this run
             "traffic": None, "traffic_source": None, "frac_by_recorded_trace": None, "trace_source": trace_file}
    if traffic is not None:
        # the summaries hold an all-miss run (P missing pairs per launch): scale to this run's missing pairs
        score["traffic"] = r4(traffic * h["missing_pairs"] / w.P)
        score["traffic_source"] = files
    if trace_us:
        score["frac_by_recorded_trace"] = r4(256.0 * w.N * w.P / trace_us / 1e3 / HBM_PEAK_GBS)
    attn = {"bound": "hbm", "kernel": "qsac_attn_kernel", "achieved": r4(h["attn_GBps"]), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": r4(h["attn_GBps"] / HBM_PEAK_GBS), "bytes_per_launch": r4(h["attn_bytes"]),
            "us_per_launch": r4(h["attn_us"]), "timed_by": "HIP events",
            # the kernel also carries the miss fill: every fetched row is written into its slot (512 B per row)
            "fill_bytes_written_per_launch": r4(512.0 * res["rows_filled_per_step"]),
            "frac_counting_fill_writes": r4((h["attn_bytes"] + 512.0 * res["rows_filled_per_step"]) / h["attn_us"] / 1e3
                                            / HBM_PEAK_GBS)}
    out["score"], out["attn"] = score, attn
    if "pcie" in res:
        p = res["pcie"]
        out["pcie"] = {"bound": "pcie", "kernel": "qsac_attn_kernel (missing rows fetched from pinned host memory on read)",
                       "achieved": r4(p["fill_on_read_GBps"]), "peak": r4(p["peak_GBps"]), "unit": "GB/s",
                       "frac": r4(p["fill_on_read_GBps"] / p["peak_GBps"]),
                       "bytes_per_launch": r4(res["host_bytes_per_step"]), "us_per_launch": r4(h["attn_us"]),
                       "timed_by": "HIP events", "peak_kind": p["peak_kind"],
                       "all_miss_frac": r4(p["fill_on_read_all_miss_GBps"] / p["peak_GBps"])}
        # HBM bytes of the same kernel as recorded with rocprofv3 on this workload at its own threshold
        traffic, files = recorded_counter(w.name, "qsac_attn")
        out["pcie"]["traffic"] = r4(traffic) if traffic is not None else None
        out["pcie"]["traffic_source"] = files or None
        if "fill_kernel_GBps" in p:
            out["pcie"]["fill_kernel_frac"] = r4(p["fill_kernel_GBps"] / p["peak_GBps"])
    return out


def brief(res):
    """The summary of a workload that is not the headline."""
    o = {"steps_per_s": r4(res["steps_per_s"]), "ms_per_step": r4(res["ms_per_step"]), "reuse_rate": r4(res["reuse_rate"]),
         "tau": res["_tau"]}
    if "hbm" in res:
        h, am = res["hbm"], res["all_miss"]
        o["score_hbm_frac"] = r4(h["score_GBps"] / HBM_PEAK_GBS) if h["score_GBps"] else None
        o["score_hbm_frac_all_miss"] = r4(am["score_GBps"] / HBM_PEAK_GBS)
        o["attn_hbm_frac"] = r4(h["attn_GBps"] / HBM_PEAK_GBS)
        o["stage_us"] = {s: r4(res["stage_us"][s]) for s in STAGES}
    if "pcie" in res:
        p = res["pcie"]
        o["fill"] = {"GBps": r4(p["fill_on_read_GBps"]), "h2d_GBps": r4(p["peak_GBps"]),
                     "frac": r4(p["fill_on_read_GBps"] / p["peak_GBps"]),
                     "all_miss_frac": r4(p["fill_on_read_all_miss_GBps"] / p["peak_GBps"])}
        if "fill_kernel_GBps" in p:
            o["fill"]["fill_kernel_frac"] = r4(p["fill_kernel_GBps"] / p["peak_GBps"])
    if "overlap" in res:
        o["overlap"] = {k: r4(v) for k, v in res["overlap"].items()}
    if "push" in res:
        o["push"] = {k: r4(v) for k, v in res["push"].items()}
    if "graph" in res:
        o["graph"] = {k: r4(v) for k, v in res["graph"].items()}
    if "staggered" in res:
        o["staggered"] = {k: (v if k == "slices" else r4(v)) for k, v in res["staggered"].items()}
    if "cpu_baseline" in res:
        c = res["cpu_baseline"]
        o["oracle"] = {"steps_per_s": r4(c["value"]), "cores": c["cores"]}
    return o


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the QSAC step has no inter-GPU part); use --gpus 1",
              file=sys.stderr)
        return 2
    B = Bench(a)
    Q, torch = B.Q, B.torch
    K_steps, W_steps = a.steps, a.warmup

    if a.calibration_copies:
        n = 256 << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(a.calibration_copies):
            Q.qsac_calibration_copy(dst.data_ptr(), src.data_ptr(), n)
        torch.cuda.synchronize()
        del src, dst

    names = [a.workload] if a.workload else list(ORDER)
    head_name = a.workload or HEADLINE
    results = {}
    for name in names:
        is_head = name == head_name
        detail = "single" if a.workload else ("headline" if is_head else "brief")
        cpu_s = 0.0 if a.no_cpu_baseline else (a.cpu_seconds or (15.0 if is_head else 4.0))
        t0 = time.perf_counter()
        results[name] = B.run(name, K_steps, W_steps, detail, cpu_s)
        print(f"bench.py: {name} done in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)

    head = results[head_name]
    w = head["_w"]
    line = {
        "metric": "QSAC decode steps/s per layer", "value": head["steps_per_s"], "unit": "steps/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W_steps, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": config_of(head, Q, a),
        "reuse_rate": r4(head["reuse_rate"]), "slot_hit_rate": r4(head["slot_hit_rate"]),
        "guided_select_rate": r4(head["guided_select_rate"]),
        "rows_filled_per_step": r4(head["rows_filled_per_step"]), "host_bytes_per_step": r4(head["host_bytes_per_step"]),
    }
    line["config"]["schedule"] = "plain: one stream, kernel after kernel"
    if a.workload and (a.flags & Q.QSAC_FLAG_STAGGER):
        line["config"]["schedule"] = "staggered (QSAC_FLAG_STAGGER)"
    if "staggered" in head:
        st = head["staggered"]
        line["schedules"] = {"plain": {"steps_per_s": r4(head["steps_per_s"]), "ms_per_step": r4(head["ms_per_step"])},
                             "staggered": {k: (v if k == "slices" else r4(v)) for k, v in st.items()}}
        if "stage_us" in head:
            # (serial - overlapped) / fill time, the fill time being the fetching attention kernel's on one stream
            line["schedules"]["staggered"]["overlap_efficiency"] = r4(
                (head["ms_per_step"] - st["ms_per_step"]) * 1e3 / head["stage_us"]["attn"])
        if st["steps_per_s"] > head["steps_per_s"]:
            # the headline is the faster of the two schedules; the stage times and rooflines below are taken kernel by
            # kernel on one stream (the plain schedule), where each kernel has the machine to itself
            line["value"], line["ms_per_step"] = st["steps_per_s"], st["ms_per_step"]
            line["config"]["schedule"] = ("staggered (QSAC_FLAG_STAGGER): batch slices of %s elements pipelined over two "
                                          "streams, a slice is scored while the rows of the slice before it are fetched"
                                          % "+".join(str(x) for x in st["slices"]))
    if "hbm" in head:
        rf = rooflines(head)
        # dominant kernel: the attention kernel fetching the missing rows over PCIe where the workload offloads,
        # the scoring pass otherwise
        line["roofline"] = rf["pcie"] if "pcie" in rf else rf["score"]
        if "pcie" in rf and "staggered" in head:
            # the figures above are the plain schedule's fetching kernel (event-timed on its stream); under the staggered
            # schedule the rows travel in qsac_fill_trickle_kernel launches beside the other kernels: host bytes over
            # the whole step's wall time is a lower bound of that kernel's own rate
            line["roofline"]["staggered_whole_step_GBps"] = r4(head["staggered"]["host_GBps_over_the_step"])
            line["roofline"]["staggered_whole_step_frac"] = r4(head["staggered"]["host_GBps_over_the_step"]
                                                               / head["pcie"]["peak_GBps"])
        line["score_roofline"], line["attn_roofline"] = rf["score"], rf["attn"]
        line["stage_us"] = {s: r4(head["stage_us"][s]) for s in STAGES}
        line["all_miss"] = {"stage_us": {s: r4(head["all_miss"]["stage_us"][s]) for s in STAGES},
                            "score_frac": r4(head["all_miss"]["score_GBps"] / HBM_PEAK_GBS),
                            "attn_frac": r4(head["all_miss"]["attn_GBps"] / HBM_PEAK_GBS)}
        for key in ("overlap", "push", "graph"):
            if key in head:
                line[key] = {k: r4(v) for k, v in head[key].items()}
    if "read_only_launch" in head:
        line["read_only_launch"] = head["read_only_launch"]
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
        line["cpu_baseline"]["value"] = r4(line["cpu_baseline"]["value"])
    if not a.workload:
        line["workloads"] = {n: brief(results[n]) for n in names if n != head_name}
    print(json.dumps(line, separators=(",", ":")))
    return 0


if __name__ == "__main__":
    sys.exit(main())
