#!/usr/bin/env python3
"""Benchmark of the LFPS decode-step hot path on one MI355X.

A "step" is one pass of the whole hot path for one attention layer over one batch of synthetic
input: candidates -> gather-score -> per-head Top-k -> sparse attention (one lfps_step call),
with the KV cache already resident in HBM.  Prints ONE JSON line:

  value        decode steps/s per layer of the named workload (whole job, this GPU)
  roofline     the dominant kernel (the scoring pass): algorithmic bytes per launch / its average launch
               duration from HIP events recorded around every launch on the launch stream
  cpu_baseline the CPU oracle (fp64 numpy, one thread) on a bounded sample of the same workload

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--all-workloads]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak

def measured_traffic(key, kernel="filter_score"):
    """HBM bytes per launch of a kernel as rocprofv3 counted them (--pmc FETCH_SIZE, then WRITE_SIZE, each scaled by
    the same counter's reading for a plain copy kernel of known size): profiles/traffic.json, written together with
    the summaries under profiles/ from the same runs.  None when that workload / kernel was not profiled."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            rec = json.load(f).get(key, {}).get(kernel)
    except (OSError, ValueError):
        return None
    return None if rec is None else float(rec["fetch_bytes"]) + float(rec["write_bytes"])


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: the workload's decode steps minus warmup)")
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--preheat-seconds", type=float, default=2.0,
                    help="untimed steps of the main workload for this many seconds before its warm-up (0: none); "
                         "what was spent is reported as `preheat` in the line")
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--all-workloads", action="store_true", default=True,
                    help="also report the other four workloads in the same line (default)")
    ap.add_argument("--main-only", dest="all_workloads", action="store_false", help="only the main workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-table-mode", action="store_true", help="skip the score-table mode legs")
    ap.add_argument("--no-paged", action="store_true", help="skip the paged-cache leg")
    ap.add_argument("--no-fp8", action="store_true", help="skip the legs with other cache formats (FP8 keys / values, fp16)")
    ap.add_argument("--fp8-only", action="store_true", help="run only the FP8-keys leg of --workload")
    ap.add_argument("--paged-only", action="store_true", help="run only the paged-cache leg of --workload")
    ap.add_argument("--paged-block", type=int, default=16, help="rows per block of the paged-cache leg")
    ap.add_argument("--paged-layout", default="block_head_row", choices=["block_head_row", "block_row_head"],
                    help="memory order inside a block of the paged-cache leg")
    ap.add_argument("--table-only", action="store_true",
                    help="run only the score-table mode of the main workload (for profiling) and print its record")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run only the plain copy kernel (1 GiB, 10 launches): the known-traffic reference for rocprofv3 --pmc")
    ap.add_argument("--host-kv-only", action="store_true",
                    help="run only the host-resident-cache leg of --workload and print its record")
    ap.add_argument("--no-host-kv", action="store_true", help="skip the host-resident-cache leg")
    ap.add_argument("--peaky-only", action="store_true",
                    help="run only the concentrated-attention variant of C4 (memoryless and score-table steps) and print its record")
    ap.add_argument("--sweep", action="store_true",
                    help="run only a grid of batch sizes and context lengths with the C4 recipe and print its record")
    ap.add_argument("--sweep-batches", default="1,4,16,32", help="batch sizes of --sweep")
    ap.add_argument("--sweep-contexts", default="32768,131072,524288", help="context lengths of --sweep")
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="CPU-oracle sample budget (per leg: one core, all cores)")
    return ap.parse_args()


class Runner:
    """Device state of one workload and the step loop."""

    def __init__(self, name, table_mode=False, n_sink=0, gated=False, paged_block=0, paged_layout="block_head_row",
                 k_dtype="", v_dtype="", kv_dtype="", override=None):
        import numpy as np
        import torch

        import gen
        from gen import device as gen_device
        from paper_2506_15704_amd.binding import Lfps

        self.torch, self.np = torch, np
        self.spec = spec = gen.WORKLOADS.get(name) or gen.EXTRA_WORKLOADS[name]
        if override:         # the same recipe at another batch size / context length / budget (--sweep)
            import dataclasses
            self.spec = spec = dataclasses.replace(spec, **override)
        if k_dtype:          # the same workload with the keys stored in another format
            import dataclasses
            self.spec = spec = dataclasses.replace(spec, name=f"{name}-{k_dtype}k" + ("v" if v_dtype else ""),
                                                   k_dtype=k_dtype, v_dtype=v_dtype)
        if kv_dtype:         # the same workload with the whole cache in another 16-bit format
            import dataclasses
            self.spec = spec = dataclasses.replace(spec, name=f"{name}-{kv_dtype}", kv_dtype=kv_dtype)
        self.case = case = gen.make_case(spec)
        self.dev = "cuda:0"
        self.K, self.V = gen_device.fill_kv(case, self.dev)
        self.block_table = None
        if paged_block:      # the same rows as a block pool in shuffled order
            Kp, Vp, self.block_table = gen_device.paginate(self.K, self.V, paged_block, seed=spec.seed,
                                                           layout=paged_layout)
            self.K, self.V = Kp, Vp
        self.ctx = Lfps(batch=spec.B, n_q_heads=spec.Hq, n_kv_heads=spec.Hkv, head_dim=spec.D,
                        kv_dtype=spec.kv_dtype, max_seq_len=case.Lcap, max_k=case.kmax, radius=spec.r,
                        n_recent=1, n_sink=n_sink, table_mode=table_mode, table_decay=0.95, table_a=0.2,
                        k_fp8=spec.k_dtype == "fp8", v_fp8=spec.v_dtype == "fp8")
        self.table_mode = table_mode
        self.gated = gated
        if gated:        # prefill priors of the bypass (Sec. 4.2 "Prefilling"), from the step-0 query
            self.kbar = torch.zeros((spec.B, spec.Hkv, spec.D), dtype=torch.float32, device=self.dev)
            self.vbar = torch.zeros_like(self.kbar)
            self.sigma2 = torch.zeros((spec.B, spec.Hq), dtype=torch.float32, device=self.dev)
            self.gate = torch.zeros((spec.B, spec.Hq), dtype=torch.int32, device=self.dev)
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        self.q = to(case.q)                                                 # [T+1, B, Hq, D]
        self.seq = to(np.stack([case.seq_lens(t) for t in range(spec.T + 1)]))  # [T+1, B]
        self.k = to(case.k)
        if paged_block:
            self.views = [self.ctx.paged_kv_view(self.K, self.V, self.block_table, self.seq[t]) for t in range(spec.T + 1)]
        else:
            self.views = [self.ctx.kv_view(self.K, self.V, self.seq[t]) for t in range(spec.T + 1)]
        shp = (spec.B, spec.Hq, case.kmax)
        self.seed = torch.zeros(shp, dtype=torch.int32, device=self.dev)
        self.buf = [torch.zeros(shp, dtype=torch.int32, device=self.dev) for _ in range(2)]
        self.out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=self.dev)
        self.cand = torch.zeros((spec.B, spec.Hkv, self.ctx.cand_cap), dtype=torch.int32, device=self.dev)
        self.sel_score = torch.zeros(shp, dtype=torch.float32, device=self.dev)
        # step 0: exact Top-k seeds the history
        self.ctx.lfps_exact_topk(self.q[0], self.views[0], self.k, self.seed)
        torch.cuda.synchronize()
        self.reset()

    def reset(self):
        self.t = 0
        self.prev = self.seed
        self.cur = 0

    def _advance(self):
        self.t += 1
        if self.t > self.spec.T:       # more steps asked than the workload has: start over from the seed
            self.t = 1
            self.prev = self.seed
        return self.t

    def step(self):
        t = self._advance()
        dst = self.buf[self.cur]
        if self.table_mode:
            if t == 1:      # (re)start of the chain: Eq. 4 tables from the step-0 query
                self.ctx.lfps_tables_init(self.q[0], self.views[0])
            if self.gated:
                self.ctx.lfps_table_step_gated(self.q[t], self.views[t], self.k, self.kbar, self.vbar, self.sigma2, 6, 0.85,
                                               dst, self.out, None, self.gate)
            else:
                self.ctx.lfps_table_step(self.q[t], self.views[t], self.k, dst, self.out)
        else:
            self.ctx.lfps_step(self.q[t], self.views[t], self.prev, self.k, dst, self.out, self.sel_score)
        self.prev = dst
        self.cur ^= 1

    def sel_score_last(self):
        """Scores of the rows selected by the last lfps_step call (its topk_score output)."""
        return self.sel_score


    def run_timed(self, steps, warmup):
        torch = self.torch
        self.reset()
        self.ctx.lfps_reset_history()
        assert warmup >= 1 or not self.table_mode, "table mode: the first step builds the tables (keep it in the warm-up)"
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def run_step_percentiles(self, steps, warmup):
        """The same steps once more with an event pair around every lfps_step call on the stream the kernels
        run on: p10 / median / p90 of the per-step device time in microseconds."""
        torch, np = self.torch, self.np
        self.reset()
        self.ctx.lfps_reset_history()
        for _ in range(warmup):
            self.step()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for a, b in ev:
            a.record()
            self.step()
            b.record()
        torch.cuda.synchronize()
        us = np.array([a.elapsed_time(b) * 1e3 for a, b in ev])
        return {"p10": round(float(np.percentile(us, 10)), 2), "median": round(float(np.median(us)), 2),
                "p90": round(float(np.percentile(us, 90)), 2)}

    def union_rows_last_step(self):
        """Rows the sparse attention of the last step had to fetch if every KV group read each selected row
        once for all its heads: sum over (b, g) of |union over the group's heads of the selected positions|."""
        torch = self.torch
        spec = self.spec
        idx = self.prev
        total = 0
        for b in range(spec.B):
            kb = int(self.case.k[b])
            rows = idx[b, :, :kb].reshape(spec.Hkv, spec.G * kb)
            for g in range(spec.Hkv):
                u = torch.unique(rows[g])
                total += int((u >= 0).sum().item())
        return total

    def run_timed_graph(self, steps, warmup):
        """The same K steps captured once into a HIP graph and replayed: removes the host launch gaps
        between the kernels of a step.  Returns (seconds per step, outputs equal to the eager run?)."""
        torch = self.torch

        def prepare():
            self.reset()
            self.ctx.lfps_reset_history()
            for _ in range(warmup):
                self.step()
            torch.cuda.synchronize()

        prepare()
        state = (self.t, self.prev, self.cur)
        for _ in range(steps):                       # eager reference of the final state
            self.step()
        torch.cuda.synchronize()
        ref_idx, ref_out = self.prev.clone(), self.out.clone()
        prepare()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(steps):
                self.step()
        self.t, self.prev, self.cur = state
        graph.replay()                               # untimed: first replay
        torch.cuda.synchronize()
        prepare()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        # the replay wrote into the same ping-pong buffers the eager run used
        final = self.buf[(state[2] + steps - 1) % 2] if steps else self.prev
        same = bool(torch.equal(final, ref_idx)) and bool(torch.equal(self.out, ref_out))
        return sec, same

    def run_kernel_timing(self, steps, warmup):
        """Second pass over the same steps (same lfps_step calls) with HIP events around every kernel
        launch; the candidate counts of each step are copied out after the step."""
        torch, spec = self.torch, self.spec
        self.reset()
        self.ctx.lfps_reset_history()
        cnts = torch.zeros((steps, spec.B, spec.Hkv), dtype=torch.int32, device=self.dev)
        for i in range(warmup):
            self.step()
        torch.cuda.synchronize()
        self.ctx.lfps_timing_enable(True)
        for i in range(steps):
            self.step()
            self.ctx.lfps_copy_cand_count(cnts[i])
        tm = self.ctx.lfps_timing_read()
        self.ctx.lfps_timing_enable(False)
        return tm, cnts.cpu().numpy()

    def time_baseline(self, which, reps):
        torch = self.torch
        t = min(self.spec.T, 2)
        idx = self.buf[0]
        fn = (lambda: self.ctx.lfps_full_attn_decode(self.q[t], self.views[t], self.out)) if which == "full" else \
             (lambda: (self.ctx.lfps_exact_topk(self.q[t], self.views[t], self.k, idx, self.sel_score),
                       self.ctx.lfps_sparse_attn(self.q[t], self.views[t], idx, self.sel_score, self.k, self.out)))
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    def recall_vs_exact(self, ex=None):
        """Eq. 2 overlap of the chained LFPS Top-k with the exact Top-k at the last step run."""
        torch = self.torch
        if ex is None:
            ex = torch.zeros_like(self.seed)
            self.ctx.lfps_exact_topk(self.q[self.t], self.views[self.t], self.k, ex)
        got = self.prev
        L = int(self.seq[self.t].max().item()) + 1
        hits = 0
        tot = 0
        for b in range(self.spec.B):
            kb = int(self.case.k[b])
            a = torch.zeros((self.spec.Hq, L), dtype=torch.bool, device=self.dev)
            a.scatter_(1, ex[b, :, :kb].long(), True)
            g = got[b, :, :kb]
            hits += int((a.gather(1, g.clamp_min(0).long()) & (g >= 0)).sum().item())
            tot += self.spec.Hq * kb
        return hits / tot

    def quality_per_step(self, n_steps):
        """The free-running chain from the seed, step by step: Eq. 2 overlap of its Top-k with the exact Top-k of
        the same query, and the largest absolute difference between its output rows and full attention's
        (both references computed by this library's baselines on the device: statistics, not parity)."""
        torch = self.torch
        self.reset()
        self.ctx.lfps_reset_history()
        ex = torch.zeros_like(self.seed)
        full = torch.zeros_like(self.out)
        rec, err, byp = [], [], []
        for _ in range(n_steps):
            self.step()
            t = self.t
            self.ctx.lfps_exact_topk(self.q[t], self.views[t], self.k, ex)
            self.ctx.lfps_full_attn_decode(self.q[t], self.views[t], full)
            rec.append(round(self.recall_vs_exact(ex), 4))
            err.append(round(float((self.out - full).abs().max().item()), 4))
            if self.gated:
                byp.append(round(float(self.gate.float().mean().item()), 4))
        res = {"steps": n_steps, "recall_vs_exact_topk": rec, "max_abs_err_vs_full_attn": err}
        if self.gated:
            res["bypassed_head_frac"] = byp      # (a bypassed head selects nothing: it counts as recall 0)
        return res

    def close(self):
        self.ctx.close()
        del self.K, self.V


def algorithmic_bytes_score(spec, case, cnts, filtered):
    """Bytes one scoring launch must move.  Per candidate row: its K row (R = D*e bytes) and its
    position (4).  Output: unfiltered, G scores per row (4G); filtered, at least the k selected
    (score, slot) pairs per head (8 k G per group).  Plus the G query rows per (b, g)."""
    e = 1 if spec.k_dtype == "fp8" else (4 if spec.kv_dtype == "f32" else 2)
    rows = cnts.sum(axis=(1, 2)).astype(float)
    per_group = spec.G * spec.D * 4
    if filtered:
        out = float(case.k.sum()) * spec.Hq * 8
        return rows * (spec.D * e + 4) + out + cnts.shape[1] * cnts.shape[2] * per_group
    return rows * (spec.D * e + 4 + 4 * spec.G) + cnts.shape[1] * cnts.shape[2] * per_group


def measure(name, steps, warmup, with_baselines=True, use_graph=True, override=None, with_quality=False,
            preheat_s=0.0):
    r = Runner(name, override=override)
    spec = r.spec
    if steps <= 0:
        steps = max(1, spec.T - warmup)
    # Untimed steps before the warm-up, by wall clock.  On some boxes the legs that run seconds into the process were
    # seen ~7 % faster than the first one, on others not at all; the cause is not established.  With this the first leg
    # is measured in the state the later ones are, and the line says how much was spent.
    preheat = {"seconds": 0.0, "steps": 0}
    if preheat_s > 0:
        r.reset()
        r.ctx.lfps_reset_history()
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < preheat_s:
            for _ in range(200):
                r.step()
            r.torch.cuda.synchronize()
            preheat["steps"] += 200
        preheat["seconds"] = round(time.perf_counter() - t0, 3)
    sec = r.run_timed(steps, warmup)
    recall = r.recall_vs_exact()
    sec_graph, graph_ok = r.run_timed_graph(steps, warmup) if use_graph else (None, None)
    tm, cnts = r.run_kernel_timing(steps, warmup)
    union_rows = r.union_rows_last_step()
    step_us = r.run_step_percentiles(steps, warmup)
    filtered = tm["filter_score"][1] > 0
    kname = "filter_score" if filtered else "gather_score"
    gs_ms, gs_n = tm[kname]
    bytes_per_launch = float(algorithmic_bytes_score(spec, r.case, cnts, filtered).mean())
    gs_avg_s = gs_ms / max(gs_n, 1) * 1e-3
    achieved = bytes_per_launch / gs_avg_s / 1e9
    res = {
        "steps_per_s": 1.0 / sec, "ms_per_step": sec * 1e3, "steps": steps, "preheat": preheat,
        "ms_per_step_hip_graph": round(sec_graph * 1e3, 4) if sec_graph else None, "hip_graph_matches_eager": graph_ok,
        "roofline": {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(spec.name, kname),
                     "bytes_per_launch": round(bytes_per_launch), "avg_launch_us": round(gs_avg_s * 1e6, 2),
                     "launches": gs_n, "timed_by": "HIP events around each launch, second pass over the same steps",
                     "note": "heads the filter leaves short are rescored inside filter_select_attend (kernel_us)"},
        "kernel_us": {k: round(v[0] / steps * 1e3, 2) for k, v in tm.items() if v[1]},   # per step
        "step_us": step_us,
        "cand_frac": round(float(cnts.mean() / (spec.L or r.case.seq_lens0.mean())), 4),
        "recall_vs_exact_topk": round(recall, 4),
    }
    # S4: V bytes if every head fetched its own rows (upper bound) and if a group fetched each row once (lower bound)
    row_bytes = spec.D * (2 if spec.kv_dtype == "bf16" else 4)
    # S4 alone: the stand-alone kernel (lfps_sparse_attn) on the last step's Top-k and scores, event-timed
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    scratch_out = torch.zeros_like(r.out)
    for i in range(3 + 20):
        if i == 3:
            e0.record()
        r.ctx.lfps_sparse_attn(r.q[r.t], r.views[r.t], r.prev, r.sel_score_last(), r.k, scratch_out)
    e1.record()
    torch.cuda.synchronize()
    at_us = e0.elapsed_time(e1) * 1e3 / 20
    upper = float(r.case.k.sum()) * spec.Hq * row_bytes
    lower = float(union_rows) * row_bytes
    res["sparse_attn"] = {"avg_launch_us": round(at_us, 2), "bytes_per_head_rows": round(upper), "bytes_group_union_last_step": round(lower),
                          "GB_per_s_at_union_bytes": round(lower / (at_us * 1e-6) / 1e9, 1) if at_us > 0 else None,
                          "GB_per_s_at_per_head_bytes": round(upper / (at_us * 1e-6) / 1e9, 1) if at_us > 0 else None}
    # The whole step against the HBM roofline: the bytes one step must move at least (per KV group with c candidates
    # and budget k per head, R bytes per row: S1 reads G k ids and writes c; S2 reads c rows and their ids and writes
    # the survivors' (score, position) pairs, at least k per head; S3 reads them and writes k (position, score) pairs
    # per head; S4 reads those and one V row per selected position of the group) over the median step time.
    e_k = 1 if spec.k_dtype == "fp8" else (4 if spec.kv_dtype == "f32" else 2)
    ksum = float(r.case.k.sum())
    rows_scored = float(cnts.sum(axis=(1, 2)).mean())
    s1 = ksum * spec.Hq * 4 + rows_scored * 4
    s2 = rows_scored * (spec.D * e_k + 4) + ksum * spec.Hq * 8 + spec.B * spec.Hq * spec.D * 4
    s3 = 2 * ksum * spec.Hq * 8
    s4 = ksum * spec.Hq * 8 + lower + spec.B * spec.Hq * spec.D * 4
    step_bytes = s1 + s2 + s3 + s4
    res["whole_step"] = {"bytes": round(step_bytes), "GB_per_s": round(step_bytes / (step_us["median"] * 1e-6) / 1e9, 1),
                         "frac_of_hbm_peak": round(step_bytes / (step_us["median"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                         "bytes_by_stage": {"S1": round(s1), "S2": round(s2), "S3": round(s3), "S4": round(s4)}}
    res["sparse_attn"]["frac_of_hbm_peak_at_union_bytes"] = round(lower / (at_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if at_us > 0 else None
    if with_quality:
        res["per_step"] = r.quality_per_step(spec.T)
    if with_baselines:
        reps = 5 if name in ("C4", "C5") or override else 20
        exact = r.time_baseline("exact", reps)
        full = r.time_baseline("full", reps)
        res.update({"exact_topk_ms": round(exact * 1e3, 4), "full_attn_ms": round(full * 1e3, 4),
                    "speedup_vs_exact_topk": round(exact / sec, 3), "speedup_vs_full_attn": round(full / sec, 3)})
        # what the bytes alone would give: the exact Top-k baseline must read every K row once and the V rows of
        # its selection; full attention every K and V row
        n_rows = float(r.case.seq_lens(min(spec.T, 2)).sum()) * spec.Hkv
        x_bytes = n_rows * spec.D * e_k + lower
        res["byte_ratio_vs_exact_topk"] = round(x_bytes / step_bytes, 3)
        res["exact_topk_frac_of_hbm_peak"] = round(x_bytes / exact / 1e9 / HBM_PEAK_GBS, 4)
        # the contiguous stream of the full-attention baseline as the "achievable" reference beside the 8 TB/s peak
        t_ref = min(spec.T, 2)
        stream_bytes = 2.0 * float(r.case.seq_lens(t_ref).sum()) * spec.Hkv * row_bytes
        stream_gbs = stream_bytes / full / 1e9
        res["stream_reference"] = {"kernel": "full_attn (contiguous K and V stream)", "bytes": round(stream_bytes),
                                   "GB_per_s": round(stream_gbs, 1), "frac_of_hbm_peak": round(stream_gbs / HBM_PEAK_GBS, 4)}
        res["roofline"]["frac_of_stream_reference"] = round(achieved / stream_gbs, 4)
    r.close()
    return res, r.case


def measure_sweep(batches, contexts, steps, warmup):
    """The C4 recipe (bf16, r = 4, budget = context / 64) over a grid of batch sizes and context lengths: how the step,
    its dominant kernel and the two baselines scale with B x L on this GPU."""
    rows = []
    for L in contexts:
        for B in batches:
            ov = dict(name=f"C4-B{B}-L{L}", B=B, L=L, k=max(64, L // 64), T=max(steps + warmup, 4))
            res, _ = measure("C4", steps, warmup, with_baselines=True, use_graph=False, override=ov)
            rows.append({"B": B, "L": L, "k": ov["k"], "ms_per_step": round(res["ms_per_step"], 4),
                         "steps_per_s": round(res["steps_per_s"], 1), "cand_frac": res["cand_frac"],
                         "score_kernel": res["roofline"]["kernel"], "score_kernel_us": res["roofline"]["avg_launch_us"],
                         "score_kernel_GB_per_s": res["roofline"]["achieved"],
                         "score_kernel_frac_of_peak": res["roofline"]["frac"],
                         "exact_topk_ms": res["exact_topk_ms"], "full_attn_ms": res["full_attn_ms"],
                         "speedup_vs_exact_topk": res["speedup_vs_exact_topk"],
                         "speedup_vs_full_attn": res["speedup_vs_full_attn"]})
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
    return rows


def measure_paged(name, steps, warmup, block_size=16, layout="block_head_row"):
    """The main workload again with the cache as a paged pool (blocks of `block_size` rows in shuffled
    order, block table per request): same steps, final Top-k and outputs compared bit for bit with the
    contiguous run."""
    r0 = Runner(name)
    spec = r0.spec
    if steps <= 0:
        steps = max(1, spec.T - warmup)
    sec0 = r0.run_timed(steps, warmup)
    ref_idx, ref_out = r0.prev.clone(), r0.out.clone()
    r0.close()
    del r0
    r = Runner(name, paged_block=block_size, paged_layout=layout)
    sec = r.run_timed(steps, warmup)
    same = bool(r.torch.equal(r.prev, ref_idx)) and bool(r.torch.equal(r.out, ref_out))
    tm, cnts = r.run_kernel_timing(steps, warmup)
    filtered = tm["filter_score"][1] > 0
    kname = "filter_score" if filtered else "gather_score"
    by = float(algorithmic_bytes_score(spec, r.case, cnts, filtered).mean())
    us = tm[kname][0] / max(tm[kname][1], 1) * 1e3
    res = {"block_size": block_size,
           "layout": ("[block, head, row, D]" if layout == "block_head_row" else "[block, row, head, D]") + ", blocks in shuffled order",
           "ms_per_step": round(sec * 1e3, 4), "contiguous_ms_per_step": round(sec0 * 1e3, 4),
           "matches_contiguous_bitwise": same,
           "kernel_us": {k: round(v[0] / steps * 1e3, 2) for k, v in tm.items() if v[1]},
           "score_kernel": {"kernel": kname, "avg_launch_us": round(us, 2),
                            "GB_per_s": round(by / (us * 1e-6) / 1e9, 1) if us > 0 else None,
                            "frac_of_hbm_peak": round(by / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if us > 0 else None}}
    r.close()
    return res


def measure_host_kv(name, steps, warmup):
    """The paper's placement (its Sec. 4 overview): the KV cache stays in pinned host memory and the kernels fetch
    only the rows they touch over the host link.  Reported: the step time, the bytes a step moves over the link
    (candidate K rows once per KV group, selected V rows per head) against the stream of all keys that a
    transfer-then-index design needs (Sec. 1), and the link rate reached; final Top-k and outputs compared bit
    for bit with the device-resident run."""
    import torch
    r0 = Runner(name)
    spec = r0.spec
    if steps <= 0:
        steps = max(1, min(spec.T - warmup, 10))
    steps = min(steps, 10)                       # a step takes milliseconds here: keep the leg short
    r0.run_timed(steps, warmup)
    ref_idx, ref_out = r0.prev.clone(), r0.out.clone()
    Kh = torch.empty(r0.K.shape, dtype=r0.K.dtype, pin_memory=True)
    Vh = torch.empty(r0.V.shape, dtype=r0.V.dtype, pin_memory=True)
    Kh.copy_(r0.K)
    Vh.copy_(r0.V)
    torch.cuda.synchronize()
    r0.K, r0.V = Kh, Vh                          # the same runner over the host-resident copy
    r0.views = [r0.ctx.kv_view(Kh, Vh, r0.seq[t]) for t in range(spec.T + 1)]
    sec = r0.run_timed(steps, warmup)
    same = bool(torch.equal(r0.prev, ref_idx)) and bool(torch.equal(r0.out, ref_out))
    tm, cnts = r0.run_kernel_timing(steps, warmup)
    e = 2 if spec.kv_dtype != "f32" else 4
    k_rows = float(cnts.sum(axis=(1, 2)).mean())
    v_rows = float(r0.case.k.sum()) * spec.Hq
    link_bytes = (k_rows + v_rows) * spec.D * e
    all_k = float(r0.case.seq_lens(min(spec.T, 2)).sum()) * spec.Hkv * spec.D * e
    res = {"workload": spec.name, "kv_in": "pinned host memory (hipHostMalloc), rows fetched by the kernels over the host link",
           "ms_per_step": round(sec * 1e3, 3), "steps": steps, "matches_device_resident_bitwise": same,
           "link_bytes_per_step": round(link_bytes), "k_rows_bytes": round(k_rows * spec.D * e),
           "v_rows_bytes_per_head_fetch": round(v_rows * spec.D * e),
           "all_keys_bytes": round(all_k), "fraction_of_all_keys_stream": round(link_bytes / all_k, 4),
           "link_GB_per_s": round(link_bytes / sec / 1e9, 1),
           "kernel_us": {k: round(v[0] / steps * 1e3, 1) for k, v in tm.items() if v[1]}}
    r0.close()
    return res


def measure_fp8_keys(name, steps, warmup, with_v=False):
    """The main workload with K (and, with_v, V) stored as OCP FP8 E4M3 (the same draws rounded to 3 mantissa
    bits): half the bytes per scored (and per gathered) row.  A different input, so nothing is compared with
    the bf16 run."""
    r = Runner(name, k_dtype="fp8", v_dtype="fp8" if with_v else "")
    spec = r.spec
    if steps <= 0:
        steps = max(1, spec.T - warmup)
    sec = r.run_timed(steps, warmup)
    recall = r.recall_vs_exact()
    tm, cnts = r.run_kernel_timing(steps, warmup)
    filtered = tm["filter_score"][1] > 0
    kname = "filter_score" if filtered else "gather_score"
    by = float(algorithmic_bytes_score(spec, r.case, cnts, filtered).mean())
    us = tm[kname][0] / max(tm[kname][1], 1) * 1e3
    exact = r.time_baseline("exact", 5)
    full = r.time_baseline("full", 5)
    res = {"k_dtype": "fp8 e4m3 (V fp8 e4m3)" if with_v else "fp8 e4m3 (V bf16)", "ms_per_step": round(sec * 1e3, 4), "steps_per_s": round(1.0 / sec, 2),
           "cand_frac": round(float(cnts.mean() / (spec.L or r.case.seq_lens0.mean())), 4),
           "recall_vs_exact_topk": round(recall, 4),
           "kernel_us": {k: round(v[0] / steps * 1e3, 2) for k, v in tm.items() if v[1]},
           "score_kernel": {"kernel": kname, "bytes_per_launch": round(by), "traffic": measured_traffic(spec.name, kname),
                            "avg_launch_us": round(us, 2),
                            "GB_per_s": round(by / (us * 1e-6) / 1e9, 1) if us > 0 else None,
                            "frac_of_hbm_peak": round(by / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if us > 0 else None},
           "exact_topk_ms": round(exact * 1e3, 4), "full_attn_ms": round(full * 1e3, 4)}
    r.close()
    return res


def measure_fp16_cache(name, steps, warmup):
    """The main workload with K and V stored as fp16 (the same draws rounded to half precision): same bytes as
    bf16, the scoring runs on the fp16 MFMA.  A different input, so nothing is compared with the bf16 run."""
    r = Runner(name, kv_dtype="f16")
    spec = r.spec
    if steps <= 0:
        steps = max(1, spec.T - warmup)
    sec = r.run_timed(steps, warmup)
    recall = r.recall_vs_exact()
    tm, cnts = r.run_kernel_timing(steps, warmup)
    filtered = tm["filter_score"][1] > 0
    kname = "filter_score" if filtered else "gather_score"
    by = float(algorithmic_bytes_score(spec, r.case, cnts, filtered).mean())
    us = tm[kname][0] / max(tm[kname][1], 1) * 1e3
    res = {"kv_dtype": "fp16", "ms_per_step": round(sec * 1e3, 4), "steps_per_s": round(1.0 / sec, 2),
           "cand_frac": round(float(cnts.mean() / (spec.L or r.case.seq_lens0.mean())), 4),
           "recall_vs_exact_topk": round(recall, 4),
           "kernel_us": {k: round(v[0] / steps * 1e3, 2) for k, v in tm.items() if v[1]},
           "score_kernel": {"kernel": kname, "bytes_per_launch": round(by), "avg_launch_us": round(us, 2),
                            "GB_per_s": round(by / (us * 1e-6) / 1e9, 1) if us > 0 else None,
                            "frac_of_hbm_peak": round(by / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if us > 0 else None}}
    r.close()
    return res


def measure_tables(name, steps, warmup, with_quality=False):
    """The same workload with the paper's own candidate rule (score tables, Eq. 7-10): lfps_table_step per step,
    tables initialised from the step-0 query (Eq. 4 with one query) during warm-up; first four rows = sinks,
    kept outside the tables as in the paper.  Reported next to the memoryless path, not as `value`."""
    r = Runner(name, table_mode=True, n_sink=4)
    spec = r.spec
    if steps <= 0:
        steps = max(1, spec.T - warmup)
    sec = r.run_timed(steps, max(warmup, 1))
    recall = r.recall_vs_exact()
    sec_graph, graph_ok = r.run_timed_graph(steps, max(warmup, 1))   # the tables' state is in device memory: replayable
    torch = r.torch
    # per-kernel times and candidate counts over the same steps
    r.reset()
    for _ in range(max(warmup, 1)):
        r.step()
    torch.cuda.synchronize()
    cnts = torch.zeros((steps, spec.B, spec.Hkv), dtype=torch.int32, device=r.dev)
    r.ctx.lfps_timing_enable(True)
    for i in range(steps):
        r.step()
        r.ctx.lfps_copy_cand_count(cnts[i])
    tm = r.ctx.lfps_timing_read()
    r.ctx.lfps_timing_enable(False)
    cn = cnts.cpu().numpy()
    heads = spec.B * spec.Hq
    lens = r.case.seq_lens0.astype(float)
    scan_bytes = float(lens.sum()) * spec.Hq * 8.0            # both fp32 tables of every head, read once per step
    scan_us = tm["table_flags"][0] / max(tm["table_flags"][1], 1) * 1e3
    res = {"steps_per_s": round(1.0 / sec, 2), "ms_per_step": round(sec * 1e3, 4), "steps": steps,
           "ms_per_step_hip_graph": round(sec_graph * 1e3, 4), "hip_graph_matches_eager": graph_ok,
           "decay": 0.95, "a": 0.2, "n_sink": 4,
           "cand_frac": round(float(cn.mean() / (spec.L or r.case.seq_lens0.mean())), 4),
           "recall_vs_exact_topk": round(recall, 4),
           "kernel_us": {k: round(v[0] / steps * 1e3, 2) for k, v in tm.items() if v[1]},
           "table_scan": {"bytes_per_launch": round(scan_bytes), "avg_launch_us": round(scan_us, 2),
                          "GB_per_s": round(scan_bytes / (scan_us * 1e-6) / 1e9, 1) if scan_us > 0 else None,
                          "frac_of_hbm_peak": round(scan_bytes / (scan_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if scan_us > 0 else None},
           "heads": heads}
    if with_quality:
        res["per_step"] = r.quality_per_step(spec.T)
    r.close()
    # the same with the head-sparsity bypass in front (Eq. 5-6, eps = 0.85, six local rows)
    rg = Runner(name, table_mode=True, n_sink=4, gated=True)
    rg.ctx.lfps_priors(rg.q[0], rg.views[0], rg.kbar, rg.vbar, rg.sigma2)
    sec_g = rg.run_timed(steps, max(warmup, 1))
    res["with_bypass"] = {"ms_per_step": round(sec_g * 1e3, 4), "eps": 0.85, "n_local": 6,
                          "bypassed_head_frac_last_step": round(float(rg.gate.float().mean().item()), 4)}
    if with_quality:
        res["with_bypass"]["per_step"] = rg.quality_per_step(spec.T)
    rg.close()
    return res


def measure_peaky(steps, warmup):
    """The concentrated-attention variant of C4 (gen.C4_PEAKY: a few hundred rows per KV group carry most of the
    softmax mass and the sinks are strong), on which the paper's own rule has something to find: the memoryless step,
    the score-table step and the score-table step with the head-sparsity bypass, each with its candidate fraction
    (the paper's Table 4 reports 1.7 % of the positions scored at 128K, a = 0.2), Eq. 2 recall and error against
    full attention per step."""
    name = "C4-peaky"
    mem, _ = measure(name, steps, warmup, with_baselines=True, use_graph=False, with_quality=True)
    tab = measure_tables(name, steps, warmup, with_quality=True)
    keep = ("ms_per_step", "steps_per_s", "cand_frac", "kernel_us", "per_step", "exact_topk_ms", "full_attn_ms",
            "speedup_vs_exact_topk", "speedup_vs_full_attn")
    return {"workload": "C4 with concentrated attention: 384 hot rows per KV group at logit +6.7, sinks at +13.5",
            "paper_table4_fraction_scored_128k_a0.2": 0.017,
            "memoryless": {k: mem[k] for k in keep if k in mem},
            "score_table": {k: tab[k] for k in ("ms_per_step", "steps_per_s", "cand_frac", "kernel_us", "per_step", "with_bypass")},
            "table_step_over_memoryless_step": round(tab["ms_per_step"] / mem["ms_per_step"], 3)}


def _oracle_chain_worker(spec, b, g, n_steps, barrier, results):
    """One host process of the all-cores oracle timing: the oracle's chained lfps_step on one (request, KV group),
    started together with the other workers (inputs are generated before the barrier and not timed)."""
    import numpy as np  # noqa: F401
    from threadpoolctl import threadpool_limits

    import gen
    from oracle import lfps_oracle as orc

    case = gen.make_case(spec)
    K, V = case.kv_group(b, g)
    kb = int(case.k[b])
    with threadpool_limits(limits=1):
        prev = [orc.exact_topk(case.q[0, b, spec.G * g + h], K, int(case.seq_lens0[b]), kb)[0] for h in range(spec.G)]
        barrier.wait()
        t0 = time.perf_counter()
        for t in range(1, n_steps + 1):
            res = orc.lfps_step(case.q[t, b, spec.G * g: spec.G * (g + 1)], K, V, prev, int(case.seq_lens(t)[b]), kb,
                                spec.r, 1, 0)
            prev = res["topk_idx"]
        results.put((n_steps, time.perf_counter() - t0))


def cpu_baseline_all_cores(spec, per_group_step_s, budget_s):
    """The oracle's lfps_step on every host core at once: one process per core, each chaining the decode steps of
    its own (request, KV group), all started together.  Returns (group-steps per second over all workers, workers,
    steps per worker)."""
    import multiprocessing as mp

    cores = int(os.environ.get("OMP_NUM_THREADS") or 0) or min(os.cpu_count() or 1, 16)
    cores = max(1, min(cores, 16, spec.B * spec.Hkv))
    n_steps = int(max(1, min(spec.T, budget_s / max(per_group_step_s, 1e-6))))
    ctx = mp.get_context("spawn")                 # the parent holds the GPU: workers start clean and never touch it
    barrier, results = ctx.Barrier(cores), ctx.Queue()
    groups = [((7 * i + 1) % spec.B, (3 * i + 2) % spec.Hkv) for i in range(cores)]
    procs = [ctx.Process(target=_oracle_chain_worker, args=(spec, b, g, n_steps, barrier, results)) for (b, g) in groups]
    import queue
    for p_ in procs:
        p_.start()
    got, deadline = [], time.perf_counter() + 600
    try:
        while len(got) < len(procs):
            try:
                got.append(results.get(timeout=1.0))
            except queue.Empty:
                if any(p_.exitcode not in (None, 0) for p_ in procs) or time.perf_counter() > deadline:
                    raise RuntimeError("a worker of the all-cores oracle timing ended early")
    except RuntimeError:
        barrier.abort()
        for p_ in procs:
            if p_.is_alive():
                p_.terminate()
        raise
    finally:
        for p_ in procs:
            p_.join(timeout=30)
    slowest = max(t for _, t in got)
    return sum(n for n, _ in got) / slowest, cores, n_steps


def cpu_baseline(case, budget_s):
    """The oracle's LFPS step (fp64 numpy) on a bounded sample of (request, KV group) pairs chained over the decode
    steps, scaled to the whole batch: on all host cores at once (`value`, one process per core) and on one thread."""
    import numpy as np
    from threadpoolctl import threadpool_limits

    from oracle import lfps_oracle as orc

    spec = case.spec
    # sampled (request, KV group) pairs, taken in this order until the time budget is spent
    groups = [(0, 0), (spec.B - 1, spec.Hkv - 1), (spec.B // 2, 3 % spec.Hkv)]
    groups += [((5 * i + 1) % spec.B, (3 * i + 1) % spec.Hkv) for i in range(24)]
    groups = list(dict.fromkeys(groups))
    n_steps_max = spec.T
    spent, done = 0.0, 0
    t_start = time.perf_counter()
    with threadpool_limits(limits=1):
        for (b, g) in groups:
            K, V = case.kv_group(b, g)                                 # input generation: not timed
            kb = int(case.k[b])
            prev = [orc.exact_topk(case.q[0, b, spec.G * g + h], K, int(case.seq_lens0[b]), kb)[0] for h in range(spec.G)]
            for t in range(1, n_steps_max + 1):
                t0 = time.perf_counter()
                res = orc.lfps_step(case.q[t, b, spec.G * g: spec.G * (g + 1)], K, V, prev,
                                    int(case.seq_lens(t)[b]), kb, spec.r, 1, 0)
                spent += time.perf_counter() - t0
                done += 1
                prev = res["topk_idx"]
                if spent > budget_s:
                    break
            if spent > budget_s or time.perf_counter() - t_start > 4 * budget_s + 60:
                break
        # the oracle's exact Top-k (+ sparse attention) and full attention on the last sampled group, for context
        t_ref = min(spec.T, 2)
        n_ref = int(case.seq_lens(t_ref)[b])
        t0 = time.perf_counter()
        for h in range(spec.G):
            I, _ = orc.exact_topk(case.q[t_ref, b, spec.G * g + h], K, n_ref, kb)
            orc.sparse_attn(case.q[t_ref, b, spec.G * g + h], K, V, I)
        exact_group = time.perf_counter() - t0
        t0 = time.perf_counter()
        for h in range(spec.G):
            orc.full_attn(case.q[t_ref, b, spec.G * g + h], K, V, n_ref)
        full_group = time.perf_counter() - t0
    per_group_step = spent / max(done, 1)
    groups_n = spec.B * spec.Hkv
    step_s = per_group_step * groups_n
    one_core = {"value": 1.0 / step_s, "unit": "steps/s", "cores": 1,
                "sample": f"{done} oracle lfps_step calls (fp64 numpy, 1 thread) on (request, KV group) samples of {spec.name}, "
                          f"{per_group_step * 1e3:.1f} ms each, scaled by B*Hkv = {groups_n} groups per step",
                "oracle_exact_topk_steps_per_s": 1.0 / (exact_group * groups_n),
                "oracle_full_attn_steps_per_s": 1.0 / (full_group * groups_n),
                "oracle_speedup_vs_exact_topk": exact_group / per_group_step}
    try:
        rate, cores, n_chain = cpu_baseline_all_cores(spec, per_group_step, budget_s)
    except Exception as exc:                        # the one-core figure stands in, and says so
        return {**one_core, "kind": "oracle", "all_cores_failed": repr(exc), "host_cores_available": os.cpu_count()}
    return {"value": rate / groups_n, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": f"{cores} host processes at once (one per core, fp64 numpy, 1 thread each), each chaining {n_chain} oracle "
                      f"lfps_step calls on its own (request, KV group) of {spec.name}; {rate:.1f} group-steps/s in all, "
                      f"scaled by B*Hkv = {groups_n} groups per step",
            "one_core": one_core, "host_cores_available": os.cpu_count()}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures the one-GPU hot path only: run it with --gpus 1 "
              "(no collective or multi-GPU path is part of this build)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)

    from paper_2506_15704_amd import build as lib_build
    lib_build.ensure_built()                      # loads what is built; compiles only if nothing is

    if args.calib_copy:
        from paper_2506_15704_amd.binding import lfps_calib_copy
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.zeros_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            lfps_calib_copy(dst, src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        assert bool((dst == 1).all())
        print(json.dumps({"calib_copy_bytes_read": 1 << 30, "calib_copy_bytes_written": 1 << 30, "launches": 10,
                          "avg_ms": round(dt * 1e3, 4), "GB_per_s_read_plus_write": round(2 * (1 << 30) / dt / 1e9, 1)}))
        return

    if args.sweep:
        rows = measure_sweep([int(x) for x in args.sweep_batches.split(",")], [int(x) for x in args.sweep_contexts.split(",")],
                             args.steps if args.steps > 0 else 6, args.warmup)
        print(json.dumps({"sweep": "C4 recipe (bf16, r=4, k=L/64)", "rows": rows}), flush=True)
        return
    if args.host_kv_only:
        print(json.dumps({"host_resident_kv": measure_host_kv(args.workload, args.steps, args.warmup)}), flush=True)
        return
    if args.peaky_only:
        print(json.dumps({"peaky_workload": measure_peaky(args.steps, args.warmup)}), flush=True)
        return
    if args.table_only:
        print(json.dumps({"workload": args.workload, "score_table_mode": measure_tables(args.workload, args.steps, args.warmup)}),
              flush=True)
        return
    if args.fp8_only:
        print(json.dumps({"workload": args.workload, "fp8_keys": measure_fp8_keys(args.workload, args.steps, args.warmup),
                          "fp8_keys_and_values": measure_fp8_keys(args.workload, args.steps, args.warmup, with_v=True)}),
              flush=True)
        return
    if args.paged_only:
        print(json.dumps({"workload": args.workload,
                          "paged_kv": measure_paged(args.workload, args.steps, args.warmup, args.paged_block, args.paged_layout)}),
              flush=True)
        return
    main_res, case = measure(args.workload, args.steps, args.warmup, with_quality=True, preheat_s=args.preheat_seconds)
    spec = case.spec
    line = {
        "metric": "LFPS decode steps/s per layer", "value": round(main_res["steps_per_s"], 2), "unit": "steps/s",
        "n_gpus": 1, "steps": main_res["steps"], "warmup": args.warmup, "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if spec.kv_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{spec.name}: B={spec.B} x L={spec.L or list(spec.L_range)}, 32/8 GQA heads, d=128, "
                               f"{spec.kv_dtype} K/V, k={spec.k or spec.k_frac}, r={spec.r}, {spec.T} decode steps",
                   "B": spec.B, "L": spec.L or list(spec.L_range), "k": spec.k or spec.k_frac, "r": spec.r},
        "roofline": main_res["roofline"],
        "preheat": main_res["preheat"],
        "kernel_us": main_res["kernel_us"], "step_us": main_res["step_us"],
        "sparse_attn": main_res["sparse_attn"], "stream_reference": main_res.get("stream_reference"),
        "ms_per_step_hip_graph": main_res["ms_per_step_hip_graph"],
        "hip_graph_matches_eager": main_res["hip_graph_matches_eager"],
        "cand_frac": main_res["cand_frac"], "recall_vs_exact_topk": main_res["recall_vs_exact_topk"],
        "exact_topk_ms": main_res.get("exact_topk_ms"), "full_attn_ms": main_res.get("full_attn_ms"),
        "speedup_vs_exact_topk": main_res.get("speedup_vs_exact_topk"),
        "speedup_vs_full_attn": main_res.get("speedup_vs_full_attn"),
        "byte_ratio_vs_exact_topk": main_res.get("byte_ratio_vs_exact_topk"),
        "exact_topk_frac_of_hbm_peak": main_res.get("exact_topk_frac_of_hbm_peak"),
        "whole_step": main_res["whole_step"], "per_step": main_res.get("per_step"),
    }
    # the paper's own figures (its Sec. 5: indexing on one Xeon Gold 6430 core, attention on an RTX 4090): context only
    line["paper_context"] = {"speedup_vs_full_attention": 22.8, "speedup_vs_exact_topk": 9.6,
                             "note": "other hardware and a trained model's attention; not a target for this metric"}
    if not args.no_table_mode:
        tab = measure_tables(args.workload, args.steps, args.warmup, with_quality=True)
        tab["speedup_vs_memoryless_step"] = round(main_res["ms_per_step"] / tab["ms_per_step"], 3)
        line["score_table_mode"] = tab
    if not args.no_fp8 and spec.kv_dtype == "bf16":
        line["fp8_keys"] = measure_fp8_keys(args.workload, args.steps, args.warmup)
        line["fp8_keys_and_values"] = measure_fp8_keys(args.workload, args.steps, args.warmup, with_v=True)
        line["fp16_cache"] = measure_fp16_cache(args.workload, args.steps, args.warmup)
    if not args.no_host_kv:
        line["host_resident_kv"] = measure_host_kv(args.workload, args.steps, args.warmup)
    if not args.no_paged:
        line["paged_kv"] = measure_paged(args.workload, args.steps, args.warmup, args.paged_block, args.paged_layout)
    if args.all_workloads:
        others = {}
        for name in ("C1", "C2", "C3", "C4", "C5"):
            if name == args.workload:
                continue
            res, _ = measure(name, 0, args.warmup, with_quality=True)
            others[name] = {k: res[k] for k in ("steps_per_s", "ms_per_step", "ms_per_step_hip_graph", "cand_frac", "recall_vs_exact_topk",
                                                "speedup_vs_exact_topk", "speedup_vs_full_attn", "byte_ratio_vs_exact_topk",
                                                "exact_topk_ms", "full_attn_ms", "kernel_us", "whole_step", "per_step")}
            others[name]["roofline_frac"] = res["roofline"]["frac"]
            others[name]["score_kernel"] = {k: res["roofline"][k] for k in ("kernel", "achieved", "frac", "bytes_per_launch", "avg_launch_us", "traffic")}
            others[name]["sparse_attn_frac_at_union_bytes"] = res["sparse_attn"]["frac_of_hbm_peak_at_union_bytes"]
            others[name]["steps_per_s"] = round(others[name]["steps_per_s"], 2)
            others[name]["ms_per_step"] = round(others[name]["ms_per_step"], 4)
            if not args.no_table_mode:
                t = measure_tables(name, 0, args.warmup)
                others[name]["score_table_mode"] = {k: t[k] for k in ("steps_per_s", "ms_per_step", "cand_frac",
                                                                        "recall_vs_exact_topk", "kernel_us")}
        line["other_workloads"] = others
        if not args.no_table_mode:
            line["peaky_workload"] = measure_peaky(args.steps, args.warmup)
    # The main workload timed once more after every other leg (GPU legs only: before the CPU oracle): the same K steps
    # behind the same warm-up, no pre-heat.  `value` stays the first measurement; this one shows whether the step time
    # drifted within the process (seen on some boxes, cause not established).
    r_end = Runner(args.workload)
    line["ms_per_step_end_of_run"] = round(r_end.run_timed(main_res["steps"], args.warmup) * 1e3, 4)
    r_end.close()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(case, args.cpu_seconds)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
