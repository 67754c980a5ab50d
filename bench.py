#!/usr/bin/env python3
"""Benchmark of the fused UniPrefill score+select+compact operator on one MI355X.

One "step" is one uniprefill_fused call (plan, two scoring passes, merge,
select+compact) over one synthetic batch that is already resident in HBM.
Prints ONE JSON line: whole-operator tokens/s, the roofline figures of the
dominant kernel (per-kernel times measured with events on the launch stream),
and the CPU oracle timed on the host cores of the same machine.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def csrc_digest():
    """SHA-256 over the code of the library's kernel sources: what a counter measurement is valid for.
    Comments and white space are left out (an edit to a comment does not change what was measured), and
    so is the stand-alone pipe microbenchmark, which is not part of the library."""
    import hashlib
    import re
    d = os.path.join(ROOT, "paper_2605_06221_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")) and name != "up_pipes_bench.hip":
            text = open(os.path.join(d, name), encoding="utf-8").read()
            text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)      # block comments
            text = re.sub(r"//[^\n]*", " ", text)                   # line comments (no string in these sources holds "//")
            h.update(name.encode())
            h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def measured_traffic(workload, kernel):
    """HBM bytes per launch (reads + writes) of one kernel on one workload, from the rocprofv3 counter
    runs recorded in profiles/hbm_traffic.json (FETCH_SIZE and WRITE_SIZE, each scaled by what the same
    counter reads for an identity gather of known size in the same run).  The record names the profile
    summary it comes from and the digest of the kernel sources it was measured on; a record taken on
    other sources is not reported.  Returns (bytes or None, provenance dict or None)."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None, None
    ent = rec.get("bytes", {}).get(workload, {}).get(kernel)
    if ent is None:
        return None, None
    prov = {"profile": rec.get("profiles", {}).get(workload), "csrc_sha256": rec.get("csrc_sha256"),
            "stale": rec.get("csrc_sha256") != csrc_digest()}
    return (None if prov["stale"] else int(ent)), prov


def record_traffic(idx, fetch_csv, write_csv, profile):
    """Turn the rocprofv3 counter tables of two runs of `bench.py --config i --calibrate-copy ...` (one
    with --pmc FETCH_SIZE, one with --pmc WRITE_SIZE; KiB per dispatch) into this workload's entry of
    profiles/hbm_traffic.json, stamped with the digest of the kernel sources at hand.  The largest
    k_rows dispatch is the calibration copy, an identity gather of all T hidden rows: it reads the rows,
    T positions and T indices and writes the rows and T positions, which fixes each counter's scale."""
    import collections
    import csv
    import workloads
    workload = workloads.CONFIG_NAMES[idx]
    T = workloads.make_config(idx, hidden_dim=8).total_tokens      # (generated only for its lengths)
    row = {1: 1024, 2: 4096, 3: 4096, 4: 5120, 5: 4096}[idx] * 2   # bytes of a hidden row (bf16)
    def table(path):
        agg = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            agg[r["Kernel_Name"]].append(float(r["Counter_Value"]) * 1024.0)
        return agg
    rd, wr = table(fetch_csv), table(write_csv)
    rows = next(k for k in rd if "k_rows<false>" in k)
    scale_r = (T * row + 8 * T) / max(rd[rows])
    scale_w = (T * row + 4 * T) / max(wr[rows])
    def mean(agg, key, drop_max=False):
        v = sorted(x for k in agg if key in k for x in agg[k])
        if drop_max:
            v = v[:-1]
        return sum(v) / len(v) if v else 0.0
    def both(key, drop_max=False):
        return mean(rd, key, drop_max) * scale_r + mean(wr, key, drop_max) * scale_w
    ent = {"row_stats": round(both("k_sweep<1")), "merge_stats": round(both("k_combine")),
           "sweep_select": round(both("k_sweep<2") + both("k_finish")), "gather": round(both("k_rows<false>", True))}
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        rec = {}
    digest = csrc_digest()
    if rec.get("csrc_sha256") != digest:      # figures taken on other sources do not stay next to new ones
        rec["bytes"], rec["profiles"], rec["scale"] = {}, {}, {}
    rec["comment"] = ("HBM bytes per launch (reads + writes) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by "
                      "what the same counter reads for an identity gather of known size in the same run; written by "
                      "`bench.py --record-traffic`; the profile summaries named here give the commands and tables")
    rec["csrc_sha256"] = digest
    rec.setdefault("bytes", {})[workload] = ent
    rec.setdefault("profiles", {})[workload] = profile
    rec.setdefault("scale", {})[workload] = {"FETCH_SIZE": round(scale_r, 4), "WRITE_SIZE": round(scale_w, 4)}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1)
        f.write("\n")
    print(json.dumps({workload: ent, "scale": rec["scale"][workload], "csrc_sha256": digest}))


def algorithmic_bytes(w, total_kept):
    """Bytes the method must move: K once, a score per token, the kept rows in and out,
    index/position words, and the query window."""
    per_token = w.num_kv_heads * w.head_dim * 2 + 4
    per_kept = 2 * w.hidden_dim * 2 + 12
    q_bytes = sum(min(w.n_obs, int(w.cu_seqlens[r + 1] - w.cu_seqlens[r])) for r in range(w.num_seqs)) \
        * w.num_q_heads * w.head_dim * 2
    return w.total_tokens * per_token + total_kept * per_kept + q_bytes


def product_flops(w):
    """Flops of one Q.K^T pass: 2 * n_eff * N * D * Hq per sequence."""
    f = 0
    for r in range(w.num_seqs):
        N = int(w.cu_seqlens[r + 1] - w.cu_seqlens[r])
        f += 2 * min(w.n_obs, N) * N * w.head_dim * w.num_q_heads
    return f


def bench_chunked(args, up, workloads, np, torch):
    """Chunks that follow earlier context: the two-pass call and the call fed with the rows' log-sum-exp."""
    if not args.lengths:
        print("bench.py: --earlier needs --lengths", file=sys.stderr)
        sys.exit(2)
    lengths = [int(x) for x in args.lengths.split(",")]
    earlier = [int(x) for x in args.earlier.split(",")]
    if len(earlier) == 1:
        earlier = earlier * len(lengths)
    w = workloads.make_custom(name=f"llama8b_shape_{len(lengths)}x{max(lengths)}_after_{max(earlier)}_r{args.keep_ratio}",
                              seed=100, lengths=lengths, keep_ratio=[args.keep_ratio] * len(lengths), hidden_dim=4096,
                              num_q_heads=32, num_kv_heads=8, block_size=128, head_dim=args.head_dim, earlier=earlier)
    cu_host = np.ascontiguousarray(w.cu_seqlens, dtype=np.int32)
    cu_k_host = np.ascontiguousarray(w.cu_seqlens_k, dtype=np.int32)
    ratio_host = np.ascontiguousarray(w.keep_ratio, dtype=np.float32)
    p = up.make_params(num_seqs=w.num_seqs, total_tokens=w.total_tokens, block_size=w.block_size, n_obs=w.n_obs,
                       n_sink=w.n_sink, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                       hidden_dim=w.hidden_dim)
    _, _, total_kept, ws_bytes = up.uniprefill_plan_chunked(p, cu_host, cu_k_host, ratio_host)
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, hidden = dev(w.q), dev(w.k), dev(w.hidden)
    pos, cu, cu_k = torch.from_numpy(w.pos).cuda(), torch.from_numpy(cu_host).cuda(), torch.from_numpy(cu_k_host).cuda()
    ratio = torch.from_numpy(ratio_host).cuda()
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    hidden_out = torch.empty((total_kept, w.hidden_dim), dtype=torch.bfloat16, device="cuda")
    pos_out = torch.empty(total_kept, dtype=torch.int32, device="cuda")
    kept_idx = torch.empty(total_kept, dtype=torch.int32, device="cuda")
    kept_lse = torch.empty_like(kept_idx)
    new_cu = torch.empty(w.num_seqs + 1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    # the rows' log-sum-exp over earlier and own keys (an input of the second call; plain torch, fp64)
    lse = torch.full((w.num_q_heads, w.total_tokens), float("nan"), dtype=torch.float32, device="cuda")
    group, sc_l = w.num_q_heads // w.num_kv_heads, 1.0 / float(np.sqrt(w.head_dim))
    for r in range(w.num_seqs):
        c0, c1, k0, k1 = int(cu_host[r]), int(cu_host[r + 1]), int(cu_k_host[r]), int(cu_k_host[r + 1])
        n_eff = min(w.n_obs, c1 - c0)
        if n_eff == 0:
            continue
        rows = torch.arange(k1 - k0 - n_eff, k1 - k0, device="cuda")[:, None]
        cols = torch.arange(k1 - k0, device="cuda")[None, :]
        for h in range(w.num_q_heads):
            logits = (q[c1 - n_eff:c1, h, :].double() @ k[k0:k1, h // group, :].double().T) * sc_l
            logits.masked_fill_(cols > rows, float("-inf"))
            lse[h, c1 - n_eff:c1] = torch.logsumexp(logits, dim=1).float()

    def two_pass():
        up.uniprefill_fused_chunked(p, q, k, hidden, pos, cu, cu_host, cu_k, cu_k_host, ratio, ratio_host, hidden_out,
                                    pos_out, kept_idx, new_cu, None, workspace, ws_bytes, stream=stream)

    def from_lse():
        up.uniprefill_fused_lse(p, q, k, lse, w.total_tokens, hidden, pos, cu, cu_host, cu_k, cu_k_host, None, 0, 16,
                                ratio, ratio_host, hidden_out, pos_out, kept_lse, new_cu, None, workspace, ws_bytes,
                                stream=stream)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t1) / args.steps

    t_lse = timed(from_lse)
    t_two = timed(two_pass)
    parity = None
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from gpu_util import oracle_run
        ref = oracle_run(w)
        parity = bool(np.array_equal(kept_idx.cpu().numpy(), ref["kept_idx"])
                      and np.array_equal(hidden_out.view(torch.int16).cpu().numpy().view(np.uint16), ref["hidden_out"]))
    print(json.dumps({
        "metric": "tokens/s through fused score+select+compact op (chunk after earlier context)",
        "value": round(w.total_tokens / t_two, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(t_two * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "total_tokens": w.total_tokens, "key_tokens": int(cu_k_host[-1]),
                   "num_seqs": w.num_seqs, "total_kept": int(total_kept)},
        "roofline": None, "cpu_baseline": None,
        "fused_from_lse": {"ms_per_step": round(t_lse * 1e3, 4), "same_kept_set_as_fused": bool(torch.equal(kept_lse, kept_idx))},
        "oracle_parity": parity}), flush=True)


class Resident:
    """One workload in HBM with its outputs and workspace, and the fused call on it."""

    def __init__(self, w, up, np, torch, input_sets):
        self.w, self.up, self.np, self.torch = w, up, np, torch
        self.cu_host = np.ascontiguousarray(w.cu_seqlens, dtype=np.int32)
        self.ratio_host = np.ascontiguousarray(w.keep_ratio, dtype=np.float32)
        self.p = up.make_params(num_seqs=w.num_seqs, total_tokens=w.total_tokens, block_size=w.block_size,
                                n_obs=w.n_obs, n_sink=w.n_sink, num_q_heads=w.num_q_heads,
                                num_kv_heads=w.num_kv_heads, head_dim=w.head_dim, hidden_dim=w.hidden_dim)
        _, self.new_cu_plan, self.total_kept, self.ws_bytes = up.uniprefill_plan(self.p, self.cu_host, self.ratio_host)
        dev_bf16 = lambda bits: torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        self.q, self.k, self.hidden = dev_bf16(w.q), dev_bf16(w.k), dev_bf16(w.hidden)
        self.pos = torch.from_numpy(w.pos).cuda()
        self.cu = torch.from_numpy(self.cu_host).cuda()
        self.ratio = torch.from_numpy(self.ratio_host).cuda()
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.hidden_out = torch.empty((self.total_kept, w.hidden_dim), dtype=torch.bfloat16, device="cuda")
        self.pos_out = torch.empty(self.total_kept, dtype=torch.int32, device="cuda")
        self.kept_idx = torch.empty(self.total_kept, dtype=torch.int32, device="cuda")
        self.new_cu = torch.empty(w.num_seqs + 1, dtype=torch.int32, device="cuda")
        self.scores = torch.empty(w.total_tokens, dtype=torch.float32, device="cuda")
        self.stream = torch.cuda.current_stream()
        # identical copies of the large inputs: step i reads copy i % n, which the steps in between
        # have pushed out of the caches
        self.n_sets = max(1, input_sets)
        self.sets = [(self.q, self.k, self.hidden)] + [(self.q.clone(), self.k.clone(), self.hidden.clone())
                                                       for _ in range(self.n_sets - 1)]

    def call_args(self, i):
        qi, ki, hi = self.sets[i % self.n_sets]
        return (self.p, qi, ki, hi, self.pos, self.cu, self.cu_host, self.ratio, self.ratio_host, self.hidden_out,
                self.pos_out, self.kept_idx, self.new_cu, self.scores, self.workspace, self.ws_bytes)

    def ramp_clocks(self, ms):
        """Set-up, before any warm-up or timed step: keep the device under this load for `ms`
        milliseconds.  The part raises its clocks only after some tens of milliseconds of work (the
        sweeps of the 128k workload take 265 + 245 us in the first calls after an idle period and
        216 + 214 us from then on), so a handful of warm-up steps alone would time the ramp."""
        torch, up = self.torch, self.up
        t0 = time.perf_counter()
        n = 0
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(8):
                up.uniprefill_fused(*self.call_args(n), stream=self.stream)
                n += 1
            torch.cuda.synchronize()
        return n

    def time_fused(self, steps, warmup):
        """W untimed calls, then exactly K calls between two synchronisations (wall clock), with an event
        after every call for the spread of the single steps."""
        torch, up = self.torch, self.up
        for i in range(warmup):
            up.uniprefill_fused(*self.call_args(i), stream=self.stream)
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t_start = time.perf_counter()
        marks[0].record(self.stream)
        for i in range(steps):
            up.uniprefill_fused(*self.call_args(warmup + i), stream=self.stream)
            marks[i + 1].record(self.stream)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        per_step_us = sorted(marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(steps))
        pick = lambda f: round(per_step_us[min(len(per_step_us) - 1, int(f * len(per_step_us)))], 2)
        return elapsed / steps, {"median": pick(0.5), "p10": pick(0.1), "p90": pick(0.9)}

    def time_phases(self, steps):
        """The launches of the fused call one by one (uniprefill_fused_phases), each bracketed by events on
        the launch stream: average microseconds per kernel, launch gap included."""
        torch, up = self.torch, self.up
        phases = [("plan", up.UP_PHASE_PLAN), ("row_stats", up.UP_PHASE_ROW_STATS),
                  ("merge_stats", up.UP_PHASE_MERGE_STATS),
                  ("sweep_select", up.UP_PHASE_SWEEP_SELECT), ("gather", up.UP_PHASE_GATHER)]
        acc = {name: 0.0 for name, _ in phases}
        all_evs = []
        for it in range(steps):      # launched back to back (one synchronisation at the end): the clocks stay up
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(phases) + 1)]
            evs[0].record(self.stream)
            for i, (name, mask) in enumerate(phases):
                up.uniprefill_fused_phases(*self.call_args(it), mask, stream=self.stream)
                evs[i + 1].record(self.stream)
            all_evs.append(evs)
        torch.cuda.synchronize()
        for evs in all_evs:
            for i, (name, _) in enumerate(phases):
                acc[name] += evs[i].elapsed_time(evs[i + 1])
        return {name: acc[name] / steps * 1e3 for name, _ in phases}

    def time_gather_in_select(self, steps):
        """The variant in which the kernel that selects also copies its kept rows (one launch less):
        average microseconds per call, measured like the per-kernel loop.  Reported next to the fused
        call's figure; it is the slower of the two, which is why the fused call gathers in a launch
        of its own."""
        torch, up = self.torch, self.up
        mask = up.UP_PHASE_ALL | up.UP_PHASE_GATHER_IN_SELECT
        for it in range(2):
            up.uniprefill_fused_phases(*self.call_args(it), mask, stream=self.stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(self.stream)
        for it in range(steps):
            up.uniprefill_fused_phases(*self.call_args(it), mask, stream=self.stream)
        e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps * 1e3

    def kernel_table(self, phase_us):
        """Per-kernel figures: the sweeps against the dense bf16 MFMA peak (flops of one Q.K^T pass) and
        against HBM (K once; pass 2 also scores and kept ids), the gather against HBM."""
        w = self.w
        flops = product_flops(w)
        gather_only_bytes = self.total_kept * (2 * w.hidden_dim * 2 + 12)      # rows in and out, pos in/out, index
        score_bytes = w.total_tokens * 4 + self.total_kept * 4
        k_bytes = w.total_tokens * w.num_kv_heads * w.head_dim * 2
        kernels = {}
        for name, us in phase_us.items():
            ent = {"avg_us": round(us, 2)}
            if name in ("row_stats", "sweep_select"):
                ent.update(bound="mfma", tflops=round(flops / (us * 1e-6) / 1e12, 1),
                           frac_mfma=round(flops / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4))
                moved = k_bytes + (score_bytes if name == "sweep_select" else 0)
                ent.update(gbs=round(moved / (us * 1e-6) / 1e9, 1),
                           frac_hbm=round(moved / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
            if name == "gather":
                ent.update(bound="hbm", gbs=round(gather_only_bytes / (us * 1e-6) / 1e9, 1),
                           frac_hbm=round(gather_only_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
            kernels[name] = ent
        return kernels

    def against_oracle(self):
        """The results of the last fused call against the fp64 CPU oracle on the same inputs: bit-exact
        kept rows / compacted tensors / positions / offsets, the worst relative score error, and the
        margin the exactness rests on -- the smallest relative gap, over all selection blocks, between
        the last kept and the first dropped oracle score (exact ties of the quantised scores aside)."""
        np, torch = self.np, self.torch
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from gpu_util import oracle_run, score_margin_report      # test infrastructure: the fp64 numpy oracle
        t1 = time.perf_counter()
        ref = oracle_run(self.w)
        cpu_s = time.perf_counter() - t1
        torch.cuda.synchronize()
        K, R = self.total_kept, self.w.num_seqs
        parity = bool(np.array_equal(self.kept_idx.cpu().numpy(), ref["kept_idx"])
                      and np.array_equal(self.hidden_out.view(torch.int16).cpu().numpy().view(np.uint16), ref["hidden_out"])
                      and np.array_equal(self.pos_out.cpu().numpy(), ref["pos_out"])
                      and np.array_equal(self.new_cu.cpu().numpy(), ref["new_cu_seqlens"]))
        got = self.scores.cpu().numpy().astype(np.float64)
        want = ref["scores"].astype(np.float64)
        nz = want > 0
        rel = float(np.max(np.abs(got[nz] - want[nz]) / want[nz])) if nz.any() else 0.0
        zeros_agree = bool(np.array_equal(got[~nz], want[~nz]))
        margin = float(score_margin_report(ref, self.w))
        return {"oracle_parity": parity, "max_score_rel_err": rel, "floored_scores_agree": zeros_agree,
                "min_selection_margin": (None if margin == float("inf") else margin),
                "oracle_seconds": round(cpu_s, 2)}, ref


def summarise(res, sec_per_step):
    w = res.w
    alg_bytes = algorithmic_bytes(w, res.total_kept)
    flops = product_flops(w)
    return {
        "total_tokens": w.total_tokens, "num_seqs": w.num_seqs, "total_kept": int(res.total_kept),
        "ms_per_step": round(sec_per_step * 1e3, 4),
        "tokens_per_s": round(w.total_tokens / sec_per_step, 1),
        "algorithmic_bytes": int(alg_bytes),
        "hbm_frac": round(alg_bytes / sec_per_step / 1e9 / HBM_PEAK_GBS, 4),
        # the larger of (algorithmic bytes at HBM peak, the two product passes at the dense bf16 MFMA
        # peak) over the measured step time
        "binding_roofline_frac": round(max(alg_bytes / (HBM_PEAK_GBS * 1e9), 2.0 * flops / (MFMA_BF16_PEAK_TFLOPS * 1e12))
                                       / sec_per_step, 4),
    }


def bench_sweep(args, up, workloads, np, torch):
    """Operator-only timing tables (the shapes of the paper's block-size, window and context/batch
    studies): block size G x observation window n on one 32768-token Llama-3-8B-shaped sequence, and
    the context-length / batch-size grid; and the head dimension on one 131072-token sequence.  One JSON
    object with the three tables."""
    def run(lengths, G, n_obs, ratio=0.3, head_dim=128):
        w = workloads.make_custom(name=f"llama8b_{len(lengths)}x{max(lengths)}_G{G}_n{n_obs}_D{head_dim}", seed=100,
                                  lengths=lengths, keep_ratio=[ratio] * len(lengths), hidden_dim=4096, num_q_heads=32,
                                  num_kv_heads=8, block_size=G, n_obs=n_obs, head_dim=head_dim)
        res = Resident(w, up, np, torch, 1 if w.total_tokens >= 131072 else 2)
        res.ramp_clocks(args.ramp_ms)
        sec, _ = res.time_fused(args.steps, args.warmup)
        ph = res.time_phases(max(3, args.steps // 4))
        row = summarise(res, sec)
        row.update(G=G, n_obs=n_obs, head_dim=head_dim, lengths=f"{len(lengths)}x{max(lengths)}",
                   kernels_us={k: round(v, 1) for k, v in ph.items()})
        del res
        torch.cuda.empty_cache()
        print(f"[bench] sweep {row['lengths']} G={G} n={n_obs} D={head_dim}: {row['ms_per_step'] * 1e3:.1f} us", file=sys.stderr,
              flush=True)
        return row
    block_window = [run([32768], G, n) for G in (32, 64, 128) for n in (32, 128, 512)]
    grid = [run(ls, 128, 128) for ls in ([4096], [8192], [16384], [32768], [65536], [131072], [8192] * 4, [8192] * 16,
                                         [8192] * 64)]
    head_dims = [run([131072], 128, 128, head_dim=D) for D in (64, 128, 256)]
    print(json.dumps({"metric": "fused score+select+compact operator, microseconds per call", "dtype": "bf16",
                      "data": "synthetic", "steps": args.steps, "warmup": args.warmup,
                      "block_size_x_window_32k": block_window, "context_and_batch_grid": grid,
                      "head_dim_128k": head_dims}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default: the 128k-token one)")
    ap.add_argument("--lengths", type=str, default=None,
                    help="instead of --config: a Llama-3-8B-shaped batch (hidden 4096, 32/8 heads x 128, block "
                         "128) with these comma-separated sequence lengths, e.g. 8192,8192")
    ap.add_argument("--keep-ratio", type=float, default=0.3, help="keep ratio of a --lengths batch")
    ap.add_argument("--head-dim", type=int, default=128, help="head dimension of a --lengths batch (64, 128, 256)")
    ap.add_argument("--earlier", type=str, default=None,
                    help="with --lengths: tokens of earlier context per request whose keys are cached (chunked "
                         "prefill), e.g. --lengths 8192 --earlier 122880; times uniprefill_fused_chunked and "
                         "uniprefill_fused_lse on that batch (no per-kernel loop)")
    ap.add_argument("--input-sets", type=int, default=3,
                    help="copies of (q, k, hidden) in HBM that the steps rotate over, so that no step "
                         "finds its inputs in the 256 MB last-level cache (1 = warm)")
    ap.add_argument("--ramp-ms", type=float, default=60.0,
                    help="set-up before the warm-up steps: milliseconds of the same call, so that the part has "
                         "raised its clocks when the warm-up starts (0 = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-phases", action="store_true", help="skip the per-kernel timing loop")
    ap.add_argument("--no-entry-points", action="store_true", help="skip timing the stand-alone entry points")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the table of the other four workloads (the headline workload only)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: operator timing over block size x window and over "
                         "context length / batch size, as one JSON object")
    ap.add_argument("--csrc-digest", action="store_true", help="print the digest of the kernel sources and exit")
    ap.add_argument("--record-traffic", nargs=3, metavar=("FETCH_CSV", "WRITE_CSV", "PROFILE_MD"),
                    help="no GPU work: read the counter_collection.csv of a --pmc FETCH_SIZE and of a --pmc WRITE_SIZE "
                         "run of `bench.py --config i --calibrate-copy` and write that workload's entry of "
                         "profiles/hbm_traffic.json (with the digest of the kernel sources)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one identity gather of the whole hidden tensor (a plain copy of known "
                         "size): the reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.record_traffic:
        record_traffic(args.config, *args.record_traffic)
        return 0
    if args.csrc_digest:
        print(csrc_digest())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no sharding or collectives are built)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if not os.path.exists(os.path.join(ROOT, "paper_2605_06221_amd", "libuniprefill.so")):
        import __graft_entry__              # nothing built yet: build, never fall back
        __graft_entry__.build()
    import paper_2605_06221_amd as up      # fails loudly if the HIP library is missing or broken
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    t0 = time.time()
    if args.earlier:
        return bench_chunked(args, up, workloads, np, torch)
    if args.sweep:
        return bench_sweep(args, up, workloads, np, torch)
    if args.lengths:
        lengths = [int(x) for x in args.lengths.split(",")]
        w = workloads.make_custom(name=f"llama8b_shape_{len(lengths)}x{max(lengths)}_r{args.keep_ratio}_hd{args.head_dim}", seed=100,
                                  lengths=lengths, keep_ratio=[args.keep_ratio] * len(lengths), hidden_dim=4096,
                                  num_q_heads=32, num_kv_heads=8, block_size=128, head_dim=args.head_dim)
    else:
        w = workloads.make_config(args.config)
    print(f"[bench] generated {w.name}: T={w.total_tokens} R={w.num_seqs} in {time.time() - t0:.1f}s",
          file=sys.stderr, flush=True)

    res = Resident(w, up, np, torch, args.input_sets)
    p, q, k, hidden, pos, cu, cu_host = res.p, res.q, res.k, res.hidden, res.pos, res.cu, res.cu_host
    ratio, ratio_host, hidden_out, pos_out, kept_idx, new_cu = (res.ratio, res.ratio_host, res.hidden_out, res.pos_out,
                                                                res.kept_idx, res.new_cu)
    scores, workspace, ws_bytes, total_kept, stream = res.scores, res.workspace, res.ws_bytes, res.total_kept, res.stream

    ramp_calls = res.ramp_clocks(args.ramp_ms) if args.ramp_ms > 0 else 0
    sec_per_step, step_us = res.time_fused(args.steps, args.warmup)
    ms_per_step = sec_per_step * 1e3
    tokens_per_s = w.total_tokens / sec_per_step
    headline = summarise(res, sec_per_step)

    # ---- per-kernel durations: the same launches one by one, each bracketed by events on the stream
    kernels = {}
    roofline = None
    if not args.no_phases:
        kernels = res.kernel_table(res.time_phases(args.steps))
        # the dominant kernel against the roofline it gets closest to (its algorithmic bytes
        # against HBM peak, or its product flops against the dense bf16 MFMA peak)
        dom = max(kernels, key=lambda n: kernels[n]["avg_us"])
        ent = kernels[dom]
        traffic, provenance = measured_traffic(w.name, dom)
        if ent.get("frac_mfma", 0.0) > ent.get("frac_hbm", 0.0):
            roofline = {"kernel": dom, "bound": "mfma", "achieved": ent["tflops"],
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ent["frac_mfma"],
                        "traffic": traffic, "traffic_source": provenance}
        else:
            roofline = {"kernel": dom, "bound": "hbm", "achieved": ent.get("gbs"),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ent.get("frac_hbm"),
                        "traffic": traffic, "traffic_source": provenance}

    # ---- the stand-alone entry points and a plain device copy of the gather's byte count
    entry_points = {}
    if not args.no_entry_points:
        def timed(fn, reps=10):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3

        gather_bytes = 2 * total_kept * w.hidden_dim * 2
        full = torch.empty_like(hidden)
        src = torch.empty(gather_bytes // 2, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        t_us = {
            "score": timed(lambda: up.uniprefill_score(p, q, k, cu, cu_host, scores, workspace, ws_bytes, stream=stream)),
            "select": timed(lambda: up.uniprefill_select(p, scores, cu, cu_host, ratio, ratio_host, kept_idx, new_cu,
                                                        stream=stream)),
            "compact": timed(lambda: up.uniprefill_compact(p, hidden, pos, kept_idx, total_kept, hidden_out, pos_out,
                                                          stream=stream)),
            "scatter": timed(lambda: up.uniprefill_scatter(p, hidden_out, kept_idx, total_kept, full, stream=stream)),
            "device_copy_same_bytes": timed(lambda: dst.copy_(src)),
        }
        # the paper's own rule (block-level top-p at the paper's p = 0.99) on the scores just computed;
        # its outputs are sized for the worst case
        try:
            top_p_host = np.full(w.num_seqs, 0.99, dtype=np.float32)
            top_p_dev = torch.from_numpy(top_p_host).cuda()
            idx_all = torch.empty(w.total_tokens, dtype=torch.int32, device="cuda")
            cu_tp = torch.empty(w.num_seqs + 1, dtype=torch.int32, device="cuda")
            t_us["select_top_p"] = timed(lambda: up.uniprefill_select_top_p(
                p, scores, cu, cu_host, top_p_dev, top_p_host, idx_all, cu_tp, workspace, ws_bytes, stream=stream))
            top_p_kept = int(cu_tp[-1].item())
            del idx_all, cu_tp
        except up.UniPrefillError as e:      # e.g. more blocks per sequence than the top-p kernel orders
            top_p_kept = None
            print(f"[bench] top-p selection skipped: {e}", file=sys.stderr, flush=True)
        # the fused call when the attention layer hands over its rows' log-sum-exp: no first pass.
        # The normalisers come from a plain torch product here (an input of the call, not part of it).
        same_kept = None
        try:
            lse = torch.full((w.num_q_heads, w.total_tokens), float("nan"), dtype=torch.float32, device="cuda")
            group = w.num_q_heads // w.num_kv_heads
            sc_l = 1.0 / float(np.sqrt(w.head_dim))
            for r in range(w.num_seqs):
                c0, c1 = int(cu_host[r]), int(cu_host[r + 1])
                n_eff = min(w.n_obs, c1 - c0)
                if n_eff == 0:
                    continue
                rows = torch.arange(c1 - c0 - n_eff, c1 - c0, device="cuda")[:, None]
                cols = torch.arange(c1 - c0, device="cuda")[None, :]
                for h in range(w.num_q_heads):
                    logits = (q[c1 - n_eff:c1, h, :].double() @ k[c0:c1, h // group, :].double().T) * sc_l
                    logits.masked_fill_(cols > rows, float("-inf"))
                    lse[h, c1 - n_eff:c1] = torch.logsumexp(logits, dim=1).float()
            idx_lse = torch.empty_like(kept_idx)
            t_us["fused_from_lse"] = timed(lambda: up.uniprefill_fused_lse(
                p, q, k, lse, w.total_tokens, hidden, pos, cu, cu_host, None, None, None, 0, 16, ratio, ratio_host,
                hidden_out, pos_out, idx_lse, new_cu, None, workspace, ws_bytes, stream=stream))
            same_kept = bool(torch.equal(idx_lse, kept_idx))
            del lse, idx_lse
        except Exception as e:                # (e.g. out of memory for the logits of a very long batch)
            print(f"[bench] fused_from_lse skipped: {e}", file=sys.stderr, flush=True)
        for name, us in t_us.items():
            ent = {"avg_us": round(us, 2)}
            if name in ("compact", "scatter", "device_copy_same_bytes"):
                ent["gbs"] = round(gather_bytes / (us * 1e-6) / 1e9, 1)
                ent["frac_hbm"] = round(gather_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
            entry_points[name] = ent
        if top_p_kept is not None:
            entry_points["select_top_p"]["kept_at_p0.99"] = top_p_kept
        if same_kept is not None:
            entry_points["fused_from_lse"]["same_kept_set_as_fused"] = same_kept
        del full, src, dst

    if args.calibrate_copy:
        ident = torch.arange(w.total_tokens, dtype=torch.int32, device="cuda")
        full = torch.empty_like(hidden)
        fpos = torch.empty_like(pos)
        up.uniprefill_compact(p, hidden, pos, ident, w.total_tokens, full, fpos, stream=stream)
        torch.cuda.synchronize()
        print(f"[bench] calibration copy: k_rows gathers {w.total_tokens} rows of {w.hidden_dim * 2} bytes "
              f"(reads and writes {w.total_tokens * w.hidden_dim * 2} bytes each)", file=sys.stderr, flush=True)
        del ident, full, fpos

    # ---- the oracle on this machine's host cores (a reported baseline, not a target), and the
    # ---- results of the timed calls against it
    cpu_baseline = None
    checks = {}
    if not args.no_cpu_baseline:
        up.uniprefill_fused(*res.call_args(0), stream=stream)
        try:
            from threadpoolctl import threadpool_info
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
        checks, _ = res.against_oracle()
        cpu_s = checks["oracle_seconds"]
        cpu_baseline = {"value": round(w.total_tokens / cpu_s, 1), "unit": "tokens/s", "cores": int(threads),
                        "kind": "oracle", "seconds": cpu_s,
                        "sample": f"the full {w.name} batch, one pass (BLAS threads = cores; numpy exp is single-threaded)"}
        # the same pass on one thread (how much of the figure above is the BLAS library's threading)
        try:
            from threadpoolctl import threadpool_limits
            sys.path.insert(0, os.path.join(ROOT, "tests"))
            from gpu_util import oracle_run
            with threadpool_limits(limits=1):
                t1 = time.perf_counter()
                oracle_run(w)
                cpu_1 = time.perf_counter() - t1
            cpu_baseline["single_thread"] = {"value": round(w.total_tokens / cpu_1, 1), "seconds": round(cpu_1, 2)}
        except Exception:
            pass

    # ---- all five workloads in the same run: time, rooflines, parity, score error and margin
    table = {}
    if not args.no_workloads and not args.lengths:
        row = dict(headline)
        row.update(checks)
        row["kernels_us"] = {n: kernels[n]["avg_us"] for n in kernels}
        if not args.no_phases:
            row["gather_in_select_us"] = round(res.time_gather_in_select(args.steps), 2)
        table[w.name] = row
        del res, q, k, hidden, hidden_out, scores, workspace
        torch.cuda.empty_cache()
        for idx in (1, 2, 3, 4, 5):
            if workloads.CONFIG_NAMES[idx] == w.name:
                continue
            t1 = time.time()
            wi = workloads.make_config(idx)
            ri = Resident(wi, up, np, torch, args.input_sets if wi.total_tokens >= 100000 else max(args.input_sets, 8))
            if args.ramp_ms > 0:
                ri.ramp_clocks(args.ramp_ms)
            steps_i = max(5, min(args.steps, 20))
            sec_i, _ = ri.time_fused(steps_i, max(3, min(args.warmup, 5)))
            row = summarise(ri, sec_i)
            if not args.no_phases:
                row["kernels_us"] = {n: round(v, 2) for n, v in ri.time_phases(max(3, steps_i // 2)).items()}
                row["gather_in_select_us"] = round(ri.time_gather_in_select(steps_i), 2)
            if not args.no_cpu_baseline:
                up.uniprefill_fused(*ri.call_args(0), stream=ri.stream)
                row.update(ri.against_oracle()[0])
            table[wi.name] = row
            print(f"[bench] {wi.name}: {row['ms_per_step'] * 1e3:.1f} us per step ({time.time() - t1:.1f}s)", file=sys.stderr, flush=True)
            del ri, wi
            torch.cuda.empty_cache()

    out = {
        "metric": "tokens/s through fused score+select+compact op; % of MI355X HBM peak",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "step_us": step_us,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "total_tokens": w.total_tokens, "num_seqs": w.num_seqs,
                   "total_kept": int(total_kept), "input_sets": max(1, args.input_sets),
                   "clock_ramp_ms_before_warmup": args.ramp_ms, "clock_ramp_calls": ramp_calls},
        "algorithmic_bytes": headline["algorithmic_bytes"],
        "hbm_frac_fused": headline["hbm_frac"],
        "product_flops_per_pass": int(product_flops(w)),
        "binding_roofline_frac": headline["binding_roofline_frac"],
        "roofline": roofline,
        "kernels": kernels,
        "entry_points": entry_points,
        "cpu_baseline": cpu_baseline,
        "oracle_parity": checks.get("oracle_parity"),
        "max_score_rel_err": checks.get("max_score_rel_err"),
        "min_selection_margin": checks.get("min_selection_margin"),
        "workloads": table,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
