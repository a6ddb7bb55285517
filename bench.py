#!/usr/bin/env python3
"""Benchmark of the verify+draft hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM: fd_verify_draft_attn followed by the workload's acceptance call
(greedy or sampling) when it has one.  The attention calls start from a plan
(fd_verify_draft_plan) that is renewed inside the timed loop once per 36 calls, the way one
decoding step of Qwen3-8B plans once for its 36 layers.  The KV pool and
the logits are rotated over enough device copies that no step finds its input in the
256 MB last-level cache.  One JSON line is printed; `value` is algorithmic KV-cache bytes
per step divided by the step time.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--headline-only] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

ATTN_KERNELS = "attn_mfma_kernel + attn_mfma_combine_kernel (every kernel of a planned attention call, one event pair)"
HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
COLD_FOOTPRINT = 1.25e9         # bytes of distinct copies a rotating input must span
LAYERS_PER_PLAN = 36            # Qwen3-8B: one plan (fd_verify_draft_plan) per decoding step serves this many attention calls
MIN_KERNEL_SAMPLES = 20         # attention launches that are event-bracketed, whatever --steps is


ALL_WORKLOADS = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "seq_draft", "par4", "par_b1", "par_b2", "q3_1p7b", "q3_14b", "q3_32b", "d64"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Step:
    """Device state of one workload: rotating KV pools / logits and the prepared C-ABI arguments."""

    def __init__(self, fd, name, torch):
        from paper_2605_20022_amd import workloads as W
        from paper_2605_20022_amd.devcall import AttnCall, to_dev
        self.fd, self.torch, self.name = fd, torch, name
        w, a = W.CONFIGS[name]
        self.w, self.a = w, a
        t0 = time.time()
        inp = W.make_attention_inputs(w)
        self.inp = inp
        self.kv_bytes = W.kv_bytes(w, inp["kv_len"])
        self.flops = W.attention_flops(w, inp["kv_len"], inp["row_indptr"])
        call = AttnCall(fd, inp, want_lse=False)
        self.call = call
        pool_bytes = call.d["k_cache"].numel() * call.d["k_cache"].element_size() * 2
        n_pools = int(min(64, max(1, np.ceil(COLD_FOOTPRINT / pool_bytes))))
        self.pools = [(call.d["k_cache"], call.d["v_cache"])]
        for _ in range(n_pools - 1):
            self.pools.append((call.d["k_cache"].clone(), call.d["v_cache"].clone()))
        self.attn_args = []
        for k, v in self.pools:
            args = fd.fd_attn_args.from_buffer_copy(call.args)
            args.k_cache = k.data_ptr(); args.v_cache = v.data_ptr()
            args.flags |= fd.FD_ATTN_PLANNED           # the plan is made in attn(), once per LAYERS_PER_PLAN calls
            self.attn_args.append(args)
        self.attn_calls = 0
        # acceptance inputs
        self.acc = None
        if a is not None:
            indptr = W.verify_row_indptr(inp)
            Rv = int(indptr[-1])
            lg = W.make_logits(a, Rv)
            if a.mode == "greedy":
                f = (lg["target_logits"].astype(np.uint32) << 16).view(np.float32) if a.dtype == "bf16" else lg["target_logits"]
                agree = np.argmax(f, axis=1)          # input synthesis only: what the stand-in drafter agrees with
                toks = W.make_draft_tokens_agreeing(a, indptr, agree)
            else:
                d32 = (lg["draft_logits"].astype(np.uint32) << 16).view(np.float32) if a.dtype == "bf16" else lg["draft_logits"]

                def q_row(j):                          # input synthesis only: the stand-in drafter's distribution
                    x = d32[j].astype(np.float64) / a.temperature
                    e = np.exp(x - x.max())
                    return e / e.sum()
                toks = W.make_draft_tokens_from_probs(a, indptr, q_row)
            B = w.batch
            d = dict(indptr=torch.from_numpy(indptr).cuda(), toks=torch.from_numpy(toks).cuda(),
                     acc=torch.zeros(B, dtype=torch.int32, device="cuda"),
                     bon=torch.zeros(B, dtype=torch.int32, device="cuda"),
                     kmax=int(np.diff(indptr).max()), Rv=Rv)
            tg = to_dev(lg["target_logits"])
            per_copy = tg.numel() * tg.element_size() * (2 if a.mode == "sample" else 1)
            n_cp = int(min(64, max(1, np.ceil(COLD_FOOTPRINT / per_copy))))
            d["target"] = [tg] + [tg.clone() for _ in range(n_cp - 1)]
            if a.mode == "sample":
                dr = to_dev(lg["draft_logits"])
                d["draft"] = [dr] + [dr.clone() for _ in range(n_cp - 1)]
                d["ua"] = torch.from_numpy(lg["u_accept"]).cuda(); d["ur"] = torch.from_numpy(lg["u_resample"]).cuda()
            d["ws"] = fd.alloc_workspace(fd.fd_accept_workspace(B, Rv, a.vocab, a.mode == "sample"))
            d["logit_bytes"] = per_copy
            self.acc = d
        self.i = 0
        log(f"[{name}] inputs ready in {time.time() - t0:.1f}s: KV {self.kv_bytes / 1e6:.1f} MB x {n_pools} pools, "
            f"rows {inp['q'].shape[0]}, acceptance {a.mode if a else 'none'}")

    def plan_if_due(self):
        """The lengths of a decoding step meet every layer: one planning call per LAYERS_PER_PLAN attention calls."""
        if self.attn_calls % LAYERS_PER_PLAN == 0:
            self.fd.fd_verify_draft_plan(self.attn_args[0])
        self.attn_calls += 1

    def attn(self):
        self.plan_if_due()
        self.fd.fd_verify_draft_attn(self.attn_args[self.i % len(self.attn_args)])

    def accept(self):
        d, a = self.acc, self.a
        j = self.i % len(d["target"])
        if a.mode == "greedy":
            self.fd.fd_accept_greedy(d["target"][j], d["indptr"], d["toks"], d["acc"], d["bon"],
                                     max_rows_per_seq=d["kmax"], workspace=d["ws"])
        else:
            self.fd.fd_accept_sample(d["target"][j], d["draft"][j], d["indptr"], d["toks"], d["ua"], d["ur"],
                                     d["acc"], d["bon"], temperature=a.temperature, max_rows_per_seq=d["kmax"],
                                     workspace=d["ws"])

    def step(self):
        self.attn()
        if self.acc is not None:
            self.accept()
        self.i += 1

    def time_append(self, steps=50):
        """fd_append_kv (commit of the anchor and the accepted drafts) on this workload.  The call is
        given lengths 16 below the real ones, so that every page list has room for the committed rows
        (they overwrite the last cached tokens of the pools: run this after everything else)."""
        torch = self.torch
        B = self.w.batch
        rng = np.random.default_rng(7)
        acc = torch.from_numpy(np.array([rng.integers(0, max(int(k), 1)) for k in self.inp["verify_len"]], dtype=np.int32)).cuda()
        short = (self.call.d["kv_len"] - 16).clamp_(min=0)
        out_len = torch.zeros(B, dtype=torch.int32, device="cuda")
        args = []
        for a in self.attn_args:
            b = self.fd.fd_attn_args.from_buffer_copy(a); b.kv_len = short.data_ptr(); args.append(b)
        for i in range(5):
            self.fd.fd_append_kv(args[i % len(args)], *self.pools[i % len(args)], acc, out_len)
        torch.cuda.synchronize()
        # back to back on a busy stream: one event pair around all calls (a lone tiny launch on an idle
        # stream measures the launch latency from idle, about 10 us, whatever the kernel does)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            self.fd.fd_append_kv(args[i % len(args)], *self.pools[i % len(args)], acc, out_len)
        e1.record()
        torch.cuda.synchronize()
        ts = [e0.elapsed_time(e1) / steps]
        rows = int((acc + 1).sum().item())
        return {"append_us": round(ts[len(ts) // 2] * 1e3, 2), "append_rows": rows}

    def timed(self, steps, warmup):
        """Wall-clock time of `steps` whole steps, nothing else on the stream."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def timed_kernels(self, steps):
        """The same loop of whole steps once more, with a HIP event pair on the launching stream
        (torch's current stream, which the binding hands to the library) around the attention call of
        every step: the time of the call's kernels, K1 + K2 where it has two.  A pair costs the stream
        a few microseconds, which is why the wall-clock pass above runs without them."""
        torch = self.torch
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for s, e in evs:
            self.plan_if_due()
            s.record(); self.fd.fd_verify_draft_attn(self.attn_args[self.i % len(self.attn_args)]); e.record()
            if self.acc is not None:
                self.accept()
            self.i += 1
        torch.cuda.synchronize()
        return [s.elapsed_time(e) for s, e in evs]

    def time_plan(self, steps=30):
        """fd_verify_draft_plan alone (event-bracketed)."""
        torch = self.torch
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for s, e in evs:
            s.record(); self.fd.fd_verify_draft_plan(self.attn_args[0]); e.record()
        torch.cuda.synchronize()
        ts = sorted(s.elapsed_time(e) for s, e in evs)
        return ts[len(ts) // 2]

    def timed_parts(self, steps, warmup):
        """Event-bracketed time of the attention call alone and the acceptance call alone."""
        torch = self.torch
        res = {}
        for label, fn in (("attn", self.attn), ("accept", self.accept if self.acc is not None else None)):
            if fn is None:
                continue
            for _ in range(warmup):
                fn(); self.i += 1
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for s, e in evs:
                s.record(); fn(); e.record(); self.i += 1
            torch.cuda.synchronize()
            ts = sorted(s.elapsed_time(e) for s, e in evs)
            res[label] = dict(median_ms=ts[len(ts) // 2], min_ms=ts[0])
        return res


def time_draft_select(fd, torch, batch=32, rows_per_seq=15, vocab=151936, steps=50, copies=4):
    """fd_draft_select on one step's worth of draft logits (bf16), rotating over several copies of
    the logits so that no call finds its input in a cache."""
    from paper_2605_20022_amd import workloads as W
    R = batch * rows_per_seq
    lg = [torch.from_numpy(W.make_peaked_logits(vocab, R, seed=c, peak_lo=10.0, peak_hi=20.0).view(np.int16)).cuda().view(torch.bfloat16)
          for c in range(copies)]
    ip = torch.arange(0, R + 1, rows_per_seq, dtype=torch.int32, device="cuda")
    tok = torch.zeros(R, dtype=torch.int32, device="cuda")
    conf = torch.zeros(R, dtype=torch.float32, device="cuda")
    keep = torch.zeros(batch, dtype=torch.int32, device="cuda")
    ws = fd.alloc_workspace(fd.fd_draft_select_workspace(R, vocab))
    run = lambda i: fd.fd_draft_select(lg[i % copies], ip, tok, keep, temperature=1.0, threshold=0.3,
                                       max_rows_per_seq=rows_per_seq, confidence=conf, workspace=ws)
    for i in range(5):
        run(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i, (s, e) in enumerate(evs):
        s.record(); run(i); e.record()
    torch.cuda.synchronize()
    ts = sorted(s.elapsed_time(e) for s, e in evs)
    med = ts[len(ts) // 2] * 1e-3
    nbytes = R * vocab * 2
    return {"rows": R, "vocab": vocab, "call_us": round(med * 1e6, 2), "logits_GBps": round(nbytes / med / 1e9, 1),
            "frac_hbm_peak": round(nbytes / med / 1e9 / HBM_PEAK_GBPS, 4), "mean_keep_len": round(float(keep.float().mean()), 2)}


def time_select_branch(fd, torch, batch=128, blocks=16, block_len=15, steps=50):
    """fd_select_branch: per sequence, keep the candidate block drafted under the accepted count."""
    B, nb, mb = batch, blocks, block_len
    toks = torch.randint(0, 151936, (B * nb * mb,), dtype=torch.int32, device="cuda")
    indptr = torch.arange(0, B * nb * mb + 1, nb * mb, dtype=torch.int32, device="cuda")
    nblocks = torch.full((B,), nb, dtype=torch.int32, device="cuda")
    acc = torch.randint(0, nb, (B,), dtype=torch.int32, device="cuda")
    out = torch.zeros(B, mb, dtype=torch.int32, device="cuda")
    fv = torch.ones(B, dtype=torch.int32, device="cuda")          # full parallel mode: block 0 saw the anchor only
    for _ in range(5):
        fd.fd_select_branch(toks, indptr, nblocks, acc, out, first_vis=fv)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fd.fd_select_branch(toks, indptr, nblocks, acc, out, first_vis=fv)
    e1.record()
    torch.cuda.synchronize()
    ts = [e0.elapsed_time(e1) / steps]          # back to back on a busy stream
    return {"batch": B, "blocks": nb, "block_len": mb, "call_us": round(ts[len(ts) // 2] * 1e3, 2)}


def cpu_baseline(name, budget_s=20.0):
    """The oracle, as it stands, on a bounded sample of the same workload: whole sequences are
    added (shortest first would bias; seeded order is used) until about budget_s of CPU time."""
    from paper_2605_20022_amd import workloads as W
    from oracle import attention as oracle_attn
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    from oracle import acceptance as oracle_acc
    w, a = W.CONFIGS[name]
    inp = W.make_attention_inputs(w)
    lg, indptr = None, None
    if a is not None:                                   # acceptance leg of the step, one sequence at a time
        indptr = W.verify_row_indptr(inp)
        lg = W.make_logits(a, int(indptr[-1]))
    order = np.random.default_rng(0).permutation(w.batch)
    done_bytes, spent, used = 0, 0.0, 0
    for i in order:
        sub = W.subset_inputs(inp, [int(i)])
        t0 = time.perf_counter()
        oracle_attn.verify_draft_attention(
            sub["q"], sub["k_new"], sub["v_new"], sub["k_cache"], sub["v_cache"], sub["page_indptr"], sub["page_indices"],
            sub["kv_len"], sub["row_indptr"], sub["verify_len"], None, sub.get("mask_blocks"), page_size=w.page_size)
        if a is not None:
            r0, r1 = int(indptr[i]), int(indptr[i + 1])
            toks = np.zeros(r1 - r0, dtype=np.int32)    # the oracle's cost does not depend on the tokens
            if a.mode == "greedy":
                oracle_acc.accept_greedy(lg["target_logits"][r0:r1], [0, r1 - r0], toks)
            else:
                oracle_acc.accept_sample(lg["target_logits"][r0:r1], lg["draft_logits"][r0:r1], [0, r1 - r0], toks,
                                         lg["u_accept"][r0:r1], lg["u_resample"][r0:r1], a.temperature)
        spent += time.perf_counter() - t0
        done_bytes += W.kv_bytes(w, sub["kv_len"]); used += 1
        if spent > budget_s:
            break
    legs = "oracle attention + acceptance" if a is not None else "oracle attention"
    return dict(value=done_bytes / spent / 1e9, unit="GB/s", cores=int(threads), kind="oracle",
                sample=f"{used} of {w.batch} sequences of {name} ({legs}; the whole step when all sequences fit "
                       f"the {budget_s:.0f} s budget), {spent:.1f} s")


def read_profile(name):
    """Figures of the committed rocprofv3 summaries of this workload (profiles/attn_mfma_<name>_pmc.txt): HBM bytes
    per launch of the streaming kernel from the FETCH_SIZE / WRITE_SIZE counters, and the streaming and combine
    kernels' own durations.  Counters and per-kernel timestamps need the profiler, so they cannot be taken live."""
    path = os.path.join(ROOT, "profiles", f"attn_mfma_{name}_pmc.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            for key in ("traffic_bytes_per_launch", "k1_rocprofv3_avg_us", "k2_rocprofv3_avg_us"):
                if line.startswith(key + ":"):
                    out[key] = float(line.split(":")[1])
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", choices=ALL_WORKLOADS)
    ap.add_argument("--all-configs", dest="all_configs", action="store_true", default=True,
                    help="also report every configuration in per_config (default)")
    ap.add_argument("--headline-only", dest="all_configs", action="store_false",
                    help="skip the per-configuration table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run the library's plain 1 GiB streaming copy (bandwidth yard-stick, counter calibration)")
    ap.add_argument("--read-probe", action="store_true",
                    help="only run the library's staged streaming read over buffers of cfg3's, cfg5's and cfg4's KV size")
    ap.add_argument("--draft-select", action="store_true",
                    help="only time fd_draft_select (selective verification) on 32 x 15 rows of vocab 151936")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(sequences, KV heads or KV ranges would shard it).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_20022_amd import flexdraft as fd
    fd.load()                                  # raises if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.draft_select:
        print(json.dumps({"draft_select": time_draft_select(fd, torch, steps=args.steps)}), flush=True)
        return
    if args.copy_probe:
        from paper_2605_20022_amd import probes
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda"); dst = torch.empty_like(src)
        for _ in range(3):
            probes.stream_copy(src, dst)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            probes.stream_copy(src, dst)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"probe": "stream_copy", "bytes_read": n, "bytes_written": n, "launches": args.steps + 3,
                          "ms": round(dt * 1e3, 4), "GBps_read_plus_write": round(2 * n / dt / 1e9, 1)}), flush=True)
        return

    if args.read_probe:
        from paper_2605_20022_amd import probes, workloads as W
        res = []
        sums = torch.empty(probes.STREAM_READ_SUMS, dtype=torch.int32, device="cuda")
        for name in ("cfg3", "cfg5", "cfg4"):
            w = W.CONFIGS[name][0]
            n = W.kv_bytes(w, W.make_lengths(w)["kv_len"]) // 32768 * 32768
            pools = max(2, -(-(5 << 28) // n))                 # >= 1.25 GB of distinct data: every launch reads cold memory
            bufs = [torch.ones(n // 4, dtype=torch.int32, device="cuda") for _ in range(pools)]
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for i in range(3):
                probes.stream_read(bufs[i % pools], sums)
            for i, (e0, e1) in enumerate(ev):
                e0.record(); probes.stream_read(bufs[i % pools], sums); e1.record()
            torch.cuda.synchronize()
            us = np.array([e0.elapsed_time(e1) * 1e3 for e0, e1 in ev])
            res.append({"bytes_of": name, "bytes": n, "launches": args.steps, "us_mean": round(float(us.mean()), 2),
                        "us_min": round(float(us.min()), 2), "GBps": round(n / us.mean() / 1e3, 1)})
            del bufs
        print(json.dumps({"probe": "stream_read", "sizes": res}), flush=True)
        return

    st = Step(fd, args.workload, torch)
    ms_per_step = st.timed(args.steps, args.warmup)
    kern_ms = st.timed_kernels(max(args.steps, MIN_KERNEL_SAMPLES))
    parts = st.timed_parts(min(args.steps, 100), 5)
    kern_avg_ms = float(np.mean(kern_ms))
    value = st.kv_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = st.kv_bytes / (kern_avg_ms * 1e-3) / 1e9
    prof = read_profile(args.workload)
    k1_us = prof.get("k1_rocprofv3_avg_us")
    out = {
        "metric": "verify+draft attn: KV GB/s & % HBM peak; acceptance seqs/s at vocab 151936",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": st.w.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={st.w.batch}, KV len {st.w.kv_len_range}, page {st.w.page_size}, "
                               f"{st.w.num_q_heads}/{st.w.num_kv_heads} heads, D={st.w.head_dim}, "
                               f"k in {st.w.verify_len_range} + m={st.w.mask_len}, acceptance "
                               f"{st.a.mode + ' V=' + str(st.a.vocab) if st.a else 'none'}",
                   "kv_bytes_per_step": st.kv_bytes, "attention_flops_per_step": st.flops,
                   "kv_pools_rotated": len(st.pools)},
        "pct_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "attn_ms": parts.get("attn"), "accept_ms": parts.get("accept"),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": prof.get("traffic_bytes_per_launch"),
                     "traffic_source": "committed rocprofv3 --pmc summary under profiles/",
                     "kernel": ATTN_KERNELS,
                     "streaming_kernel_alone_us_rocprofv3": k1_us,
                     "streaming_kernel_alone_frac": round(st.kv_bytes / (k1_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if k1_us else None,
                     "kernel_avg_ms": round(kern_avg_ms, 5), "kernel_min_ms": round(float(np.min(kern_ms)), 5),
                     "kernel_launches_timed": len(kern_ms), "attention_calls_per_plan": LAYERS_PER_PLAN,
                     "mfma_tflops": round(st.flops / (kern_avg_ms * 1e-3) / 1e12, 2)},
    }
    if "accept" in parts:
        out["accept_seqs_per_s"] = round(st.w.batch / (parts["accept"]["median_ms"] * 1e-3), 1)
        out["accept_logits_GBps"] = round(st.acc["logit_bytes"] / (parts["accept"]["median_ms"] * 1e-3) / 1e9, 1)
    del st
    torch.cuda.empty_cache()

    if args.all_configs:
        per = {}
        for name in ALL_WORKLOADS:
            s2 = Step(fd, name, torch)
            n = 50
            s2.timed(5, 5)
            km = s2.timed_kernels(n)
            p2 = s2.timed_parts(n, 3)
            k_ms = float(np.mean(km))
            per[name] = {"kv_MB": round(s2.kv_bytes / 1e6, 2), "kernels_us": round(k_ms * 1e3, 2),
                         "kernels_kv_GBps": round(s2.kv_bytes / (k_ms * 1e-3) / 1e9, 1),
                         "kernels_frac_hbm_peak": round(s2.kv_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "attn_call_us": round(p2["attn"]["median_ms"] * 1e3, 2),
                         "plan_us": round(s2.time_plan() * 1e3, 2),
                         "mfma_tflops": round(s2.flops / (k_ms * 1e-3) / 1e12, 2)}
            if "accept" in p2:
                per[name]["accept_us"] = round(p2["accept"]["median_ms"] * 1e3, 2)
                per[name]["accept_seqs_per_s"] = round(s2.w.batch / (p2["accept"]["median_ms"] * 1e-3), 1)
            if name in ("cfg3", "cfg4"):
                per[name].update(s2.time_append(n))
            del s2
            torch.cuda.empty_cache()
        per["draft_select"] = time_draft_select(fd, torch)
        per["select_branch"] = time_select_branch(fd, torch)
        out["per_config"] = per

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
