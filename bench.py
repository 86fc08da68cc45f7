#!/usr/bin/env python3
"""Benchmark of the MiniKV decode step on one MI355X.

One "step" = append the new token's K/V row + attention over a 2-bit, evicted cache, i.e. the per-token
hot path of Algorithm 1's Decoding procedure, as minikv_decode_step runs it: both in ONE launch (the same
step as the two calls kv_append_residual + minikv_decode_attn is timed next to it, and so are the other
decode workloads).  Every step runs on its OWN
seeded cache copy (different data, different addresses), so nothing is served from L2 or the Infinity
Cache and no state has to be reset inside the timed region; all inputs are resident in HBM before the
clock starts.  The other four baseline configurations, the prefill-side kv_quantize_pack, the flush, the
token selection, the prefill attention and the per-token quantized variant are timed separately and
reported in extra fields of the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--variant V]

Prints ONE JSON line (see the keys below).  `value` is effective HBM GB/s = algorithmic bytes per step
/ time per step; `roofline` is the decode kernel against the 8 TB/s HBM peak; `cpu_baseline` is the CPU
oracle timed on the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes one launch of the decode kernel moves, from hardware counters (rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE runs of this script, each reading scaled by what the same counter shows for the plain
# 1 GiB device copies of --calibrate-copy); the summaries are kept under profiles/.  Counter runs cannot
# be made from inside a timed run, so the figure is recorded here per workload; None = not measured.
MEASURED_TRAFFIC_BYTES = {
    "cfg4_llama3_8b_gqa_32k": 182781338,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--max-copies", type=int, default=0, help="cap on distinct cache copies (0: steps+warmup)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference dispatches for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def build_copies(api, W, torch, w, ncopy, dev, keep_first_inputs=False):
    """ncopy seeded cache copies of workload w, prefill-quantized on the GPU, residual one short of full.
    Returns (shape, copies, first inputs or None, kv_quantize_pack times in ms, bytes the quantizer moved)."""
    shape = None
    copies, quant_ms = [], []
    first = None
    gathered_bytes = 0
    for i in range(ncopy):
        inp = W.make_inputs(w, dev, seed_offset=i)
        if shape is None:
            # ragged workloads draw new lengths for every copy: size the caches for the longest possible
            tcap = w.tcap(w.L // w.G * w.G) if w.keep_range is not None else inp.Tcap
            shape = api.make_shape(w.B, w.Hq, w.Hkv, w.D, w.G, tcap, w.Rcap)
        cache = api.Cache(shape, device=dev)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        api.kv_quantize_pack(shape, inp.K, inp.V, w.L, inp.idx, inp.idx.shape[1], inp.n_tok, int(inp.n_tok.max()), cache)
        e1.record()
        r0 = w.Rcap - 1                                    # the timed step appends the last residual token
        cache.Rk.view(w.units, w.Rcap, w.D)[:, :r0].copy_(inp.Rk[:, :r0])
        cache.Rv.view(w.units, w.Rcap, w.D)[:, :r0].copy_(inp.Rv[:, :r0])
        cache.r_len.fill_(r0)
        k_new = inp.Rk[:, r0].contiguous()
        v_new = inp.Rv[:, r0].contiguous()
        out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float16, device=dev)
        torch.cuda.synchronize()
        quant_ms.append(e0.elapsed_time(e1))
        r_next = torch.zeros_like(cache.r_len)            # where minikv_decode_step leaves the next lengths
        copies.append(dict(cache=cache, q=inp.q, k_new=k_new, v_new=v_new, out=out, n_tok=inp.n_tok, r_next=r_next))
        if i == 0:
            nt = int(inp.n_tok.sum())
            gathered_bytes = nt * w.D * 2 * 2 + nt * (64 + 8 * w.D // w.G)
            if keep_first_inputs:
                first = inp
        del inp
        if i == 1 and (ncopy - 2) * (cache.nbytes() + 64 * 2**20) > torch.cuda.mem_get_info()[0] * 0.8:
            ncopy = max(2, int(torch.cuda.mem_get_info()[0] * 0.8 / (cache.nbytes() + 64 * 2**20)))
        if len(copies) >= ncopy:
            break
    return shape, copies, first, quant_ms, gathered_bytes


def time_attention(api, torch, shape, copies, sm, steps, offset=0):
    """Average duration of back-to-back minikv_decode_attn launches (one event pair around all of them: the
    figure holds the kernel and the dispatch of the next one) and the median of singly bracketed launches."""
    n = len(copies)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        c = copies[(offset + i) % n]
        api.minikv_decode_attn(shape, c["q"], c["cache"], sm, c["out"])
    e1.record()
    torch.cuda.synchronize()
    avg_ms = e0.elapsed_time(e1) / steps
    evs = []
    for i in range(steps):
        c = copies[(offset + i) % n]
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        api.minikv_decode_attn(shape, c["q"], c["cache"], sm, c["out"])
        b.record()
        evs.append((a, b))
    torch.cuda.synchronize()
    durs = sorted(a.elapsed_time(b) for a, b in evs)
    return avg_ms, durs[len(durs) // 2]


def parity_sample(api, W, torch, np, ref, w, shape, inp, got_out, units, sm):
    """Oracle on the listed units of the inputs `inp` (cache rebuilt by the oracle from the same rows) against the
    GPU output got_out [B, Hq, D] of the step that appended the last residual token.  Returns (parity dict,
    seconds of the oracle's quantizer, seconds per decode run, bytes of the sampled units)."""
    rep = w.Hq // w.Hkv
    dev = inp.K.device
    sel = torch.as_tensor(units, device=dev)
    rs = ref.RefShape(len(units), rep, 1, w.D, w.G, int(shape.Tcap), w.Rcap)
    rc = ref.RefCache(rs)
    t0 = time.perf_counter()
    assert ref.quantize_pack(rc, inp.K[sel].cpu().numpy(), inp.V[sel].cpu().numpy(),
                             inp.n_tok[sel].cpu().numpy(), inp.idx[sel].cpu().numpy()) == 0
    t_quant = time.perf_counter() - t0
    rc.Rk[:] = inp.Rk[sel].cpu().numpy(); rc.Rv[:] = inp.Rv[sel].cpu().numpy(); rc.r_len[:] = w.Rcap
    qs = inp.q.view(w.B, w.Hkv, rep, w.D).reshape(w.units, rep, w.D)[sel].cpu().numpy()
    times = []
    for _ in range(3):
        a = time.perf_counter()
        want, _, _ = ref.decode_attn(rc, qs, sm)
        times.append(time.perf_counter() - a)
    got = got_out.view(w.B, w.Hkv, rep, w.D).reshape(w.units, rep, w.D)[sel].float().cpu().numpy()
    # tolerance: 2e-3, or one fp16 step of the oracle's value where that is larger (|o| >= 2)
    wantf = want.astype(np.float32)
    diff = np.abs(got - wantf)
    step16 = np.spacing(np.abs(want).astype(np.float16)).astype(np.float32)
    q_len = inp.n_tok.cpu().tolist()
    par = {"max_abs_err_vs_oracle": float(diff.max()), "tolerance": "max(2e-3, one fp16 step of the value)",
           "max_abs_oracle_value": float(np.abs(wantf).max()), "sample_units": len(units),
           "ok": bool(np.all(diff <= np.maximum(2e-3, step16)))}
    return par, t_quant, sorted(times)[1], W.algorithmic_bytes(w, [q_len[u] for u in units], [w.Rcap] * len(units))


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the decode path shards over (batch, KV-head) units with "
              "no communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2411_18077_amd import api
    from paper_2411_18077_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    api.lib()                                             # fails loudly when libminikv.so is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = W.by_name(args.workload)
    sm = 1.0 / math.sqrt(w.D)
    api.minikv_set_variant(args.variant)

    # ------------------------------------------------------------------ build the cache copies
    ncopy = args.steps + args.warmup
    if args.max_copies:
        ncopy = min(ncopy, args.max_copies)
    t_build = time.time()
    shape, copies, sample_src, quant_times, gathered_bytes = build_copies(api, W, torch, w, ncopy, dev, keep_first_inputs=True)
    ncopy = len(copies)
    t_build = time.time() - t_build

    q_len = copies[0]["n_tok"].cpu().tolist()
    bytes_of = [W.algorithmic_bytes(w, c["n_tok"].cpu().tolist(), [w.Rcap] * w.units) for c in copies]
    alg_bytes = int(round(sum(bytes_of[(args.warmup + i) % ncopy] for i in range(args.steps)) / args.steps))

    def step(i):
        c = copies[i % ncopy]
        api.minikv_decode_step(shape, c["q"], c["k_new"], c["v_new"], c["cache"], c["r_next"], sm, c["out"])
        c["r_next"] = c["cache"].swap_r_len(c["r_next"])  # (host-side pointer swap: the lengths after the append)

    def step_two_calls(i):
        c = copies[i % ncopy]
        api.kv_append_residual(shape, c["k_new"], c["v_new"], c["cache"])
        api.minikv_decode_attn(shape, c["q"], c["cache"], sm, c["out"])

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.int32, device=dev).fill_(1)     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def warm_up(fn):
        """The W warm-up steps, then about 50 ms more of attention launches over the warm-up copies only: the host
        work since the caches were built leaves the GPU idle long enough for its clocks to drop, and W steps
        (half a millisecond) do not bring them back."""
        for i in range(args.warmup):
            fn(i)
        for i in range(1200 if args.warmup else 0):
            c = copies[i % min(args.warmup, ncopy)]
            api.minikv_decode_attn(shape, c["q"], c["cache"], sm, c["out"])
        torch.cuda.synchronize()

    # ------------------------------------------------------------------ timed region
    warm_up(step)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = alg_bytes / (ms_per_step * 1e-3) / 1e9

    # ------------------------------------------------------------------ the same step as two calls (residual one short again)
    for c in copies:
        c["cache"].r_len.fill_(w.Rcap - 1)
    warm_up(step_two_calls)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_two_calls(args.warmup + i)
    torch.cuda.synchronize()
    two_call_us = (time.perf_counter() - t0) * 1e6 / args.steps

    # ------------------------------------------------------------------ timing of the attention launch alone (events)
    attn_ms_avg, attn_ms_med = time_attention(api, torch, shape, copies, sm, args.steps, offset=args.warmup)
    achieved = alg_bytes / (attn_ms_avg * 1e-3) / 1e9

    result = {
        "metric": "decode_attn_effective_hbm_bandwidth_2bit_kv",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "higher_is_better": True,
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": w.name, "seed": "%d + 7919 per cache copy" % w.seed, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "context": w.L,
            "retained_per_unit": int(max(q_len)) if w.keep is not None else "ragged %d..%d" % (min(q_len), max(q_len)),
            "G": w.G, "residual": w.Rcap, "Tcap": int(shape.Tcap), "cache_copies": ncopy,
            "algorithmic_bytes_per_step": alg_bytes, "variant": args.variant,
            "step": "minikv_decode_step (append + attend in one launch)",
            "arithmetic": "2-bit codes as fp16 operands, fp32 accumulation, fp16 result",
        },
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 1),
        "step_as_two_calls": {"what": "kv_append_residual + minikv_decode_attn, same copies, same loop",
                              "us_per_step": round(two_call_us, 2),
                              "GB/s": round(alg_bytes / (two_call_us * 1e-6) / 1e9, 1)},
        "roofline": {
            "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
            "kernel": "decode_stream_kernel (the single launch of minikv_decode_attn)",
            "algorithmic_bytes_per_launch": alg_bytes,
            "avg_launch_us": round(attn_ms_avg * 1e3, 2), "median_single_bracketed_launch_us": round(attn_ms_med * 1e3, 2),
        },
    }

    # ------------------------------------------------------------------ parity + CPU baseline: the oracle on the whole workload
    if not args.no_cpu_baseline:
        from oracle import ref
        # every unit while that stays within about 10-30 s of CPU work, else a seeded sample (the extremes of a
        # ragged workload included)
        total_tok = sum(q_len)
        if total_tok * (w.Hq // w.Hkv) <= 8_000_000:
            units = list(range(w.units))
        else:
            rng = np.random.default_rng(w.seed)
            units = sorted(rng.choice(w.units, min(w.units, 32), replace=False).tolist())
            if w.keep is None:
                units = sorted(set(units[:-2] + [int(np.argmin(q_len)), int(np.argmax(q_len))]))
        # copies[0] was last run by the attention timing loops: its output is the step's result
        par, t_quant, cpu_s, samp_bytes = parity_sample(api, W, torch, np, ref, w, shape, sample_src, copies[0]["out"], units, sm)
        result["parity"] = par
        result["cpu_baseline"] = {
            "value": round(samp_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
            "kind": "oracle",
            "sample": "%d of %d (batch, KV-head) units of %s, all query heads, median of 3 runs (%.2f s each)"
                      % (len(units), w.units, w.name, cpu_s),
            "quantize_pack_s": round(t_quant, 3),
        }
    if not args.no_extras:
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        # kv_quantize_pack of the prompt's retained rows again, warm and back to back (the calls that built the cache
        # copies ran between host-side input generation, with the clocks down: their median is kept as "ms_cold")
        qt = sorted(quant_times[1:] or quant_times)
        qc = api.Cache(shape, device=dev)
        src = sample_src
        q_each = []
        for i in range(3 + 7):
            qc.q_len.zero_()
            a.record()
            api.kv_quantize_pack(shape, src.K, src.V, w.L, src.idx, src.idx.shape[1], src.n_tok, int(src.n_tok.max()), qc)
            b.record()
            torch.cuda.synchronize()
            if i >= 3:
                q_each.append(a.elapsed_time(b))
        q_ms = sorted(q_each)[len(q_each) // 2]
        result["quantize_pack"] = {
            "what": "kv_quantize_pack of the retained rows (gather + quantize + pack), median of 7 warm calls",
            "ms": round(q_ms, 4), "bytes": gathered_bytes, "GB/s": round(gathered_bytes / (q_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(gathered_bytes / (q_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 3),
            "ms_cold": round(qt[len(qt) // 2], 4),
        }
        del qc, src
    del sample_src

    if not args.no_extras:
        # the allocation-free entry point on the same copies (same kernel, workspace inside the library)
        if api.lib().minikv_static_workspace_units() >= w.units * ((w.Hq // w.Hkv + 3) // 4):
            for i in range(4 + args.steps):
                if i == 4:
                    a.record()
                cc = copies[i % ncopy]
                api.minikv_decode_attn_static(shape, cc["q"], cc["cache"], sm, cc["out"])
            b.record()
            torch.cuda.synchronize()
            result["decode_attn_static"] = {"what": "minikv_decode_attn_static, back-to-back launches",
                                            "us": round(a.elapsed_time(b) * 1e3 / args.steps, 2)}
        # flush: every unit quantizes its full residual (n_r tokens) into the packed cache.  Timed last among the
        # uses of these copies (it changes their lengths): one untimed call, then up to eight copies back to back.
        nfl = min(8, ncopy - 1)
        api.kv_flush_residual(shape, copies[ncopy - 1]["cache"])
        a.record()
        for i in range(nfl):
            api.kv_flush_residual(shape, copies[i]["cache"])
        b.record()
        torch.cuda.synchronize()
        fl_ms = a.elapsed_time(b) / max(nfl, 1)
        result["flush_residual"] = {"ms": round(fl_ms, 4), "tokens_per_unit": w.Rcap, "calls": nfl,
                                    "amortised_us_per_step": round(fl_ms * 1e3 / w.Rcap, 3)}
        # reference point: a plain streaming read of 4 GiB (far beyond the 256 MB Infinity Cache), best of 5
        probe_src = torch.empty(1 << 30, dtype=torch.int32, device=dev).fill_(1)
        probe_sums = torch.zeros(2048, dtype=torch.int32, device=dev)
        best = 1e9
        for i in range(6):
            a.record()
            api.minikv_stream_read_probe(probe_src, probe_sums)
            b.record()
            torch.cuda.synchronize()
            if i:
                best = min(best, a.elapsed_time(b))
        ceiling = probe_src.numel() * 4 / (best * 1e-3) / 1e9
        del probe_src
        result["streaming_read_ceiling"] = {
            "what": "plain 128-bit streaming read of 4 GiB (minikv_stream_read_probe), best of 5",
            "GB/s": round(ceiling, 1),
            "decode_kernel_pct_of_it": round(100.0 * result["roofline"]["achieved"] / ceiling, 1),
        }
        # prefill-side token selection on this workload's shape: each unit keeps as many tokens as its cache
        # holds, half of them heavy hitters and half recent window, from synthetic cumulative attention scores
        rep = w.Hq // w.Hkv
        A = W.make_scores(w.units * rep, w.L, seed=w.seed + 5, device="cuda", kind="attention")
        kept = copies[0]["n_tok"]
        n_hh = (kept // 2 // w.G * w.G).to(torch.int32)
        n_rw = (kept - n_hh).to(torch.int32)
        stride = int(kept.max())
        sel_idx = torch.empty(w.units, stride, dtype=torch.int32, device="cuda")
        sel_n = torch.empty(w.units, dtype=torch.int32, device="cuda")
        nws = api.kv_select_workspace_bytes(w.units, rep, w.L)
        sel_ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
        reps = 10
        for i in range(2 + reps):
            if i == 2:
                a.record()
            api.kv_select_hh_rw(w.units, rep, w.L, A, n_hh, n_rw, sel_idx, stride, sel_n, sel_ws)
        b.record()
        torch.cuda.synchronize()
        sel_us = a.elapsed_time(b) * 1e3 / reps
        sel_bytes = W.selection_bytes(w.units, rep, w.L, sel_n.cpu().tolist())
        result["select_hh_rw"] = {
            "what": "kv_select_hh_rw on this shape (sum of the group's query heads, top n_hh by score + recent "
                    "window, ascending positions), mean of %d back-to-back calls" % reps,
            "us": round(sel_us, 2), "bytes": sel_bytes, "GB/s": round(sel_bytes / sel_us / 1e3, 1),
            "frac_of_hbm_peak": round(sel_bytes / sel_us / 1e3 / HBM_PEAK_GBS, 3),
        }
        del A, sel_idx, sel_ws
        # ... and on a few long prompts (the ragged configuration's shape: 8 units of 4 heads, 131072 tokens, 40 %
        # kept), where the selection runs with several workgroups per unit
        Ul, Ll, kl = 8, 131072, 26208
        A = W.make_scores(Ul * rep, Ll, seed=w.seed + 6, device="cuda", kind="attention")
        n_hh = torch.full((Ul,), kl, dtype=torch.int32, device="cuda")
        sel_idx = torch.empty(Ul, 2 * kl, dtype=torch.int32, device="cuda")
        sel_n = torch.empty(Ul, dtype=torch.int32, device="cuda")
        sel_ws = torch.empty(max(api.kv_select_workspace_bytes(Ul, rep, Ll), 16), dtype=torch.uint8, device="cuda")
        for i in range(2 + reps):
            if i == 2:
                a.record()
            api.kv_select_hh_rw(Ul, rep, Ll, A, n_hh, n_hh, sel_idx, 2 * kl, sel_n, sel_ws)
        b.record()
        torch.cuda.synchronize()
        long_us = a.elapsed_time(b) * 1e3 / reps
        long_bytes = W.selection_bytes(Ul, rep, Ll, sel_n.cpu().tolist())
        result["select_hh_rw"]["few_long_prompts"] = {
            "units": Ul, "rep": rep, "L": Ll, "us": round(long_us, 2), "bytes": long_bytes,
            "GB/s": round(long_bytes / long_us / 1e3, 1)}
        del A, sel_idx, sel_ws

        # prefill attention with cumulative scores (both passes), one sequence with this workload's heads and
        # context, and the longest prompt of the paper's kernel table (8192 tokens, 32 heads)
        def time_prefill(Bp, Hq, Hkv, Lp, reps):
            Qp, Kp, Vp = W.make_prefill_inputs(Bp, Hq, Hkv, Lp, w.seed + 9, device="cuda")
            xo = torch.empty_like(Qp)
            lse = torch.empty(Bp, Hq, Lp, dtype=torch.float32, device="cuda")
            acc = torch.empty(Bp, Hq, Lp, dtype=torch.float32, device="cuda")
            pws = torch.empty(api.selective_flash_attn_workspace_bytes(Bp, Hkv, Lp), dtype=torch.uint8, device="cuda")
            for i in range(1 + reps):
                if i == 1:
                    a.record()
                api.selective_flash_attn(Bp, Hq, Hkv, Lp, Qp, Kp, Vp, 1.0 / math.sqrt(w.D), xo, lse, acc, pws)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / reps
            fl = W.prefill_flops(Bp, Hq, Lp)
            return {"B": Bp, "Hq": Hq, "Hkv": Hkv, "L": Lp, "ms": round(ms, 3), "TFLOP/s": round(fl / ms / 1e9, 1),
                    "frac_of_fp16_mfma_peak": round(fl / ms / 1e9 / 2500.0, 3)}
        result["selective_flash_attn"] = {
            "what": "selective_flash_attn (X_O, LSE and A_cumul: transpose of V + row-block pass + column-block pass); "
                    "flops = 6*D per causal (query, key) pair; peak 2500 TFLOP/s (dense fp16 matrix instructions)",
            "this_shape": time_prefill(1, w.Hq, w.Hkv, w.L, 3),
            "paper_table_longest": time_prefill(1, 32, 32, 8192, 10),
            "paper_table_lengths": {
                "what": "ms at the four lengths of the paper's kernel latency table (32 heads of 128, one sequence; "
                        "the table's own batch and head count are not stated), next to its A100-40GB figures",
                "L": [1024, 2048, 4096, 8192],
                "ms": [time_prefill(1, 32, 32, Lt, 10)["ms"] for Lt in (1024, 2048, 4096, 8192)],
                "paper_ms_a100": [5.21, 14.85, 48.04, 187.83],
            },
        }

        # per-token quantized variant (the appendix's 4-bit baseline: bits = 4, one group per head) on this shape
        inp = W.make_inputs(w, dev, seed_offset=0)
        n16 = (inp.n_tok // 16 * 16).to(torch.int32)
        tcap_pt = (int(n16.max()) + 63) // 64 * 64
        pts = api.make_pt_shape(w.B, w.Hq, w.Hkv, w.D, 128, 4, tcap_pt)
        ptc = [api.PtCache(pts) for _ in range(3)]
        pt_q_ms = []
        for pc in ptc:
            a.record()
            api.kv_quantize_pack_pt(pts, inp.K, inp.V, w.L, inp.idx, inp.idx.shape[1], n16, int(n16.max()), pc)
            b.record()
            torch.cuda.synchronize()
            pt_q_ms.append(a.elapsed_time(b))
        pt_out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float16, device=dev)
        reps = 12
        for i in range(3 + reps):
            if i == 3:
                a.record()
            api.minikv_decode_attn_pt(pts, inp.q, ptc[i % 3], sm, pt_out)
        b.record()
        torch.cuda.synchronize()
        pt_us = a.elapsed_time(b) * 1e3 / reps
        pt_bytes = int(n16.sum()) * 2 * (w.D * 4 // 8 + 4) + 2 * w.B * w.Hq * w.D * 2
        pt_qbytes = int(n16.sum()) * (w.D * 2 * 2 + 2 * (w.D * 4 // 8 + 4))
        result["per_token_4bit_variant"] = {
            "what": "kv_quantize_pack_pt / minikv_decode_attn_pt with bits = 4, G = 128 (keys and values per token, the "
                    "appendix's 4-bit baseline) on this shape; 3 cache copies in rotation",
            "decode_us": round(pt_us, 2), "decode_bytes": pt_bytes, "decode_GB/s": round(pt_bytes / pt_us / 1e3, 1),
            "decode_frac_of_hbm_peak": round(pt_bytes / pt_us / 1e3 / HBM_PEAK_GBS, 3),
            "quantize_ms": round(sorted(pt_q_ms)[1], 4), "quantize_GB/s": round(pt_qbytes / (sorted(pt_q_ms)[1] * 1e-3) / 1e9, 1),
        }
        del inp, ptc

        # ---------------------------------------------------------------- the other baseline configurations
        del copies
        torch.cuda.empty_cache()
        others = {}
        for ow in W.WORKLOADS:
            if ow.name == w.name:
                continue
            cache_mb = W.algorithmic_bytes(ow, [int(ow.L * (ow.keep or 0.55))] * ow.units, [ow.Rcap] * ow.units) / 1e6
            nc = int(min(12, max(3, math.ceil(600.0 / max(cache_mb, 1.0)))))        # > 512 MB of distinct caches in rotation
            oshape, ocopies, oinp, oq_ms, _ = build_copies(api, W, torch, ow, nc, dev, keep_first_inputs=True)
            osteps = 40
            for i in range(len(ocopies)):                                            # the step: append, then attend
                oc = ocopies[i]
                api.kv_append_residual(oshape, oc["k_new"], oc["v_new"], oc["cache"])
                api.minikv_decode_attn(oshape, oc["q"], oc["cache"], sm, oc["out"])
            torch.cuda.synchronize()
            o_avg, o_med = time_attention(api, torch, oshape, ocopies, sm, osteps)
            ob = [W.algorithmic_bytes(ow, oc["n_tok"].cpu().tolist(), [ow.Rcap] * ow.units) for oc in ocopies]
            o_bytes = int(round(sum(ob[i % len(ocopies)] for i in range(osteps)) / osteps))
            entry = {"us_per_launch": round(o_avg * 1e3, 2), "median_single_launch_us": round(o_med * 1e3, 2),
                     "algorithmic_bytes": o_bytes, "GB/s": round(o_bytes / (o_avg * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak": round(o_bytes / (o_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "cache_copies": len(ocopies)}
            if not args.no_cpu_baseline:
                from oracle import ref
                oq = ocopies[0]["n_tok"].cpu().tolist()
                rng = np.random.default_rng(ow.seed)
                ou = sorted(rng.choice(ow.units, min(ow.units, 4), replace=False).tolist())
                if ow.keep is None:
                    ou = sorted(set(ou[:-2] + [int(np.argmin(oq)), int(np.argmax(oq))]))
                par, _, o_cpu_s, o_sb = parity_sample(api, W, torch, np, ref, ow, oshape, oinp, ocopies[0]["out"], ou, sm)
                entry["parity"] = par
                entry["oracle_GB/s"] = round(o_sb / o_cpu_s / 1e9, 4)
            if ow.name.startswith("cfg3"):
                # the prefill of this configuration: kv_quantize_pack of ALL 16384 tokens of every unit (no gather)
                inp3 = oinp
                full_n = torch.full((ow.units,), ow.L, dtype=torch.int32, device=dev)
                s3 = api.make_shape(ow.B, ow.Hq, ow.Hkv, ow.D, ow.G, ow.L, ow.Rcap)
                c3 = api.Cache(s3, device=dev)
                t3 = []
                for _ in range(3):
                    c3.q_len.zero_()
                    a.record()
                    api.kv_quantize_pack(s3, inp3.K, inp3.V, ow.L, None, 0, full_n, ow.L, c3)
                    b.record()
                    torch.cuda.synchronize()
                    t3.append(a.elapsed_time(b))
                b3 = ow.units * ow.L * (ow.D * 2 * 2 + 64 + 8 * ow.D // ow.G)
                entry["prefill_quantize_pack_all_tokens"] = {
                    "tokens_per_unit": ow.L, "ms": round(sorted(t3)[1], 4), "bytes": b3,
                    "GB/s": round(b3 / (sorted(t3)[1] * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(b3 / (sorted(t3)[1] * 1e-3) / 1e9 / HBM_PEAK_GBS, 3)}
                del c3, inp3
            others[ow.name] = entry
            del ocopies, oinp
            torch.cuda.empty_cache()
        result["other_configurations"] = {
            "what": "minikv_decode_attn on the other baseline configurations (back-to-back launches over rotating cache "
                    "copies, parity of one step against the oracle on sampled units)", **others}
        result["input_build_s"] = round(t_build, 1)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
