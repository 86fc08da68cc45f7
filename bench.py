#!/usr/bin/env python3
"""Benchmark of the MiniKV decode step on one MI355X.

One "step" = kv_append_residual (the new token's K/V row) + minikv_decode_attn over a 2-bit, evicted
cache, i.e. the per-token hot path of Algorithm 1's Decoding procedure.  Every step runs on its OWN
seeded cache copy (different data, different addresses), so nothing is served from L2 or the Infinity
Cache and no state has to be reset inside the timed region; all inputs are resident in HBM before the
clock starts.  The prefill-side kv_quantize_pack and the flush are timed separately and reported in
extra fields of the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--variant V]

Prints ONE JSON line (see the keys below).  `value` is effective HBM GB/s = algorithmic bytes per step
/ time per step; `roofline` is the decode kernel against the 8 TB/s HBM peak; `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload.
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
    "cfg4_llama3_8b_gqa_32k": 181774746,
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
    free_b, _ = torch.cuda.mem_get_info()
    copies = []
    shape = None
    sample_src = None
    t_build = time.time()
    quant_times = []
    for i in range(ncopy):
        inp = W.make_inputs(w, dev, seed_offset=i)
        if shape is None:
            # ragged workloads draw new lengths for every copy: size the caches for the longest possible
            tcap = w.tcap(w.L // w.G * w.G) if w.keep_range is not None else inp.Tcap
            shape = api.make_shape(w.B, w.Hq, w.Hkv, w.D, w.G, tcap, w.Rcap)
        cache = api.Cache(shape, device=dev)
        n_max = int(inp.n_tok.max())
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        api.kv_quantize_pack(shape, inp.K, inp.V, w.L, inp.idx, inp.idx.shape[1], inp.n_tok, n_max, cache)
        e1.record()
        # residual holds Rcap-1 tokens; the timed step appends the last one
        r0 = w.Rcap - 1
        cache.Rk.view(w.units, w.Rcap, w.D)[:, :r0].copy_(inp.Rk[:, :r0])
        cache.Rv.view(w.units, w.Rcap, w.D)[:, :r0].copy_(inp.Rv[:, :r0])
        cache.r_len.fill_(r0)
        k_new = inp.Rk[:, r0].contiguous()
        v_new = inp.Rv[:, r0].contiguous()
        out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float16, device=dev)
        torch.cuda.synchronize()
        quant_times.append(e0.elapsed_time(e1))
        copies.append(dict(cache=cache, q=inp.q, k_new=k_new, v_new=v_new, out=out, n_tok=inp.n_tok))
        if i == 0:
            sample_src = inp                               # kept for the parity / cpu-baseline sample
            gathered_bytes = int(inp.n_tok.sum()) * w.D * 2 * 2 + int(inp.n_tok.sum()) * (64 + 8 * w.D // w.G)
        else:
            del inp
        if i == 1 and (ncopy - 2) * (cache.nbytes() + 64 * 2**20) > torch.cuda.mem_get_info()[0] * 0.8:
            ncopy = max(2, int(torch.cuda.mem_get_info()[0] * 0.8 / (cache.nbytes() + 64 * 2**20)))
    ncopy = len(copies)
    t_build = time.time() - t_build

    q_len = copies[0]["n_tok"].cpu().tolist()
    bytes_of = [W.algorithmic_bytes(w, c["n_tok"].cpu().tolist(), [w.Rcap] * w.units) for c in copies]
    alg_bytes = int(round(sum(bytes_of[(args.warmup + i) % ncopy] for i in range(args.steps)) / args.steps))
    append_bytes = 2 * w.units * w.D * 2 * 2               # read + write of the new K and V rows

    def step(i):
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

    # ------------------------------------------------------------------ timed region
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = alg_bytes / (ms_per_step * 1e-3) / 1e9

    # ------------------------------------------------------------------ timing of the attention launch alone (events)
    # One pair of events around K back-to-back launches (each on its own cache copy): the average then
    # holds the kernel and the dispatch of the next one, not the cost of recording events in between.
    # A second loop brackets every launch with its own pair, for the spread.
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(args.steps):
        c = copies[(args.warmup + i) % ncopy]
        api.minikv_decode_attn(shape, c["q"], c["cache"], sm, c["out"])
    e1.record()
    torch.cuda.synchronize()
    attn_ms_avg = e0.elapsed_time(e1) / args.steps
    evs = []
    for i in range(args.steps):
        c = copies[(args.warmup + i) % ncopy]
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        api.minikv_decode_attn(shape, c["q"], c["cache"], sm, c["out"])
        b.record()
        evs.append((a, b))
    torch.cuda.synchronize()
    durs = sorted(a.elapsed_time(b) for a, b in evs)
    attn_ms_med = durs[len(durs) // 2]
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
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": w.name, "seed": "%d + 7919 per cache copy" % w.seed, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "context": w.L,
            "retained_per_unit": int(max(q_len)) if w.keep is not None else "ragged %d..%d" % (min(q_len), max(q_len)),
            "G": w.G, "residual": w.Rcap, "Tcap": int(shape.Tcap), "cache_copies": ncopy,
            "algorithmic_bytes_per_step": alg_bytes, "variant": args.variant,
            "step": "kv_append_residual + minikv_decode_attn",
            "arithmetic": "2-bit codes as fp16 operands, fp32 accumulation, fp16 result",
        },
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 1),
        "roofline": {
            "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
            "kernel": "decode_stream_kernel (the single launch of minikv_decode_attn)",
            "algorithmic_bytes_per_launch": alg_bytes,
            "avg_launch_us": round(attn_ms_avg * 1e3, 2), "median_single_bracketed_launch_us": round(attn_ms_med * 1e3, 2),
        },
    }

    # ------------------------------------------------------------------ parity + CPU baseline on a bounded sample
    if not args.no_cpu_baseline:
        from oracle import ref
        import numpy as np
        nsamp = min(w.units, 64)
        rng = np.random.default_rng(w.seed)
        units = sorted(rng.choice(w.units, nsamp, replace=False).tolist())
        if w.keep is None:                                 # ragged: make sure the extremes are in
            units = sorted(set(units[:-2] + [int(np.argmin(q_len)), int(np.argmax(q_len))]))
            nsamp = len(units)
        rep = w.Hq // w.Hkv
        inp = sample_src
        sel = torch.as_tensor(units, device=dev)
        rs = ref.RefShape(nsamp, rep, 1, w.D, w.G, int(shape.Tcap), w.Rcap)
        rc = ref.RefCache(rs)
        t_q0 = time.perf_counter()
        assert ref.quantize_pack(rc, inp.K[sel].cpu().numpy(), inp.V[sel].cpu().numpy(),
                                 inp.n_tok[sel].cpu().numpy(), inp.idx[sel].cpu().numpy()) == 0
        t_q1 = time.perf_counter()
        rc.Rk[:] = inp.Rk[sel].cpu().numpy(); rc.Rv[:] = inp.Rv[sel].cpu().numpy(); rc.r_len[:] = w.Rcap
        qs = inp.q.view(w.B, w.Hkv, rep, w.D).reshape(w.units, rep, w.D)[sel].cpu().numpy()
        times = []
        for _ in range(5):
            a = time.perf_counter()
            want, _, _ = ref.decode_attn(rc, qs, sm)
            times.append(time.perf_counter() - a)
        cpu_s = sorted(times)[2]
        samp_bytes = W.algorithmic_bytes(w, [q_len[u] for u in units], [w.Rcap] * nsamp)
        got = copies[0]["out"].view(w.B, w.Hkv, rep, w.D).reshape(w.units, rep, w.D)[sel].float().cpu().numpy()
        # copies[0] was last run in the event loop or the timed loop; its output is the step's result
        # tolerance: 2e-3, or one fp16 step of the oracle's value where that is larger (|o| >= 2)
        wantf = want.astype(np.float32)
        diff = np.abs(got - wantf)
        step16 = np.spacing(np.abs(want).astype(np.float16)).astype(np.float32)
        err = float(diff.max())
        result["parity"] = {"max_abs_err_vs_oracle": err, "tolerance": "max(2e-3, one fp16 step of the value)",
                            "max_abs_oracle_value": float(np.abs(wantf).max()), "sample_units": nsamp,
                            "ok": bool(np.all(diff <= np.maximum(2e-3, step16)))}
        result["cpu_baseline"] = {
            "value": round(samp_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
            "kind": "oracle",
            "sample": "%d of %d (batch, KV-head) units of %s, all query heads, median of 5 runs (%.2f s each)"
                      % (nsamp, w.units, w.name, cpu_s),
            "quantize_pack_s": round(t_q1 - t_q0, 3),
        }

    if not args.no_extras:
        qt = sorted(quant_times[1:] or quant_times)
        q_ms = qt[len(qt) // 2]
        result["quantize_pack"] = {
            "what": "kv_quantize_pack of the retained rows (gather + quantize + pack), median over the cache copies",
            "ms": round(q_ms, 4), "bytes": gathered_bytes, "GB/s": round(gathered_bytes / (q_ms * 1e-3) / 1e9, 1),
        }
        # flush: every unit quantizes its full residual (n_r tokens) into the packed cache
        c = copies[0]
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        api.kv_flush_residual(shape, c["cache"])
        b.record()
        torch.cuda.synchronize()
        result["flush_residual"] = {"ms": round(a.elapsed_time(b), 4), "tokens_per_unit": w.Rcap,
                                    "amortised_us_per_step": round(a.elapsed_time(b) * 1e3 / w.Rcap, 3)}
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
        }
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
        result["build_s"] = round(t_build, 1)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
