#!/usr/bin/env python3
"""Benchmark of the BiLD decoding path on one MI355X.

A "step" is one whole BiLD generation (Algorithm 1) of `max_new` tokens for one
request of the chosen synthetic pair, with the source already encoded and all
weights resident in HBM.  Prints one JSON line:
  value        generated tokens / second of the BiLD loop (batch 1)
  roofline     the weight-streaming GEMM kernel: algorithmic weight bytes per
               launch / mean launch duration (its launches replayed alone between
               two HIP events on the library's stream), vs 8 TB/s
  cpu_baseline the CPU oracle timed on this host on the same workload
plus per-pass achieved GB/s (algorithmic bytes of one decoder pass / its time),
large-model-only greedy tokens/s and the BiLD-vs-large-only speedup.
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

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="t5", choices=["tiny", "t5", "mt5", "llama", "t5ee", "t5rel"])
    ap.add_argument("--shared-trunk", action="store_true",
                    help="early-exit workloads (tiny, t5ee): build the pair from the large model alone, so the two "
                         "models share the trunk's K/V cache and a large pass runs the upper layers only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-spread", action="store_true",
                    help="skip the 100 single passes per pass type (keeps a profiled run's kernel mix to the timed work)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="counter-collection run: one 1 GiB device copy of known size, then --steps BiLD steps; "
                         "no timing, no JSON (run under rocprofv3 --pmc with BILD_NO_GRAPH=1)")
    ap.add_argument("--top-p", type=float, default=0.0,
                    help="> 0: the sampling variant, both models draw from the nucleus of this mass (uniform numbers "
                         "from the seeded input generator)")
    ap.add_argument("--probe-stream", action="store_true",
                    help="no benchmark: print how fast 1..256 workgroups stream private regions of 32 KiB..1 MiB "
                         "(the per-compute-unit bandwidth the launch shapes are built around)")
    ap.add_argument("--alpha-fb", type=float, default=None)
    ap.add_argument("--alpha-rb", type=float, default=None)
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (--gpus 1); multi-GPU execution is not part of it.")
        return 2

    import numpy as np

    import bild_inputs as bi
    import paper_2302_07863_amd as pkg

    pkg.lib()  # fails loudly if the HIP library has not been built
    cfg = bi.PAIRS[args.workload]()
    fb = cfg.alpha_fb if args.alpha_fb is None else args.alpha_fb
    rb = cfg.alpha_rb if args.alpha_rb is None else args.alpha_rb
    t0 = time.time()
    ws, wl = bi.make_pair_weights(cfg)
    src = bi.make_source(cfg)
    log(f"[bench] weights generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    large = pkg.Model(pkg.config_from_shape(cfg.large), [wl[n] for n in bi.tensor_names(cfg.large)])
    if args.shared_trunk:
        if not cfg.early_exit:
            log(f"bench.py: --shared-trunk needs a workload whose small model is a prefix of the large one, not {cfg.name}")
            return 2
        pair = pkg.Pair.early_exit(large, cfg.small.n_dec, cfg.small.logit_scale)
    else:
        small = pkg.Model(pkg.config_from_shape(cfg.small), [ws[n] for n in bi.tensor_names(cfg.small)])
        pair = pkg.Pair(small, large)
    n0 = len(src) if cfg.decoder_only else 1
    st = pkg.State(pair, len(src), n0 + cfg.max_new + 2, cfg.n_max)
    log(f"[bench] models uploaded in {time.time() - t0:.1f}s")

    sampler_u = None
    if args.top_p > 0:
        n_u = n0 + cfg.max_new + 2
        sampler_u = (bi.make_uniforms(n_u, cfg.input_seed, 0), bi.make_uniforms(n_u, cfg.input_seed, 1))
        st.set_sampling(args.top_p, *sampler_u)
    t0 = time.perf_counter()
    st.encode(src)
    encode_ms = (time.perf_counter() - t0) * 1e3

    if args.probe_stream:
        print("groups  KiB/group   us/launch   GB/s per group   GB/s total")
        for groups in (1, 8, 32, 64, 128, 256, 512):
            for kib in (32, 64, 128, 256, 512, 1024):
                us = st.probe_stream(groups, kib, 8)
                print(f"{groups:6d} {kib:10d} {us:11.2f} {kib * 1.024 / us * 1e0:16.1f} {groups * kib * 1.024 / us:12.1f}", flush=True)
        print(f"empty launch: {st.probe_launch(2000):.2f} us")
        return 0

    if args.pmc_probe:
        st.gemm_tally(reset=True)          # count the decode GEMMs only (the encoder's row-block GEMMs are another kernel)
        st.probe_copy(1 << 30, 3)          # bild::probe_copy_kernel: reads 1 GiB and writes 1 GiB per launch
        for _ in range(args.steps):
            st.seq_truncate(n0)
            st.generate(None, fb, rb, cfg.max_new)
        tally = st.gemm_tally()
        log(f"[bench] pmc probe done: gemm launches issued {tally['launches']}, algorithmic weight bytes "
            f"{tally['bytes']}, mean {tally['bytes'] / max(tally['launches'], 1):.0f} B/launch")
        return 0

    def one_step():
        st.seq_truncate(n0)          # back to <s> / the prompt; caches cut to match
        return st.generate(None, fb, rb, cfg.max_new)

    for _ in range(args.warmup):
        toks, stats = one_step()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        toks, stats = one_step()
    dt = time.perf_counter() - t0
    n_tok = len(toks)
    tok_s = args.steps * n_tok / dt
    log(f"[bench] BiLD: {tok_s:.1f} tok/s, {dt / args.steps * 1e3:.2f} ms/step, stats {stats}")

    # large-model-only greedy on the same request (vanilla inference, the paper's reference point)
    def large_only():
        st.seq_truncate(n0)
        return st.greedy(pkg.LARGE, None, cfg.max_new)

    large_only()
    reps = max(2, args.steps // 4)
    t0 = time.perf_counter()
    for _ in range(reps):
        gl = large_only()
    large_tok_s = reps * len(gl) / (time.perf_counter() - t0)
    log(f"[bench] large-only greedy: {large_tok_s:.1f} tok/s")

    # per-pass achieved bandwidth at the end-of-generation cache length
    toks, stats = one_step()
    ln = st.lengths()
    passes = {}
    for name, which, rows in (("small_step", pkg.SMALL, 1), ("large_step", pkg.LARGE, 1),
                              ("large_verify_11", pkg.LARGE, 11)):
        t_cache = ln["y_len"] - rows
        have = st.lengths()["len_small" if which == pkg.SMALL else "len_large"]
        st.kv_truncate(which, min(have, t_cache))
        ms = st.bench_pass(which, rows, 50)
        nbytes = st.pass_bytes(which, t_cache, rows)
        passes[name] = dict(rows=rows, t_cache=t_cache, ms=round(ms, 4), bytes=nbytes,
                            gbs=round(nbytes / ms / 1e6, 1), frac_of_peak=round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4))
        # spread: 100 passes timed one by one (each between its own pair of events, so each includes the gap until
        # the host has submitted it; `ms` above is the mean of 50 passes submitted back to back)
        if not args.no_spread:
            singles = sorted(st.bench_pass(which, rows, 1) for _ in range(100))
            passes[name].update(single_p10_ms=round(singles[10], 4), single_median_ms=round(singles[50], 4),
                                single_p90_ms=round(singles[90], 4))
        log(f"[bench] {name}: {passes[name]}")

    # Roofline of the dominant kernel (the weight-streaming GEMM): its launches replayed alone, in pass
    # order and from the same captured graphs, between two HIP events on the library's stream; weighted by
    # the pass mix of the timed BiLD steps (small passes of 1 row, large passes of the mean review length).
    rows_l = max(1, round(stats["rows_verified"] / max(stats["large_calls"], 1)))

    def uncovered(which, rows):  # leave exactly `rows` tokens unconsumed by model `which`
        have = st.lengths()
        st.kv_truncate(which, min(have["len_small" if which == pkg.SMALL else "len_large"], have["y_len"] - rows))

    uncovered(pkg.SMALL, 1)
    g_s = st.bench_gemm(pkg.SMALL, 1, 50)
    uncovered(pkg.LARGE, rows_l)
    g_l = st.bench_gemm(pkg.LARGE, rows_l, 50)
    n_s, n_l = stats["small_steps"], stats["large_calls"]
    tot_l = n_s * g_s["launches"] + n_l * g_l["launches"]
    tot_b = n_s * g_s["bytes"] + n_l * g_l["bytes"]
    tot_ms = n_s * g_s["ms_per_pass"] + n_l * g_l["ms_per_pass"]
    achieved = tot_b / tot_ms / 1e6
    # HBM bytes per GEMM launch from hardware counters: taken from the committed rocprofv3 --pmc summary
    traffic = None
    pmc_file = os.path.join(ROOT, "profiles", f"gemm_{cfg.name}_pmc.txt")
    if os.path.exists(pmc_file):
        for line in open(pmc_file):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = int(line.split("=")[1])
    # one device function behind three thin launch wrappers (any rows / one row / merging attention partials)
    roofline = dict(bound="hbm", kernel="bild::gemm_kernel, gemm_row_kernel, gemm_few_kernel, gemm_merge_kernel (one body, %s)" %
                    ("bf16" if cfg.large.dtype == bi.DT_BF16 else "f32"),
                    achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                    traffic=traffic, launches_per_step=tot_l, mean_launch_us=round(tot_ms / tot_l * 1e3, 3),
                    mean_bytes_per_launch=int(tot_b / tot_l),
                    small_pass=dict(launches=g_s["launches"], us_per_launch=round(g_s["ms_per_pass"] / g_s["launches"] * 1e3, 3),
                                    gbs=round(g_s["bytes"] / g_s["ms_per_pass"] / 1e6, 1)),
                    large_pass=dict(rows=rows_l, launches=g_l["launches"],
                                    us_per_launch=round(g_l["ms_per_pass"] / g_l["launches"] * 1e3, 3),
                                    gbs=round(g_l["bytes"] / g_l["ms_per_pass"] / 1e6, 1)))
    log(f"[bench] roofline {roofline}")

    # The third line of the report: these passes are chains of dependent stages, so beside the bandwidth roofline stands
    # stage count x the cost of a launch that does nothing.
    launch_us = st.probe_launch(2000)

    def stages(shape):
        return 1 + shape.n_dec * (8 if shape.cross else 5) + 2     # embed, layer pieces, LM head, policy

    stage_latency = dict(empty_launch_us=round(launch_us, 3),
                         small_pass=dict(stages=stages(cfg.small), launch_floor_ms=round(stages(cfg.small) * launch_us * 1e-3, 4),
                                         measured_ms=passes["small_step"]["ms"]),
                         large_pass=dict(stages=stages(cfg.large), launch_floor_ms=round(stages(cfg.large) * launch_us * 1e-3, 4),
                                         measured_ms=passes["large_step"]["ms"]))
    log(f"[bench] stage latency {stage_latency}")

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        compact = args.workload == "llama"
        t0 = time.time()
        req = oracle.Request(oracle.Model(cfg.small, ws, compact), oracle.Model(cfg.large, wl, compact), src,
                             cfg.decoder_only)
        log(f"[bench] oracle set up + encoded in {time.time() - t0:.1f}s")
        n_cpu = cfg.max_new if args.workload != "llama" else 8
        t0 = time.perf_counter()
        smp = oracle.Sampler(args.top_p, *sampler_u) if sampler_u else None
        ref = oracle.bild_generate(req, fb, rb, cfg.n_max, n_cpu, sampler=smp)
        cdt = time.perf_counter() - t0
        cpu = dict(value=round(len(ref.tokens) / cdt, 2), unit="tokens/s", cores=int(cores), kind="oracle",
                   sample=f"one BiLD generation of {n_cpu} tokens on the same request (float64 numpy, decode only)",
                   tokens_equal_gpu=bool(ref.tokens == toks[:len(ref.tokens)]))
        log(f"[bench] cpu oracle {cpu}")

    out = {
        "metric": "generated tokens/sec (batch 1, BiLD loop)",
        "value": round(tok_s, 2),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.large.dtype == bi.DT_BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.small.name}+{cfg.large.name}, src {len(src)} tokens, "
                               f"{cfg.max_new} new tokens, alpha_FB={fb}, alpha_RB={rb}, n_max={cfg.n_max}"
                               + (", shared trunk (early-exit pair)" if args.shared_trunk else "")
                               + (f", nucleus sampling top_p={args.top_p}" if args.top_p > 0 else ""),
                   "tokens_per_step": n_tok},
        "roofline": roofline,
        "stage_latency": stage_latency,
        "cpu_baseline": cpu,
        "bild_stats": stats,
        "large_only_tokens_per_s": round(large_tok_s, 2),
        "speedup_vs_large_only": round(tok_s / large_tok_s, 3),
        "encode_ms": round(encode_ms, 2),
        # per request, the paper's "end-to-end latency per example": encode (or prompt prefill) + generation
        "end_to_end_tokens_per_s": round(n_tok / (encode_ms * 1e-3 + dt / args.steps), 2),
        "passes": passes,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
