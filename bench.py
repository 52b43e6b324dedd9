#!/usr/bin/env python3
"""Benchmark of the BiLD decoding path on one MI355X.

A "step" is one whole BiLD generation (Algorithm 1) of `max_new` tokens for one
request of the chosen synthetic pair, with the source already encoded and all
weights resident in HBM.  Prints one JSON line:
  value        generated tokens / second of the BiLD loop (batch 1), passes replayed from captured graphs
  roofline     the weight-streaming GEMM kernel (the dominant kernel): algorithmic weight bytes per launch /
               mean duration of a launch (its launches of one BiLD generation replayed alone between two HIP
               events on the library's stream), vs 8 TB/s; rocprofv3's mean for the same launches beside it
  cpu_baseline the CPU oracle timed on this host on the same workload
plus per-pass achieved GB/s (algorithmic bytes of one decoder pass / its time) for this pair and, in the default
run, for the mT5-shaped pair as well, large-model-only greedy tokens/s and the BiLD-vs-large-only speedup.

  --workload verify   config 5: the large model's review pass alone on the 7B-shaped model with a cache of 4096
                      rows, T = 1, 4, 8, 16, 32 rows: time, GB/s, TFLOP/s and the sequential-vs-parallel ratio.
  --profile-run       what the committed rocprofv3 summaries are taken from: one encode and --steps BiLD
                      generations, nothing else (run with BILD_NO_GRAPH=1 under rocprofv3).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from dataclasses import replace
from types import SimpleNamespace

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profile_value(name: str, key: str):
    """`key=<number>` from a committed rocprofv3 summary under profiles/ (None if absent)."""
    path = os.path.join(ROOT, "profiles", name)
    if os.path.exists(path):
        for line in open(path):
            if line.startswith(key + "="):
                return float(line.split("=")[1])
    return None


def setup(workload: str, shared_trunk: bool = False, top_p: float = 0.0):
    """Seeded weights and source of one pair, uploaded, with the request encoded."""
    import bild_inputs as bi
    import paper_2302_07863_amd as pkg

    cfg = bi.PAIRS[workload]()
    t0 = time.time()
    ws, wl = bi.make_pair_weights(cfg)
    src = bi.make_source(cfg)
    log(f"[bench] {workload}: weights generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    large = pkg.Model(pkg.config_from_shape(cfg.large), [wl[n] for n in bi.tensor_names(cfg.large)])
    if shared_trunk:
        if not cfg.early_exit:
            raise SystemExit(f"bench.py: --shared-trunk needs a workload whose small model is a prefix of the large one, not {cfg.name}")
        pair = pkg.Pair.early_exit(large, cfg.small.n_dec, cfg.small.logit_scale)
    else:
        small = pkg.Model(pkg.config_from_shape(cfg.small), [ws[n] for n in bi.tensor_names(cfg.small)])
        pair = pkg.Pair(small, large)
    n0 = len(src) if cfg.decoder_only else 1
    st = pkg.State(pair, len(src), n0 + cfg.max_new + 2, cfg.n_max)
    log(f"[bench] {workload}: models uploaded in {time.time() - t0:.1f}s")
    sampler_u = None
    if top_p > 0:
        n_u = n0 + cfg.max_new + 2
        sampler_u = (bi.make_uniforms(n_u, cfg.input_seed, 0), bi.make_uniforms(n_u, cfg.input_seed, 1))
        st.set_sampling(top_p, *sampler_u)
    t0 = time.perf_counter()
    st.encode(src)
    encode_ms = (time.perf_counter() - t0) * 1e3
    return SimpleNamespace(cfg=cfg, ws=ws, wl=wl, src=src, pair=pair, st=st, n0=n0, sampler_u=sampler_u,
                           encode_ms=encode_ms, pkg=pkg, bi=bi, top_p=top_p)


def time_generation(c, fb, rb, steps, warmup):
    def one_step():
        c.st.seq_truncate(c.n0)          # back to <s> / the prompt; caches cut to match
        return c.st.generate(None, fb, rb, c.cfg.max_new)

    for _ in range(warmup):
        toks, stats = one_step()
    t0 = time.perf_counter()
    for _ in range(steps):
        toks, stats = one_step()
    dt = time.perf_counter() - t0
    return toks, stats, dt


def time_passes(c, spread: bool, rows_review: int = 11):
    """Per-pass time and achieved bandwidth at the end-of-generation cache length (state must hold a finished generation)."""
    pkg, st = c.pkg, c.st
    ln = st.lengths()
    passes = {}
    for name, which, rows in (("small_step", pkg.SMALL, 1), ("large_step", pkg.LARGE, 1),
                              (f"large_verify_{rows_review}", pkg.LARGE, rows_review)):
        t_cache = ln["y_len"] - rows
        have = st.lengths()["len_small" if which == pkg.SMALL else "len_large"]
        st.kv_truncate(which, min(have, t_cache))
        ms = st.bench_pass(which, rows, 50)
        nbytes = st.pass_bytes(which, t_cache, rows)
        passes[name] = dict(rows=rows, t_cache=t_cache, ms=round(ms, 4), bytes=nbytes,
                            gbs=round(nbytes / ms / 1e6, 1), frac_of_peak=round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4))
        # spread: 100 passes timed one by one (each between its own pair of events, so each includes the gap until
        # the host has submitted it; `ms` above is the mean of 50 passes submitted back to back)
        if spread:
            singles = sorted(st.bench_pass(which, rows, 1) for _ in range(100))
            passes[name].update(single_p10_ms=round(singles[10], 4), single_median_ms=round(singles[50], 4),
                                single_p90_ms=round(singles[90], 4))
        log(f"[bench] {c.cfg.name} {name}: {passes[name]}")
    return passes


def concurrent_leg(c, fb, rb, streams: int, reps: int, want_tokens):
    """Several independent requests at once, each a state of its own on a stream of its own, driven by one host thread
    each (the library's calls are blocking per request; ctypes releases the interpreter lock while they run).  Batch 1
    per request, as in the headline metric: this leg shows how much of the chip one request leaves idle."""
    import threading
    pkg, cfg = c.pkg, c.cfg
    states = [pkg.State(c.pair, len(c.src), c.n0 + cfg.max_new + 2, cfg.n_max) for _ in range(streams)]
    for st in states:
        if c.sampler_u:
            st.set_sampling(c.top_p, *c.sampler_u)
        st.encode(c.src)
        st.generate(None, fb, rb, cfg.max_new)  # captures the graphs of this state
    results = [None] * streams
    barrier = threading.Barrier(streams + 1)

    def worker(i):
        st = states[i]
        barrier.wait()
        for _ in range(reps):
            st.seq_truncate(c.n0)
            results[i] = st.generate(None, fb, rb, cfg.max_new)[0]
        barrier.wait()

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(streams)]
    for t in threads:
        t.start()
    barrier.wait()
    t0 = time.perf_counter()
    barrier.wait()
    dt = time.perf_counter() - t0
    for t in threads:
        t.join()
    same = all(r == want_tokens for r in results)
    for st in states:
        st.close()
    n_tok = len(want_tokens)
    return dict(streams=streams, tokens_per_s=round(streams * reps * n_tok / dt, 1),
                ms_per_generation=round(dt / reps * 1e3, 3), same_tokens_as_single_stream=same)


def review_histogram(c, fb, rb):
    """Rows per large-model pass of one BiLD generation, from the same generation driven through the low-level calls."""
    st, cfg = c.st, c.cfg
    st.seq_truncate(c.n0)
    hist, small_steps = {}, 0
    while st.lengths()["y_len"] - c.n0 < cfg.max_new:
        tok, flag, _ = st.small_step(fb)
        small_steps += 1
        if flag:
            ln = st.lengths()
            rows = ln["y_len"] - ln["draft_start"] + 1
            hist[rows] = hist.get(rows, 0) + 1
            st.large_verify(rb)
    return small_steps, hist


def roofline_leg(c, fb, rb, stats):
    """The dominant kernel, the weight-streaming GEMM (layer projections and LM head of both models: one device
    function).  Its launches are replayed ALONE, in pass order and from the same captured graphs, between two HIP events
    on the library's stream: the small model's pass and the large model's pass at every row count the BiLD generation
    uses, weighted by how often each occurs.  Elapsed time / launches is the mean duration of a launch including the
    gap to the next one (an empty kernel measured the same way costs 1.5 us, of which rocprofv3 reports 1.4 us as the
    kernel's own duration).  An event pair around every single launch is not used: around a kernel that does nothing
    such a pair already reads about 6 us."""
    pkg, st, cfg = c.pkg, c.st, c.cfg
    small_steps, hist = review_histogram(c, fb, rb)
    assert small_steps == stats["small_steps"] and sum(hist.values()) == stats["large_calls"], (small_steps, hist, stats)

    def uncovered(which, rows):  # leave exactly `rows` tokens unconsumed by model `which`
        have = st.lengths()
        st.kv_truncate(which, min(have["len_small" if which == pkg.SMALL else "len_large"], have["y_len"] - rows))

    uncovered(pkg.SMALL, 1)
    g_s = st.bench_gemm(pkg.SMALL, 1, 50)
    stages = {"small": st.pass_stages()}
    launches = small_steps * g_s["launches"]
    nbytes = small_steps * g_s["bytes"]
    ms = small_steps * g_s["ms_per_pass"]
    by_rows = {}
    for rows, count in sorted(hist.items()):
        uncovered(pkg.LARGE, rows)
        g = st.bench_gemm(pkg.LARGE, rows, 20)
        stages[f"large_{rows}"] = st.pass_stages()
        launches += count * g["launches"]
        nbytes += count * g["bytes"]
        ms += count * g["ms_per_pass"]
        by_rows[rows] = dict(passes=count, launches=g["launches"], us_per_launch=round(g["ms_per_pass"] / g["launches"] * 1e3, 3),
                             gbs=round(g["bytes"] / g["ms_per_pass"] / 1e6, 1))
    achieved = nbytes / ms / 1e6
    traffic = profile_value(f"gemm_{cfg.name}_pmc.txt", "traffic_bytes_per_launch")
    rocprof_us = profile_value(f"bild_{cfg.name}_kernel_stats.txt", "gemm_mean_us")
    return dict(bound="hbm",
                kernel="bild::gemm_kernel / gemm_row_kernel / gemm_few_kernel / gemm_merge_kernel (one body, %s)" %
                       ("bf16" if cfg.large.dtype == c.bi.DT_BF16 else "f32"),
                achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                traffic=None if traffic is None else int(traffic),
                launches_per_step=launches, mean_launch_us=round(ms / launches * 1e3, 3),
                mean_bytes_per_launch=int(nbytes / launches),
                stages_per_pass=stages,
                rocprofv3_mean_us=rocprof_us,
                frac_at_rocprofv3_mean=None if rocprof_us is None else round(nbytes / launches / rocprof_us / 1e3 / HBM_PEAK_GBS, 4),
                small_pass=dict(passes=small_steps, launches=g_s["launches"],
                                us_per_launch=round(g_s["ms_per_pass"] / g_s["launches"] * 1e3, 3),
                                gbs=round(g_s["bytes"] / g_s["ms_per_pass"] / 1e6, 1)),
                large_pass_by_rows=by_rows)


def cpu_baseline(c, fb, rb, top_p, gpu_tokens):
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        how = "BLAS threads reported by threadpoolctl"
    except Exception:
        cores = os.cpu_count() or 1
        how = "os.cpu_count()"
    cfg = c.cfg
    compact = cfg.name == "llama"
    t0 = time.time()
    req = oracle.Request(oracle.Model(cfg.small, c.ws, compact), oracle.Model(cfg.large, c.wl, compact), c.src,
                         cfg.decoder_only)
    log(f"[bench] oracle set up + encoded in {time.time() - t0:.1f}s")
    n_cpu = cfg.max_new if cfg.name != "llama" else 8
    t0 = time.perf_counter()
    smp = oracle.Sampler(top_p, *c.sampler_u) if c.sampler_u else None
    ref = oracle.bild_generate(req, fb, rb, cfg.n_max, n_cpu, sampler=smp)
    cdt = time.perf_counter() - t0
    return dict(value=round(len(ref.tokens) / cdt, 2), unit="tokens/s", cores=int(cores), cores_from=how, kind="oracle",
                sample=f"one BiLD generation of {n_cpu} tokens on the same request (float64 numpy, decode only)",
                tokens_equal_gpu=bool(ref.tokens == gpu_tokens[:len(ref.tokens)]))


def verify_workload(args) -> int:
    """Config 5: large_verify alone on the 7B-shaped large model, cache of 4096 rows, T in {1, 4, 8, 16, 32}."""
    import numpy as np

    import bild_inputs as bi
    import paper_2302_07863_amd as pkg

    pkg.lib()
    base = bi.llama_pair()
    kv = 4096
    cfg = replace(base, name="verify", small=replace(base.small, n_dec=1, name="llama-small-1"), n_src=kv + 1, max_new=40)
    t0 = time.time()
    ws, wl = bi.make_pair_weights(cfg)
    src = bi.make_source(cfg)
    log(f"[bench] verify: weights generated in {time.time() - t0:.1f}s")
    large = pkg.Model(pkg.config_from_shape(cfg.large), [wl[n] for n in bi.tensor_names(cfg.large)])
    small = pkg.Model(pkg.config_from_shape(cfg.small), [ws[n] for n in bi.tensor_names(cfg.small)])
    pair = pkg.Pair(small, large)
    n0 = len(src)
    st = pkg.State(pair, n0, n0 + 40, 31)
    t0 = time.perf_counter()
    st.encode(src)
    prefill_ms = (time.perf_counter() - t0) * 1e3
    log(f"[bench] verify: prompt of {n0} tokens prefilled in {prefill_ms:.1f} ms (both models)")
    table, t1 = [], None
    reps = max(5, args.steps)
    for T in (1, 4, 8, 16, 32):
        block = [int(t) for t in bi.make_tokens(cfg.large.vocab, T - 1, seed=300 + T)]
        st.force_tokens(n0, block, n0)
        st.probe_launch(1)                 # a run of empty kernels: separates the row counts in a profiler's dispatch list
        ms = st.bench_pass(pkg.LARGE, T, reps)
        nbytes = st.pass_bytes(pkg.LARGE, kv, T)
        flops = cfg.large.pass_flops(kv, 0, T)
        t1 = ms if T == 1 else t1
        row = dict(rows=T, ms=round(ms, 4), gbs=round(nbytes / ms / 1e6, 1), frac_hbm=round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4),
                   tflops=round(flops / ms / 1e9, 2), frac_mfma_bf16=round(flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 5),
                   sequential_ms=round(T * t1, 4), parallel_speedup=round(T * t1 / ms, 2),
                   mfma_util_counters=profile_value("verify_llama_mfma.txt", f"mfma_util_T{T}"))
        table.append(row)
        log(f"[bench] verify T={T}: {row}")
    # rollback: kv_truncate at random rows is a length write; the next pass recomputes what was cut
    rng = np.random.default_rng(5)
    cuts = [int(v) for v in rng.integers(kv - 256, kv, size=20)]
    t0 = time.perf_counter()
    for cpos in cuts:
        st.kv_truncate(pkg.LARGE, min(cpos, st.lengths()["len_large"]))
    trunc_us = (time.perf_counter() - t0) / len(cuts) * 1e6
    best = table[-1]
    out = {
        "metric": "verified rows/sec (large_verify alone, 7B-shaped large model, KV 4096)",
        "value": round(best["rows"] / best["ms"] * 1e3, 1), "unit": "rows/s", "n_gpus": 1, "steps": reps, "warmup": 1,
        "ms_per_step": best["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"verify: {cfg.large.name} alone, cache of {kv} rows, review passes of 1/4/8/16/32 rows"},
        "roofline": {"bound": "hbm", "achieved": best["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": best["frac_hbm"],
                     "traffic": None, "note": "whole 32-row pass: algorithmic bytes of the pass / its time"},
        "cpu_baseline": None,
        "verify_table": table, "prefill_ms": round(prefill_ms, 1), "kv_truncate_us": round(trunc_us, 1),
    }
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="t5", choices=["tiny", "t5", "mt5", "llama", "t5ee", "t5rel", "verify"])
    ap.add_argument("--shared-trunk", action="store_true",
                    help="early-exit workloads (tiny, t5ee): build the pair from the large model alone, so the two "
                         "models share the trunk's K/V cache and a large pass runs the upper layers only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-spread", action="store_true", help="skip the 100 single passes per pass type")
    ap.add_argument("--no-extra", action="store_true",
                    help="t5 workload: skip the second pair (mT5 shapes), whose passes the default run times as well")
    ap.add_argument("--profile-run", action="store_true",
                    help="one encode and --steps BiLD generations, nothing else: the run the rocprofv3 summaries under "
                         "profiles/ are taken from (with BILD_NO_GRAPH=1)")
    ap.add_argument("--profile-rows", type=int, default=0,
                    help="with --profile-run: instead of generations, --steps large-model passes of this many rows")
    ap.add_argument("--profile-model", choices=("small", "large"), default="large",
                    help="with --profile-rows: the model whose passes are run")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="counter-collection run: one 1 GiB device copy of known size, then --steps BiLD steps; "
                         "no timing, no JSON (run under rocprofv3 --pmc with BILD_NO_GRAPH=1)")
    ap.add_argument("--top-p", type=float, default=0.0,
                    help="> 0: the sampling variant, both models draw from the nucleus of this mass (uniform numbers "
                         "from the seeded input generator)")
    ap.add_argument("--probe-stream", action="store_true",
                    help="no benchmark: print how fast 1..256 workgroups stream private regions of 32 KiB..1 MiB "
                         "(the per-compute-unit bandwidth the launch shapes are built around)")
    ap.add_argument("--concurrent", default="2",
                    help="comma-separated counts of independent requests run at once, each on a stream of its own (an extra "
                         "figure beside the batch-1 headline; more than two only scale with GPU_MAX_HW_QUEUES above the "
                         "box's default of 4)")
    ap.add_argument("--alpha-fb", type=float, default=None)
    ap.add_argument("--alpha-rb", type=float, default=None)
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (--gpus 1); multi-GPU execution is not part of it.")
        return 2
    if args.workload == "verify":
        return verify_workload(args)

    import paper_2302_07863_amd as pkg

    pkg.lib()  # fails loudly if the HIP library has not been built
    c = setup(args.workload, args.shared_trunk, args.top_p)
    cfg, st, n0, bi = c.cfg, c.st, c.n0, c.bi
    fb = cfg.alpha_fb if args.alpha_fb is None else args.alpha_fb
    rb = cfg.alpha_rb if args.alpha_rb is None else args.alpha_rb

    if args.probe_stream:
        print("groups  KiB/group   us/launch   GB/s per group   GB/s total")
        for groups in (1, 8, 32, 64, 128, 256, 512):
            for kib in (32, 64, 128, 256, 512, 1024):
                us = st.probe_stream(groups, kib, 8)
                print(f"{groups:6d} {kib:10d} {us:11.2f} {kib * 1.024 / us * 1e0:16.1f} {groups * kib * 1.024 / us:12.1f}", flush=True)
        print(f"empty launch: {st.probe_launch(2000):.2f} us")
        return 0

    if args.pmc_probe or args.profile_run:
        st.gemm_tally(reset=True)          # count the decode GEMMs only (the encoder's row-block GEMMs are another kernel)
        if args.pmc_probe:
            st.probe_copy(1 << 30, 3)      # bild::probe_copy_kernel: reads 1 GiB and writes 1 GiB per launch
        st.probe_launch(200)               # bild::probe_empty_kernel: what a launch that does nothing costs
        if args.profile_rows > 0:
            toks, _ = st.generate(None, fb, rb, cfg.max_new)
            ln = st.lengths()
            which = pkg.SMALL if args.profile_model == "small" else pkg.LARGE
            have = ln["len_small"] if which == pkg.SMALL else ln["len_large"]
            st.kv_truncate(which, min(have, ln["y_len"] - args.profile_rows))
            st.bench_pass(which, args.profile_rows, args.steps)
        else:
            for _ in range(args.steps):
                st.seq_truncate(n0)
                st.generate(None, fb, rb, cfg.max_new)
        tally = st.gemm_tally()
        log(f"[bench] profile run done: gemm launches issued {tally['launches']}, algorithmic weight bytes "
            f"{tally['bytes']}, mean {tally['bytes'] / max(tally['launches'], 1):.0f} B/launch")
        return 0

    toks, stats, dt = time_generation(c, fb, rb, args.steps, args.warmup)
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
    st.seq_truncate(n0)
    toks, stats = st.generate(None, fb, rb, cfg.max_new)
    passes = time_passes(c, not args.no_spread)

    roofline = roofline_leg(c, fb, rb, stats)
    st.seq_truncate(n0)
    toks, stats = st.generate(None, fb, rb, cfg.max_new)
    log(f"[bench] roofline {roofline}")

    # The third line of the report: these passes are chains of dependent stages, so beside the bandwidth roofline stands
    # stage count x the cost of a launch that does nothing.
    launch_us = st.probe_launch(2000)

    # kernel launches of a single-row pass as the library issues them (embedding, layer pieces, LM head, policy)
    n_small = roofline["stages_per_pass"]["small"]
    n_large = roofline["stages_per_pass"].get("large_1")
    if n_large is None:
        uncov = st.lengths()
        st.kv_truncate(pkg.LARGE, min(uncov["len_large"], uncov["y_len"] - 1))
        st.bench_gemm(pkg.LARGE, 1, 1)
        n_large = st.pass_stages()
    stage_latency = dict(empty_launch_us=round(launch_us, 3),
                         small_pass=dict(stages=n_small, launch_floor_ms=round(n_small * launch_us * 1e-3, 4),
                                         measured_ms=passes["small_step"]["ms"]),
                         large_pass=dict(stages=n_large, launch_floor_ms=round(n_large * launch_us * 1e-3, 4),
                                         measured_ms=passes["large_step"]["ms"]))
    log(f"[bench] stage latency {stage_latency}")

    # several independent requests at once (one state and one stream each): what the chip delivers when it is not left
    # waiting for one request's chain of dependent stages
    concurrent = None
    if not args.no_extra:
        concurrent = {f"x{n}": concurrent_leg(c, fb, rb, n, max(2, args.steps // 4), toks) for n in [int(v) for v in args.concurrent.split(",") if v]}
        log(f"[bench] concurrent requests {concurrent}")

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(c, fb, rb, args.top_p, toks)
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
        "config": {"workload": f"{cfg.name}: {cfg.small.name}+{cfg.large.name}, src {len(c.src)} tokens, "
                               f"{cfg.max_new} new tokens, alpha_FB={fb}, alpha_RB={rb}, n_max={cfg.n_max}"
                               + (", shared trunk (early-exit pair)" if args.shared_trunk else "")
                               + (f", nucleus sampling top_p={args.top_p}" if args.top_p > 0 else ""),
                   "tokens_per_step": n_tok},
        "roofline": roofline,
        # matrix-core utilisation of the review GEMMs by row count (config 5: 7B-shaped large model, cache of 4096 rows), read
        # from the committed rocprofv3 counter summary (profiles/verify_llama_mfma.txt; `--workload verify` times the same passes)
        "mfma_util_verify_gemm": {f"T{T}": profile_value("verify_llama_mfma.txt", f"mfma_util_T{T}") for T in (1, 4, 8, 16, 32)},
        "stage_latency": stage_latency,
        "cpu_baseline": cpu,
        "bild_stats": stats,
        "large_only_tokens_per_s": round(large_tok_s, 2),
        "speedup_vs_large_only": round(tok_s / large_tok_s, 3),
        "encode_ms": round(c.encode_ms, 2),
        # per request, the paper's "end-to-end latency per example": encode (or prompt prefill) + generation
        "end_to_end_tokens_per_s": round(n_tok / (c.encode_ms * 1e-3 + dt / args.steps), 2),
        "passes": passes,
        # not the headline metric (that is one request at batch 1): aggregate tokens/s of 2 and 3 independent requests
        # running at once on streams of their own
        "concurrent_requests": concurrent,
    }

    # The bandwidth target is stated on the T5-large AND the mT5-large shapes: the default run also times the passes
    # (and a few generations) of the mT5-shaped pair.
    if args.workload == "t5" and not args.no_extra:
        st.close()
        c.pair.close()
        del c, st
        m = setup("mt5")
        mt, ms_, mdt = time_generation(m, m.cfg.alpha_fb, m.cfg.alpha_rb, 5, 2)
        mg_reps = 2
        m.st.seq_truncate(m.n0)
        m.st.greedy(pkg.LARGE, None, m.cfg.max_new)
        t0 = time.perf_counter()
        for _ in range(mg_reps):
            m.st.seq_truncate(m.n0)
            g = m.st.greedy(pkg.LARGE, None, m.cfg.max_new)
        m_large = mg_reps * len(g) / (time.perf_counter() - t0)
        m.st.seq_truncate(m.n0)
        m.st.generate(None, m.cfg.alpha_fb, m.cfg.alpha_rb, m.cfg.max_new)
        out["passes_mt5"] = time_passes(m, False)
        out["mt5"] = dict(workload=f"mt5: {m.cfg.small.name}+{m.cfg.large.name}, src {len(m.src)} tokens, {m.cfg.max_new} new tokens",
                          tokens_per_s=round(5 * len(mt) / mdt, 2), large_only_tokens_per_s=round(m_large, 2),
                          speedup_vs_large_only=round(5 * len(mt) / mdt / m_large, 3), bild_stats=ms_,
                          encode_ms=round(m.encode_ms, 2))
        log(f"[bench] mt5 {out['mt5']}")
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
