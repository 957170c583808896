#!/usr/bin/env python3
"""Benchmark of the shared-attention decoder step on one MI355X.

A "step" is one pass of the whole hot path over all batch*beam rows:
san_decode_step (embedding, every decoder layer under the sharing policy, output
layer) + san_topk + san_beam_reorder, on the Transformer-base workload (64
sentences x beam 4, source lengths U[20,60], 64 decode steps per sentence batch,
fp32, self-attention shared in pairs, enc-dec attention in groups of 3), inputs and
weights resident in HBM, the encoder run once beforehand.

What is timed.  The cost of a step grows with the number of cached positions, so a
timed window must see the same mix of cache lengths as a whole decode:
  --steps K >= 64 : K is rounded down to whole decodes (the cache grows 1..64 in each);
  --steps K <  64 : the K positions in the middle of a decode, (64-K)/2 .. (64+K)/2 - 1,
                    whose mean cache length is the decode's; the run-up to the first of
                    them is not timed.
The window is timed REPS times (11 by default), each bracketed by device
synchronisations, and the median is reported; `steps` stays K.  Every comparison leg
(unshared, mode S, un-cached ...) is timed over the same positions.

Prints ONE JSON line: metric/value (decoded tokens/s over batch*beam rows), the
roofline of the dominant attention kernel (HIP events on the library's stream,
second identical pass; next to it the rocprofv3 figures kept under profiles/), the
same kernels under the unshared / share-S / un-cached configurations, a short leg for
each of the other workloads (long, big, aan), and the CPU oracle timed on the host
cores over the same window.
"""
import argparse
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
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--reps", type=int, default=11, help="how often the timed window is repeated (median reported)")
    ap.add_argument("--config", default="base", choices=["tiny", "base", "big", "long", "aan"])
    ap.add_argument("--no-compare", action="store_true", help="skip the unshared / share-S / un-cached runs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--no-configs", action="store_true", help="skip the short legs on the other workloads")
    ap.add_argument("--cpu-steps", type=int, default=20,
                    help="decode steps the CPU oracle is timed on (the middle of a decode, like a short GPU window)")
    ap.add_argument("--beam-sweep", default="", help="comma-separated beam sizes: also time SAN vs unshared "
                    "cached decoding at these beams (the paper's Fig. 5 axis), e.g. 4,8,12,16,20")
    ap.add_argument("--loop-only", default="", choices=["", "eager", "graph", "logits"],
                    help="time only whole decodes driven by san_decode_n (eager, replayed HIP graph, or graph with "
                         "SAN_LOOP_LOGITS) and print a short JSON line: the command kernel traces of the loop use")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a kernel of known "
                         "traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def window_of(T, steps):
    """(first position, number of steps, text) of the timed window, see the module docstring."""
    if steps >= T:
        k = (steps // T) * T
        return 0, k, f"{k // T} whole decode(s): positions 0-{T - 1} of {T}, {k // T} time(s) per repetition"
    p0 = (T - steps) // 2
    return p0, steps, f"positions {p0}-{p0 + steps - 1} of {T} (the middle of a decode: its mean cache length)"


class Runner:
    """Device-resident decode loop: no host synchronisation inside."""

    def __init__(self, torch, gpu, cfg, src, lens):
        self.torch, self.gpu, self.cfg = torch, gpu, cfg
        self.batch, self.beam, self.T = cfg["batch"], cfg["beam"], cfg["steps"]
        B, V = self.batch * self.beam, cfg["V"]
        self.B = B
        dev = "cuda"
        self.src = torch.from_numpy(src).to(dev)
        self.len = torch.from_numpy(lens).to(dev)
        self.logits = torch.empty((B, V), dtype=torch.float32, device=dev)
        self.bos = torch.full((B,), 1, dtype=torch.int32, device=dev)
        cum0 = torch.full((B,), float("-inf"), dtype=torch.float32, device=dev)
        cum0[0::self.beam] = 0.0
        self.cum0 = cum0
        # two sets of beam-step outputs: step s reads set s-1 and writes set s
        self.tok = [torch.empty((self.batch, self.beam), dtype=torch.int32, device=dev) for _ in range(2)]
        self.par = [torch.empty((self.batch, self.beam), dtype=torch.int32, device=dev) for _ in range(2)]
        self.sc = [torch.empty((self.batch, self.beam), dtype=torch.float32, device=dev) for _ in range(2)]
        gpu.encode(self.src, self.len)
        self.pos = 0

    def steps(self, k):
        g = self.gpu
        for _ in range(k):
            if self.pos == 0:
                g.rewind()
                tokens, cum = self.bos, self.cum0
            else:
                i = (self.pos - 1) & 1
                tokens, cum = self.tok[i].view(-1), self.sc[i].view(-1)
            o = self.pos & 1
            g.decode_step(tokens, self.logits)
            g.topk(self.logits, cum, self.beam, self.tok[o], self.par[o], self.sc[o])
            g.beam_reorder(self.par[o].view(-1))
            self.pos = (self.pos + 1) % self.T

    def window(self, p0, k, reps, warmup=0):
        """Median wall time of the k steps that start at position p0 of a decode, over `reps`
        repetitions; each repetition starts from a rewound decoder and runs up to p0 untimed."""
        torch = self.torch
        self.pos = 0
        self.steps(warmup)
        times = []
        for _ in range(reps):
            self.pos = 0
            self.steps(p0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.steps(k)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
        times.sort()
        return times[len(times) // 2], times


def loop_leg(torch, make_gpu, cfg, src, lens, use_graph, keep_logits, reps=5):
    """ms per whole decode driven by san_decode_n: one host call per decode on a stream of its own
    (the NULL stream cannot be captured); median of `reps` after one untimed decode."""
    import numpy as np
    T, B = cfg["steps"], cfg["batch"] * cfg["beam"]
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        g = make_gpu()
        r = Runner(torch, g, cfg, src, lens)
        o_tok = torch.zeros((T, B), dtype=torch.int32, device="cuda")
        o_par = torch.zeros((T, B), dtype=torch.int32, device="cuda")

        def one_decode():
            g.rewind()
            cum = r.cum0.clone()
            g.decode_n(T, r.bos, cum, o_tok, o_par, r.logits, use_graph, keep_logits=keep_logits)

        one_decode()
        st.synchronize()
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            one_decode()
            st.synchronize()
            ts.append(time.perf_counter() - t0)
        g.close()
        del r
    return float(np.median(ts))


def ragged_finish(torch, gpu, cfg, src, lens, compact, reps=3):
    """Wall time of one decode in which sentence b is taken to end after
    T/2 + b*T/(2*batch) steps (a mix of lengths; the synthetic weights never emit the
    end symbol themselves).  compact: at every 8th step the sentences past their end
    leave the batch (san_compact); otherwise they ride along to the last step, as in a
    fixed batch.  Returns (seconds per decode, useful row-steps per decode)."""
    import numpy as np
    batch, beam, T, V = cfg["batch"], cfg["beam"], cfg["steps"], cfg["V"]
    B = batch * beam
    end = T // 2 + (np.arange(batch) * (T - T // 2)) // batch + 1          # steps sentence b needs
    src_d, len_d = torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda()
    logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
    bos = torch.full((B,), 1, dtype=torch.int32, device="cuda")
    cum0 = torch.full((B,), float("-inf"), dtype=torch.float32, device="cuda")
    cum0[0::beam] = 0.0
    gpu.encode(src_d, len_d)
    times = []
    for rep in range(reps + 1):
        gpu.rewind()
        alive = np.arange(batch)
        tokens, cum = bos, cum0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(T):
            if compact and s and s % 8 == 0:
                keep = np.nonzero(end[alive] > s)[0]
                if len(keep) < len(alive):
                    gpu.compact(keep)
                    rows = torch.from_numpy((keep[:, None] * beam + np.arange(beam)[None, :]).reshape(-1)).cuda()
                    tokens, cum = tokens[rows].contiguous(), cum[rows].contiguous()
                    alive = alive[keep]
            nb = len(alive)
            o_tok = torch.empty((nb, beam), dtype=torch.int32, device="cuda")
            o_par = torch.empty((nb, beam), dtype=torch.int32, device="cuda")
            o_sc = torch.empty((nb, beam), dtype=torch.float32, device="cuda")
            gpu.decode_step(tokens, logits)
            gpu.topk(logits, cum, beam, o_tok, o_par, o_sc)
            gpu.beam_reorder(o_par.view(-1))
            tokens, cum = o_tok.view(-1), o_sc.view(-1)
        torch.cuda.synchronize()
        if rep:
            times.append(time.perf_counter() - t0)
    return float(np.median(times)), int(end.sum()) * beam


def attention_bytes(cfg, esz, heads_self, followers_self, heads_ctx, s_followers_ctx, mean_src):
    """Algorithmic bytes of the attention kernels, summed over one decode of T
    steps: a block head streams K and V of the n cached positions of every row, a
    follower only V; an enc-dec head streams the sentence's memory K and V once per
    sentence."""
    B, d, T = cfg["batch"] * cfg["beam"], cfg["d"], cfg["steps"]
    sum_n = T * (T + 1) // 2
    self_head = 2 * B * d * esz * sum_n * heads_self
    self_apply = 1 * B * d * esz * sum_n * followers_self
    ctx_head = 2 * cfg["batch"] * mean_src * d * esz * T * heads_ctx
    ctx_apply = 1 * cfg["batch"] * mean_src * d * esz * T * s_followers_ctx
    return {"attn_self": self_head, "attn_apply": self_apply, "attn_ctx": ctx_head, "attn_ctx_apply": ctx_apply}


def gemm_flops_per_step(cfg, heads_self, followers_self, heads_ctx):
    B, d, F, V, Ld = cfg["batch"] * cfg["beam"], cfg["d"], cfg["F"], cfg["V"], cfg["n_dec"]
    proj = 2 * B * d * d * (3 * heads_self + followers_self + heads_ctx)
    out = 2 * B * d * d * 2 * Ld
    ffn = 2 * B * d * F * 2 * Ld
    logits = 2 * B * d * V
    return {"proj": proj, "out": out, "ffn": ffn, "logits": logits}


def step_roofline(cfg, esz, self_pi, ctx_pi, mean_src, ms_per_step):
    """What one decode step has to move and multiply under the sharing policy, each needed
    weight once, each live cache element once per layer that uses it (average over the T
    steps), memory K/V once per sentence, logits written and read once: the step-level
    HBM and MFMA bounds next to the measured step."""
    B, batch, d, F, V, Ld, T = (cfg["batch"] * cfg["beam"], cfg["batch"], cfg["d"], cfg["F"], cfg["V"], cfg["n_dec"],
                                cfg["steps"])
    aan = cfg["self_kind"] == "aan"
    hs, fs = (0, 0) if aan else (len(self_pi), sum(self_pi) - len(self_pi))
    hc, fc = len(ctx_pi), sum(ctx_pi) - len(ctx_pi)
    n_mean = (T + 1) / 2
    w_elems = (4 * hs + 2 * fs) * d * d + (2 * hc + fc) * d * d + Ld * 2 * d * F + V * d
    state = (2 * hs + fs) * B * n_mean * d * esz + (2 * hs + fs) * B * d * esz            # cache reads + appends
    if aan:
        w_elems += Ld * (2 * d * F + 4 * d * d)
        state = Ld * 2 * B * d * 4                                                        # running sums, read + write
    mem = hc * 2 * batch * mean_src * d * esz
    logits = 2 * B * V * 4
    total = w_elems * esz + state + mem + logits
    flops = 2 * B * ((3 * hs + fs + hs + fs) * d * d + (2 * hc + fc) * d * d + Ld * 2 * d * F + V * d)
    if aan:
        flops += 2 * B * Ld * (2 * d * F + 4 * d * d)
    hbm_us = total / (HBM_PEAK_GBS * 1e9) * 1e6
    mfma_us = flops / (MFMA_PEAK_TFLOPS[cfg["dtype"]] * 1e12) * 1e6
    bound = max(hbm_us, mfma_us)
    return {"algorithmic_MB": total / 1e6, "weights_MB": w_elems * esz / 1e6, "state_MB": state / 1e6,
            "memory_kv_MB": mem / 1e6, "logits_MB": logits / 1e6, "hbm_us_at_peak": hbm_us,
            "gemm_GFLOP": flops / 1e9, "mfma_us_at_peak": mfma_us, "bound": "hbm" if hbm_us >= mfma_us else "mfma",
            "bound_us": bound, "measured_us": ms_per_step * 1e3, "frac": bound / (ms_per_step * 1e3)}


def profiled_figures(config, key):
    """The rocprofv3 figures kept under profiles/ for this workload's dominant kernel: average
    duration from the --kernel-trace summary, HBM bytes per launch from the two --pmc
    summaries.  They come from earlier runs of this same command under the profiler, NOT from
    this run; absent files or lines give None."""
    role = {"attn_self": "head", "attn_ctx": "ctx", "attn_apply": "apply"}[key]
    out = {"rocprofv3_avg_us": None, "rocprofv3_source": None, "fetch_MB": None, "write_MB": None,
           "traffic_source": None}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"attention_and_step_kernels_{config}*.txt"))):
        for line in open(path):
            m = re.match(rf"{role}\s+all steps: avg ([0-9.]+) us per launch", line)
            if m:
                out["rocprofv3_avg_us"] = float(m.group(1))
                out["rocprofv3_source"] = "profiles/" + os.path.basename(path)
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"attention_hbm_traffic_{config}*.txt"))):
        counter = None
        for line in open(path):
            m = re.match(r"(FETCH_SIZE|WRITE_SIZE):", line)
            if m:
                counter = m.group(1)
            m = re.match(rf"attention {role}\s*:.*->\s*([0-9.]+) MB per launch", line)
            if m and counter:
                out["fetch_MB" if counter == "FETCH_SIZE" else "write_MB"] = float(m.group(1))
                out["traffic_source"] = "profiles/" + os.path.basename(path)
    return out


def kernel_pass(torch, gpu, run, cfg, esz, mean_src, config_name):
    """Second, identical pass over one decode with every launch bracketed by event markers on
    the library's stream.  A marker pair costs about 2 us of stream time per launch; that cost
    is estimated as (sum of bracketed times - unmarked wall time of the same decode) / launches
    and taken off every launch, so that the per-kernel figures add up to the unmarked step time
    (the decode is GPU-bound: kernels run back to back).  rocprofv3 --kernel-trace gives the
    same per-kernel averages (profiles/)."""
    T = cfg["steps"]
    wall_T, _ = run.window(0, T, 3)          # unmarked time of exactly one decode
    run.pos = 0
    gpu.profile(True)
    gpu.profile_read(reset=True)
    run.steps(T)
    prof = gpu.profile_read(reset=True)
    gpu.profile(False)
    raw_ms = sum(ms for ms, n in prof.values())
    n_pairs = sum(n for ms, n in prof.values())
    marker_us = max(0.0, (raw_ms - wall_T * 1e3) / n_pairs * 1e3)
    prof = {k: (max(ms - n * marker_us * 1e-3, 0.0), n) for k, (ms, n) in prof.items()}
    aan = cfg["self_kind"] == "aan"
    hs, fs = (0, 0) if aan else (len(cfg["self_pi"]), sum(cfg["self_pi"]) - len(cfg["self_pi"]))
    hc = len(cfg["encdec_pi"])
    ab = attention_bytes(cfg, esz, hs, fs, hc, 0, mean_src)
    gf = gemm_flops_per_step(cfg, hs, fs, hc)
    kernels = {}
    for k, (ms, n) in prof.items():
        if n == 0:
            continue
        ent = {"ms_per_step": ms / T, "launches_per_step": n / T, "avg_us": ms / n * 1e3}
        if k in ab and ab[k] > 0:
            ent["algo_GBps"] = ab[k] / (ms * 1e-3) / 1e9
            ent["frac_hbm_peak"] = ent["algo_GBps"] / HBM_PEAK_GBS
        if k in gf:
            ent["TFLOPs"] = gf[k] * T / (ms * 1e-3) / 1e12
            ent["frac_mfma_peak"] = ent["TFLOPs"] / MFMA_PEAK_TFLOPS[cfg["dtype"]]
        kernels[k] = ent
    key = "attn_ctx" if aan else "attn_self"
    ms, n = prof[key]
    achieved = ab[key] / (ms * 1e-3) / 1e9
    pf = profiled_figures(config_name, key)
    traffic = None
    if pf["fetch_MB"] is not None and pf["write_MB"] is not None:
        traffic = (pf["fetch_MB"] + pf["write_MB"]) * 1e6
    roofline = {"kernel": "attention_kernel (block-head " + ("enc-dec" if aan else "self") + " attention)",
                "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_note": "HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE runs of this command "
                                "kept under profiles/ (not measured in this run)" if traffic else
                                "no counter run of this workload is kept under profiles/: unmeasured",
                "traffic_source": pf["traffic_source"],
                "bytes_per_launch": ab[key] / n, "avg_launch_us": ms / n * 1e3, "launches": n,
                "event_marker_us_removed_per_launch": marker_us,
                "rocprofv3_avg_launch_us": pf["rocprofv3_avg_us"], "rocprofv3_source": pf["rocprofv3_source"]}
    if traffic:
        roofline["counter_GBps"] = traffic / (ms / n * 1e-3) / 1e9     # what actually left / entered HBM
    if pf["rocprofv3_avg_us"]:
        roofline["frac_by_rocprofv3"] = ab[key] / n / (pf["rocprofv3_avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS
    return kernels, roofline


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "decoding shards by sentence (independent replicas, no communication)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_1906_11024_amd import binding as sb
    from paper_1906_11024_amd import workloads as wl

    if not os.path.exists(sb.LIB_PATH):
        from paper_1906_11024_amd import build
        build.build(verbose=False)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    lib_state = sb.lib_state()

    cfg = wl.get_config(args.config)
    T = cfg["steps"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    weights = wl.make_weights(cfg, seed=0)
    blob = wl.pack_weights(cfg, weights)
    src, lens = wl.make_source(cfg, 0)
    mean_src = float(lens.mean())
    B = cfg["batch"] * cfg["beam"]

    def make(self_pi, ctx_pi, share=sb.SAN_SHARE_A, use_cache=1):
        sc = sb.make_config(cfg, encdec_share=share, use_cache=use_cache)
        return sb.San(sc, blob, self_pi, ctx_pi)

    if args.loop_only:
        w = loop_leg(torch, lambda: make(cfg["self_pi"], cfg["encdec_pi"]), cfg, src, lens,
                     args.loop_only != "eager", args.loop_only == "logits", reps=max(1, args.reps))
        print(json.dumps({"metric": "decoded tokens/sec (batch x beam rows per step), san_decode_n", "value": B * T / w,
                          "unit": "tokens/s", "ms_per_step": w / T * 1e3, "steps": T, "mode": args.loop_only,
                          "config": {"workload": args.config}, "lib_source_hash": lib_state["built_from"]}))
        return

    # ------------------------------------------------ headline: SAN policy, cached
    p0, K, window_text = window_of(T, args.steps)
    gpu = make(cfg["self_pi"], cfg["encdec_pi"])
    run = Runner(torch, gpu, cfg, src, lens)
    wall, walls = run.window(p0, K, max(1, args.reps), args.warmup)
    tok_per_s = B * K / wall
    ms_per_step = wall / K * 1e3
    launches = gpu.last_launch_count

    # ------------------------------------------------ per-kernel pass (HIP events)
    kernels, roofline = {}, None
    if not args.no_profile:
        kernels, roofline = kernel_pass(torch, gpu, run, cfg, esz, mean_src, args.config)
    # ------------------------------------------------ latency, encode time, streaming-read yardstick
    # (after the timed region; each of these synchronises per call, the headline loop does not)
    extras = {"step_roofline": step_roofline(cfg, esz, cfg["self_pi"], cfg["encdec_pi"], mean_src, ms_per_step)}
    if not args.no_profile:
        lat = []
        run.pos = 0
        torch.cuda.synchronize()
        for _ in range(2 * T):
            t0 = time.perf_counter()
            run.steps(1)
            torch.cuda.synchronize()
            lat.append((time.perf_counter() - t0) * 1e3)
        lat = np.sort(np.asarray(lat[T:]))           # second decode: warmed up
        extras["step_latency_ms_synchronised"] = {"mean": float(lat.mean()), "p50": float(lat[len(lat) // 2]),
                                                  "p99": float(lat[min(len(lat) - 1, int(0.99 * len(lat)))])}
        enc = []
        for _ in range(5):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            gpu.encode(run.src, run.len)
            torch.cuda.synchronize()
            enc.append((time.perf_counter() - t0) * 1e3)
        extras["encode_ms"] = float(np.median(enc))
        if roofline is not None:
            # plain read kernel over a buffer of the dominant kernel's average size, and over 1 GiB
            for label, nbytes in (("launch_sized", int(roofline["bytes_per_launch"])), ("1GiB", 1 << 30)):
                buf = torch.empty(nbytes // 4, dtype=torch.int32, device="cuda").zero_()
                for _ in range(3):
                    gpu.stream_read(buf)
                torch.cuda.synchronize()
                reps = 50 if nbytes < (1 << 28) else 5
                t0 = time.perf_counter()
                for _ in range(reps):
                    gpu.stream_read(buf)
                torch.cuda.synchronize()
                w = (time.perf_counter() - t0) / reps
                roofline["plain_read_" + label] = {"bytes": buf.numel() * 4, "us": w * 1e6, "GBps": buf.numel() * 4 / w / 1e9}
                del buf
    gpu.close()
    del run

    # ------------------------------------------------ same kernels, other policies, same positions
    compare = {}
    if not args.no_compare:
        Ld = cfg["n_dec"]
        aan = cfg["self_kind"] == "aan"
        variants = [("unshared_cached", [1] * Ld, [1] * Ld, sb.SAN_SHARE_A, 1)]
        if not aan:
            variants.append(("san_share_s", cfg["self_pi"], cfg["encdec_pi"], sb.SAN_SHARE_S, 1))
            if Ld == 6:
                # the uniform policy of Sec. 4.2: one self-attention block over the stack, enc-dec {3,3}
                variants.append(("san_uniform_policy", [6], [3, 3], sb.SAN_SHARE_A, 1))
        variants.append(("san_no_cache", cfg["self_pi"], cfg["encdec_pi"], sb.SAN_SHARE_A, 0))
        variants.append(("unshared_no_cache", [1] * Ld, [1] * Ld, sb.SAN_SHARE_A, 0))
        # the comparison legs run at most two decodes per repetition (the un-cached ones: one)
        for name, spi, cpi, share, cache in variants:
            k_leg = K if K < T else (min(K, 2 * T) if cache else T)
            g = make(spi, cpi, share, cache)
            r = Runner(torch, g, cfg, src, lens)
            w, _ = r.window(p0, k_leg, 5 if cache else 3, T if cache else 0)
            compare[name] = {"tokens_per_s": B * k_leg / w, "ms_per_step": w / k_leg * 1e3, "steps": k_leg,
                             "first_position": p0, "kernels_per_step": g.last_launch_count,
                             "weight_MB": g.device_bytes(0) / 1e6, "state_MB": g.device_bytes(1) / 1e6}
            g.close()
            del r
        # the same decode driven by san_decode_n: one host call per decode, pairs of
        # steps replayed from a captured HIP graph (own stream: the NULL stream cannot be captured)
        # (default: the output layer hands the search per-tile candidates; *_logits: SAN_LOOP_LOGITS, the
        # logits are stored and read back as in the separate calls)
        for name, use_graph, keep in (("san_decode_n_eager", False, False), ("san_decode_n_graph", True, False),
                                      ("san_decode_n_graph_logits", True, True)):
            w = loop_leg(torch, lambda: make(cfg["self_pi"], cfg["encdec_pi"]), cfg, src, lens, use_graph, keep)
            compare[name] = {"tokens_per_s": B * T / w, "ms_per_step": w / T * 1e3, "steps": T,
                             "window": "one whole decode per repetition, median of 5"}
        # sentences of different lengths: finished ones leave the batch (san_compact) or ride along
        rf = {}
        for name, cmpct in (("fixed_batch", False), ("compacting", True)):
            g = make(cfg["self_pi"], cfg["encdec_pi"])
            w, useful = ragged_finish(torch, g, cfg, src, lens, cmpct)
            rf[name] = {"ms_per_decode": w * 1e3, "useful_tokens_per_s": useful / w}
            g.close()
        rf["speedup"] = rf["fixed_batch"]["ms_per_decode"] / rf["compacting"]["ms_per_decode"]
        rf["schedule"] = "sentence b ends after T/2 + b*T/(2*batch) steps; the batch is compacted every 8 steps"
        compare["ragged_finish"] = rf
        compare["san_cached"] = {"tokens_per_s": tok_per_s, "ms_per_step": ms_per_step, "steps": K, "first_position": p0}
        compare["positions"] = "every leg above san_decode_n_* is timed over the same positions as the headline " \
                               "(whole decodes when the headline is whole decodes)"
        compare["speedup_san_vs_unshared_cached"] = tok_per_s / compare["unshared_cached"]["tokens_per_s"]
        if "unshared_no_cache" in compare:
            compare["speedup_san_vs_unshared_no_cache"] = tok_per_s / compare["unshared_no_cache"]["tokens_per_s"]
            compare["speedup_cache_vs_no_cache_unshared"] = (compare["unshared_cached"]["tokens_per_s"]
                                                             / compare["unshared_no_cache"]["tokens_per_s"])

    # ------------------------------------------------ the other workloads, one short leg each
    configs = {}
    if not args.no_configs and args.config == "base":
        for name in ("long", "big", "aan"):
            c2 = wl.get_config(name)
            e2 = 2 if c2["dtype"] == "bf16" else 4
            w2 = wl.make_weights(c2, seed=0)
            blob2 = wl.pack_weights(c2, w2)
            del w2
            src2, lens2 = wl.make_source(c2, 0)
            g = sb.San(sb.make_config(c2), blob2, c2["self_pi"], c2["encdec_pi"])
            del blob2
            r = Runner(torch, g, c2, src2, lens2)
            T2, B2 = c2["steps"], c2["batch"] * c2["beam"]
            w, _ = r.window(0, T2, 3, T2)            # one whole decode per repetition
            ent = {"workload": f"transformer-{name}: batch {c2['batch']} x beam {c2['beam']}, {T2} decode steps, "
                               f"{c2['dtype']}, self policy {c2['self_pi'] if c2['self_kind'] != 'aan' else 'AAN'}, "
                               f"enc-dec policy {c2['encdec_pi']}",
                   "window": f"one whole decode (positions 0-{T2 - 1}) per repetition, median of 3",
                   "tokens_per_s": B2 * T2 / w, "ms_per_step": w / T2 * 1e3, "kernels_per_step": g.last_launch_count,
                   "dtype": c2["dtype"]}
            ks, rl = kernel_pass(torch, g, r, c2, e2, float(lens2.mean()), name)
            ent["roofline"] = rl
            ent["kernels"] = {k: v for k, v in ks.items() if k.startswith("attn") or k in ("logits", "ffn", "proj", "out")}
            ent["step_roofline"] = step_roofline(c2, e2, c2["self_pi"], c2["encdec_pi"], float(lens2.mean()), w / T2 * 1e3)
            g.close()
            del r
            blob2 = wl.pack_weights(c2, wl.make_weights(c2, seed=0))
            wl_ = loop_leg(torch, lambda: sb.San(sb.make_config(c2), blob2, c2["self_pi"], c2["encdec_pi"]), c2, src2,
                           lens2, False, False, reps=3)
            del blob2
            ent["san_decode_n"] = {"ms_per_step": wl_ / T2 * 1e3, "tokens_per_s": B2 * T2 / wl_,
                                   "window": "one whole decode per host call, median of 3"}
            torch.cuda.empty_cache()
            configs[name] = ent

    # ------------------------------------------------ beam-size sweep (Fig. 5 axis)
    beam_sweep = {}
    if args.beam_sweep:
        Ld = cfg["n_dec"]
        for bm in [int(v) for v in args.beam_sweep.split(",")]:
            c2 = dict(cfg, beam=bm)
            ent = {}
            for name, spi, cpi in (("san", cfg["self_pi"], cfg["encdec_pi"]), ("unshared", [1] * Ld, [1] * Ld)):
                g = sb.San(sb.make_config(c2), blob, spi, cpi)
                r = Runner(torch, g, c2, src, lens)
                w, _ = r.window(0, 2 * T, 3, T)
                ent[name] = {"tokens_per_s": c2["batch"] * bm * 2 * T / w, "sentence_tokens_per_s": c2["batch"] * 2 * T / w,
                             "ms_per_step": w / (2 * T) * 1e3}
                g.close()
                del r
            ent["speedup"] = ent["san"]["tokens_per_s"] / ent["unshared"]["tokens_per_s"]
            beam_sweep[str(bm)] = ent

    # ------------------------------------------------ CPU oracle on the host cores
    cpu = None
    if not args.no_cpu:
        from oracle import san_oracle as so
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        orc = so.SanOracle(cfg, weights, cfg["self_pi"], cfg["encdec_pi"])
        orc.encode(src, lens)
        ksteps = min(args.cpu_steps, T)
        c0 = (T - ksteps) // 2                       # the middle of a decode, as the GPU's short window
        tokens = np.full(B, 1, dtype=np.int64)
        cum = np.full(B, -np.inf)
        cum[0::cfg["beam"]] = 0.0
        t0 = None
        for s in range(c0 + ksteps):
            if s == c0:
                t0 = time.perf_counter()
            lg = orc.decode_step(tokens)
            tk, par, sc, _ = orc.topk(lg, cum, cfg["beam"])
            orc.beam_reorder(par.reshape(-1))
            tokens, cum = tk.reshape(-1).astype(np.int64), sc.reshape(-1)
        cw = time.perf_counter() - t0
        cpu = {"value": B * ksteps / cw, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"positions {c0}-{c0 + ksteps - 1} of the {T} decode steps of the same batch ({cfg['batch']} "
                         f"sentences x beam {cfg['beam']}; mean cache length = the decode's), the oracle as it stands "
                         f"(numpy fp64, BLAS threads = cores); the {c0} steps before them run untimed",
               "ms_per_step": cw / ksteps * 1e3}

    if args.calib_copy_mb:
        n = args.calib_copy_mb * (1 << 20) // 4
        a = torch.ones(n, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    out = {
        "metric": "decoded tokens/sec (batch x beam rows per step)", "value": tok_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"transformer-{args.config}: {cfg['n_enc']}+{cfg['n_dec']} layers, d={cfg['d']}, "
                               f"H={cfg['H']}, d_ff={cfg['F']}, vocab={cfg['V']}, batch {cfg['batch']} x beam "
                               f"{cfg['beam']}, src len U{list(cfg['src_len'])}, {T} decode steps, cached, "
                               f"self policy {cfg['self_pi']}, enc-dec policy {cfg['encdec_pi']} (share A); "
                               f"timed window: {window_text}",
                   "window_first_position": p0, "window_steps": K, "repetitions": len(walls),
                   "ms_per_step_min_max": [min(walls) / K * 1e3, max(walls) / K * 1e3],
                   "rows": B, "kernels_per_step": launches,
                   "sentence_tokens_per_s": cfg["batch"] * K / wall,
                   "lib_source_hash": lib_state["built_from"], "lib_stale": lib_state["stale"]},
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "compare": compare, **extras,
    }
    if configs:
        out["configs"] = configs
    if beam_sweep:
        out["beam_sweep"] = beam_sweep
    print(json.dumps(out))


if __name__ == "__main__":
    main()
