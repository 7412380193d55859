#!/usr/bin/env python3
"""Throughput of the predictive delta-coding path on one MI355X.

One step = one pass of the whole path over a synthetic KV cache that is already
resident in HBM: encode (predict/residual/quantise, histogram, frequency tables,
rANS encode) followed by decode (rANS decode, reconstruct).  The headline value is
GB/s of fp16 KV pushed through that round trip on the largest configuration (64
sessions); the other four configurations are timed the same way and reported in
the same JSON line under `configs`.  Prints ONE JSON line on stdout; per-kernel
tables go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak
ALL_CONFIGS = ("tiny", "llama8b", "long", "70b", "batched")
GROUP_MIN_STREAMS = 2048   # streams a group holds at least when a cache is coded as independent groups (codec.GroupedCodec)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="batched", help="headline workload: tiny | llama8b | long | 70b | batched | miss20")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="time the headline workload only (by default the other four configurations are timed too and "
                         "reported under `configs`)")
    ap.add_argument("--chunk-syms", type=int, default=0,
                    help="rANS unit length; 0 = one unit per (session, layer, head) stream")
    ap.add_argument("--layout", default="lhnkd", choices=["lhnkd", "lnkhd"])
    ap.add_argument("--sessions", type=int, default=None, help="override the number of sessions")
    ap.add_argument("--groups", type=int, default=1,
                    help="code a cache of thousands of streams as this many independent groups of sessions (or layers), "
                         "the entropy coding of one group on a second HIP stream beside the next group's prediction "
                         "pass (codec.GroupedCodec); 1 = one codec over everything, which measured faster")
    ap.add_argument("--no-overlap", action="store_true",
                    help="with groups: every call on one stream (no entropy coding beside the next group's prediction pass)")
    ap.add_argument("--separate-histogram", action="store_true",
                    help="take the symbol statistics with plc_histogram after the prediction pass instead of inside it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain elementwise kernel that reads and writes 256 MiB, as the known-size "
                         "reference for scaling HBM byte counters in a profiler run")
    ap.add_argument("--cpu-sessions", type=int, default=2,
                    help="sessions of the 64-session workload the CPU oracle is timed on (the Llama-shaped one is timed whole)")
    ap.add_argument("--cpu-streams", type=int, default=256, help="streams of other workloads the CPU oracle is timed on")
    ap.add_argument("--also-chunked", type=int, default=4096,
                    help="Llama-shaped side measurement: the same workload with rANS units of this many symbols (0 = skip)")
    ap.add_argument("--no-side-paths", action="store_true",
                    help="skip every side measurement on the Llama-shaped workload (the flags below skip them one by one)")
    ap.add_argument("--no-lnkhd", action="store_true", help="skip the run with the candidates stored [L,n,k,H,d]")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="skip the measurement with the steps dealt to several streams")
    ap.add_argument("--pipeline-streams", type=int, default=3, help="streams of that measurement")
    ap.add_argument("--no-conditional", action="store_true",
                    help="skip the token-conditional path (prediction = the true token's candidate, its index coded in a "
                         "stream of its own)")
    ap.add_argument("--no-adaptive", action="store_true",
                    help="skip the surprisal-adaptive quantiser (bit depth per position from the token's surprisal, one "
                         "table per depth) on the token-conditional path")
    ap.add_argument("--no-linear", action="store_true",
                    help="skip the linear-embedding predictor (two fp16 contractions on the matrix cores)")
    ap.add_argument("--no-padded-vocabulary", action="store_true",
                    help="linear predictor: skip the extra timing of the first contraction with the vocabulary padded to a multiple of 64")
    ap.add_argument("--two-call-decode", action="store_true",
                    help="decode with plc_rans_decode then plc_reconstruct instead of the single call that "
                         "reconstructs inside the entropy decoder")
    ap.add_argument("--no-prefix-index", action="store_true", help="skip the host-side prefix index measurement")
    ap.add_argument("--adaptive-b0", type=float, default=3.0, help="target average bit depth b0")
    ap.add_argument("--adaptive-range", type=float, default=0.32, help="quantiser range: step = range / 2^depth")
    return ap.parse_args()


class KernelTimer:
    """HIP event pairs that libplc records around the main kernel of each call, on the stream of the call:
    one pair per kernel, timed step and launch of the step (a cache coded in groups launches each kernel
    once per group)."""

    def __init__(self, plc, torch, steps, launches=1, conditional=False, linear=False, fused=False,
                 fused_counts=False):
        self.plc, self.ids = plc, {"predict_residual": plc.TRACE_PREDICT, "reconstruct": plc.TRACE_RECONSTRUCT,
                                   "histogram": plc.TRACE_HISTOGRAM, "rans_encode": plc.TRACE_RANS_ENCODE,
                                   "rans_decode": plc.TRACE_RANS_DECODE}
        if conditional:
            del self.ids["predict_residual"], self.ids["reconstruct"]
            self.ids.update(predict_residual_cond=plc.TRACE_PREDICT_COND, reconstruct_cond=plc.TRACE_RECONSTRUCT_COND)
        if linear:
            del self.ids["predict_residual"], self.ids["reconstruct"]
            self.ids.update(expected_embedding=plc.TRACE_EXPECTED_EMBEDDING, predict_linear=plc.TRACE_PREDICT_LINEAR,
                            reconstruct_linear=plc.TRACE_RECONSTRUCT_LINEAR)
        if fused_counts:    # the statistics are taken inside the prediction pass: no histogram launch
            self.ids.pop("histogram", None)
        if fused:       # one kernel decodes and reconstructs
            for name in ("reconstruct", "reconstruct_cond", "rans_decode"):
                self.ids.pop(name, None)
            self.ids["rans_decode_reconstruct"] = plc.TRACE_RANS_DECODE
        self.launches = launches
        self.ev = {}
        for name in self.ids:
            pairs = []
            for _ in range(steps * launches):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                b.record()          # creates the underlying hipEvent_t
                pairs.append((a, b))
            self.ev[name] = pairs

    def arm(self, step, launch=0):
        for name, kid in self.ids.items():
            a, b = self.ev[name][step * self.launches + launch]
            self.plc.plc_trace_kernel_events(kid, a.cuda_event, b.cuda_event)

    def disarm(self):
        for kid in self.ids.values():
            self.plc.plc_trace_kernel_events(kid, None, None)

    def mean_ms(self):
        return {name: sum(a.elapsed_time(b) for a, b in pairs) / len(pairs) for name, pairs in self.ev.items()}

    def spread_ms(self):
        """(median, min) of the launch durations of each kernel."""
        out = {}
        for name, pairs in self.ev.items():
            t = sorted(a.elapsed_time(b) for a, b in pairs)
            mid = len(t) // 2
            out[name] = (t[mid] if len(t) % 2 else 0.5 * (t[mid - 1] + t[mid]), t[0])
        return out


def measured_traffic(kernel, config_name):
    """HBM bytes per launch of `kernel` (its name as the profiler prints it, template arguments included)
    from the committed rocprofv3 counter summary, or None when there is none for this workload or the
    kernels' sources have changed since the counters were taken."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{config_name}.txt")
    if not os.path.exists(path):
        return None
    h = hashlib.sha256()
    for f in ("plc_predict.hip", "plc_rans.hip", "plc_hist_freq.hip", "plc_device.h"):
        with open(os.path.join(ROOT, "paper_2604_15356_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    for line in open(path):
        m = re.match(r"machine-readable: kernel=(.+) traffic_bytes_per_launch=(\d+) source_sha256=(\w+)", line)
        if m and m.group(1) == kernel and m.group(3) == h.hexdigest():
            return int(m.group(2))
    return None


class Run:
    """One workload resident in HBM with its codec(s) and output buffers."""

    def __init__(self, name, args, torch, layout=None, chunk_syms=None, groups=None):
        from paper_2604_15356_amd.codec import GroupedCodec, KVDeltaCodec
        from paper_2604_15356_amd.workloads import make_workload
        self.name, self.torch = name, torch
        self.layout = layout or args.layout
        self.chunk_syms = args.chunk_syms if chunk_syms is None else chunk_syms
        dev = torch.device("cuda:0")
        overrides = {"S": args.sessions} if args.sessions else None
        t0 = time.perf_counter()
        self.w = w = make_workload(name, device=dev, layout=self.layout, overrides=overrides)
        torch.cuda.synchronize()
        log(f"workload {name}: S{w.S} L{w.L} H{w.H} d{w.d} n{w.n} k{w.k} delta {w.delta} candidates {self.layout} "
            f"({w.kv_bytes / 1e9:.3f} GB fp16 KV, {w.cand_k.numel() * 4 / 1e9:.2f} GB candidates) drawn in "
            f"{time.perf_counter() - t0:.1f} s")
        kw = dict(chunk_syms=self.chunk_syms, device=dev, cand_stride=w.cand_k.stride()[:5],
                  act_stride=w.act_k.stride()[:4])
        want = args.groups if groups is None else groups
        want = min(want, w.n_streams // GROUP_MIN_STREAMS)       # a group keeps the many-unit kernels busy
        self.grouped = want > 1 and self.chunk_syms == 0
        if self.grouped:
            self.codec = GroupedCodec(w.S, w.L, w.H, w.n, w.k, w.d, w.delta, w.qmax, groups=want, **kw)
            self.launches = len(self.codec.codecs)
        else:
            self.codec = KVDeltaCodec(w.S, w.L, w.H, w.n, w.k, w.d, w.delta, w.qmax, **kw)
            self.launches = 1
        self.out_k, self.out_v = torch.empty_like(w.act_k), torch.empty_like(w.act_v)
        self.fused = not args.two_call_decode
        self.overlap = not args.no_overlap
        self.fused_counts = self.grouped or not args.separate_histogram
        # whether the single decode call runs its one-kernel form for this shape (see include/plc.h)
        self.one_kernel = self.fused and self.chunk_syms == 0 and w.k <= 8

    def step(self, marks=None):
        w, c = self.w, self.codec
        if marks:
            marks[0].record()
        if self.grouped:
            c.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, overlap=self.overlap)
        else:
            c.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, fused_counts=self.fused_counts)
        if marks:
            marks[1].record()
        if self.grouped:
            c.decode(w.cand_k, w.cand_v, w.probs, self.out_k, self.out_v, fused=self.fused, overlap=False)
        else:
            c.decode(w.cand_k, w.cand_v, w.probs, self.out_k, self.out_v, fused=self.fused)
        if marks:
            marks[2].record()

    def codecs(self):
        return self.codec.codecs if self.grouped else [self.codec]

    def max_abs_error(self):
        torch, w = self.torch, self.w
        worst = 0.0
        for s_ in range(w.S):
            for l_ in range(w.L):
                for got, want in ((self.out_k, w.act_k), (self.out_v, w.act_v)):
                    diff = (got[s_, l_].float() - want[s_, l_].float()).abs()
                    worst = max(worst, float(torch.nan_to_num(diff, nan=0.0, posinf=0.0).max()))
        return worst

    def close(self):
        self.codec = self.w = self.out_k = self.out_v = None
        self.torch.cuda.empty_cache()


def time_run(run, args, plc, torch, calibrate=False):
    """Warm-ups, then exactly args.steps timed steps; returns the result dictionary of this workload."""
    import numpy as np
    w = run.w
    for _ in range(args.warmup):
        run.step()
    torch.cuda.synchronize()
    run.codec.check_status("warmup")
    if calibrate:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device=w.cand_k.device)
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)      # 256 MiB read + 256 MiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst
    timer = KernelTimer(plc, torch, args.steps, launches=run.launches, fused=run.one_kernel,
                        fused_counts=run.fused_counts)
    if run.grouped:
        state = {"step": 0}
        run.codec.hook = lambda launch: timer.arm(state["step"], launch)
    # events at the start, between encode and decode, and at the end of every step: the two directions apart
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if run.grouped:
            state["step"] = i
        else:
            timer.arm(i)
        run.step(marks[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    timer.disarm()
    if run.grouped:
        run.codec.hook = None
    run.codec.check_status("timed steps")
    ms_per_step = dt / args.steps * 1e3
    value = w.kv_bytes / (dt / args.steps) / 1e9
    encode_ms = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps
    decode_ms = sum(m[1].elapsed_time(m[2]) for m in marks) / args.steps

    # ---- what was produced
    E = w.n_streams * w.syms_per_stream
    cs = run.codecs()
    n_units = sum(c.n_units for c in cs)
    total_words = sum(int(c.n_words.to(torch.int64).sum()) for c in cs)
    n_esc = sum(int(c.esc_cnt.to(torch.int64).sum()) for c in cs)
    payload = 16 * total_words + 16 * n_esc
    total_bits = payload + 32 * 32 * n_units + (256 * 16 + 3 * 32) * w.n_streams
    roundtrip_exact = all(bool(torch.equal(c.dec_symbols, c.symbols)) for c in cs)
    max_err = run.max_abs_error()

    # ---- per-kernel accounting (algorithmic bytes per launch / mean launch duration)
    ms = timer.mean_ms()
    word_bytes = 2.0 * total_words
    L = run.launches
    alg_bytes = {"predict_residual": (2 * w.k + 3) * E / L, "reconstruct": (2 * w.k + 3) * E / L, "histogram": 1.0 * E / L,
                 "rans_encode": (E + word_bytes) / L, "rans_decode": (E + word_bytes) / L,
                 # words in, symbols out, 2k bytes of candidates in and 2 bytes of KV out per component
                 "rans_decode_reconstruct": ((2 * w.k + 3) * E + word_bytes) / L}
    kernels = {}
    spread = timer.spread_ms()
    for name, t in ms.items():
        gbs = alg_bytes[name] / (t * 1e-3) / 1e9
        kernels[name] = dict(ms=round(t, 4), median_ms=round(spread[name][0], 4), min_ms=round(spread[name][1], 4),
                             launches_per_step=L, ms_per_step=round(t * L, 4),
                             GBs=round(gbs, 1), frac_hbm=round(gbs / HBM_PEAK_GBS, 4))
        log(f"  {name:24s} {L:2d} x {t:9.4f} ms  {gbs:8.1f} GB/s algorithmic  {100 * gbs / HBM_PEAK_GBS:5.1f} % of HBM peak")
    log(f"  step (encode+decode) {ms_per_step:9.4f} ms = {value:.1f} GB/s of KV;  encode {encode_ms:.4f} ms "
        f"({w.kv_bytes / encode_ms / 1e6:.1f} GB/s), decode {decode_ms:.4f} ms ({w.kv_bytes / decode_ms / 1e6:.1f} GB/s)")
    # The roofline object describes the kernel a step spends most time in.  All of them are priced against
    # HBM: the step holds no contraction, and the entropy coder's chains have no tighter ceiling to name.
    # the kernels' names as the profiler prints them (template arguments included), for the traffic lookup
    units_per_launch = n_units // L
    streams_per_launch = w.n_streams // L
    few = run.chunk_syms == 0 and units_per_launch <= 1024      # the whole-stream kernels for few units
    if few:
        enc_name, dec_name = "rans_encode_pipe_kernel<false>", "rans_decode_chain_kernel<0, false, 4>"
    elif run.chunk_syms == 0:                                   # many whole streams: two per wavefront
        pairs = (units_per_launch + 1) // 2
        enc_name = f"rans_encode_pair_kernel<1, true, {2 if 2048 < pairs <= 2816 else 4}>"
        dec_name = "rans_decode_kernel<1, false, true>"
    else:
        n_full = w.syms_per_stream // run.chunk_syms
        ups = (w.syms_per_stream + run.chunk_syms - 1) // run.chunk_syms
        slots = n_full // 2 + (n_full & 1) + (1 if n_full < ups else 0)
        pw = 1
        while pw < 4 and 2 * pw <= slots:
            pw *= 2
        dw = 1
        while dw < 8 and 2 * dw <= ups:
            dw *= 2
        enc_name, dec_name = f"rans_encode_pair_kernel<{pw}, false, 4>", f"rans_decode_kernel<{dw}, false, true>"
    dense = streams_per_launch > 512
    if dense and w.k <= 4:              # 4-byte entries, four workgroups per compute unit
        fused_name = f"rans_decode_depths_kernel<{w.k}, 1>"
    else:                               # three-block word ring for k = 5, 6 and many streams
        fused_name = f"rans_decode_chain_kernel<{w.k}, false, {3 if (dense and w.k <= 6) else 4}>"
    symbol = {"predict_residual": f"predict_residual_hist_kernel<{w.k}>" if run.fused_counts else
              f"predict_residual_kernel<{w.k}>", "reconstruct": f"reconstruct_kernel<{w.k}, false>",
              "histogram": "histogram_kernel", "rans_encode": enc_name, "rans_decode": dec_name,
              "rans_decode_reconstruct": fused_name}
    dom_name = max(ms, key=lambda nm: ms[nm] * L)
    dom = kernels[dom_name]
    plain = run.layout == "lhnkd" and not args.sessions and run.chunk_syms == 0
    roofline = dict(bound="hbm", kernel=symbol[dom_name], achieved=dom["GBs"], peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=dom["frac_hbm"],
                    traffic=measured_traffic(symbol[dom_name], run.name) if plain else None,
                    bytes_per_launch=int(alg_bytes[dom_name]), components_per_launch=E // L)
    for name, kd in kernels.items():
        kd["traffic"] = measured_traffic(symbol[name], run.name) if plain else None
    how = "one kernel (reconstruction inside the entropy decoder)" if run.one_kernel else "two kernels"
    config = {"workload": f"{run.name}: S={w.S} L={w.L} H={w.H} d={w.d} n={w.n} k={w.k} delta={w.delta} qmax=127, "
                          f"candidates {run.layout}", "chunk_syms": run.chunk_syms, "rans_units": n_units, "decode": how}
    if run.grouped:
        sl = run.codec.slices
        what = f"{sl[0][1] - sl[0][0]} sessions" if sl[0][3] - sl[0][2] == w.L else f"{sl[0][3] - sl[0][2]} layers"
        config["groups"] = L
        config["encode"] = (f"{L} independent groups of {what}; the statistics, tables and rANS encoder of a group run on a "
                            "second HIP stream beside the next group's prediction pass" if run.overlap else
                            f"{L} independent groups of {what}, every call on one stream")
    return {
        "value": round(value, 2), "unit": "GB/s", "ms_per_step": round(ms_per_step, 4), "config": config,
        "roofline": roofline, "kernels": kernels,
        "directions": {"encode_ms": round(encode_ms, 4), "encode_GBs": round(w.kv_bytes / encode_ms / 1e6, 1),
                       "decode_ms": round(decode_ms, 4), "decode_GBs": round(w.kv_bytes / decode_ms / 1e6, 1)},
        "kv_GB": round(w.kv_bytes / 1e9, 3),
        "coded_bits_per_token": round(total_bits / (w.S * w.n), 1),
        "payload_bits_per_symbol": round(payload / E, 4),
        "fp16_bits_per_token": 2 * w.L * w.H * w.d * 16,
        "escape_rate": round(n_esc / E, 6),
        "roundtrip_symbols_exact": roundtrip_exact,
        "max_abs_reconstruction_error": round(max_err, 6),
    }


def cpu_baseline(run, n_streams, torch):
    """The oracle, as it stands, on the first n_streams streams of the workload, one stream per task; and the
    GPU's artefacts for those streams checked against it (symbols up to fp32/fp64 near-ties; the oracle's
    decoder on the GPU's tables, states and words)."""
    import numpy as np
    from oracle import plc_oracle as O
    O.build()
    w = run.w
    n_sample = min(n_streams, w.n_streams)
    nproc = os.cpu_count() or 1
    threads = max(1, min(16, nproc, n_sample))
    host = lambda t: t.contiguous().cpu().numpy()
    jobs = []
    for st in range(n_sample):
        s, r = divmod(st, w.L * w.H)
        l, h = divmod(r, w.H)
        jobs.append(dict(ck=host(w.cand_k[s, l, h]), cv=host(w.cand_v[s, l, h]), ak=host(w.act_k[s, l, h]),
                         av=host(w.act_v[s, l, h]), p=host(w.probs[s])))
    dm = O.make_dims(1, 1, 1, w.n, w.k, w.d, w.delta, w.qmax)

    def one(j):
        r = O.predict_residual(dm, j["ck"], j["cv"], j["p"], j["ak"], j["av"], mode=O.F64)
        counts = O.histogram(r["symbols"])
        freq, _ = O.build_freq(counts)
        enc = O.rans_encode(r["symbols"], freq)
        dec = O.rans_decode(freq, enc["states"], enc["words"], enc["word_off"], enc["n_words"], 1, r["symbols"].shape[1])
        O.reconstruct(dm, j["ck"], j["cv"], j["p"], dec, r["esc_vals"], r["esc_off"], mode=O.F64)
        return r["symbols"]

    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        syms = list(ex.map(one, jobs))
    dt = time.perf_counter() - t0
    n_single = min(4, n_sample)
    t1 = time.perf_counter()
    for j in jobs[:n_single]:
        one(j)
    dt1 = time.perf_counter() - t1
    stream_bytes = 2 * w.n * w.d * 2
    kv_bytes = n_sample * stream_bytes
    whole = n_sample == w.n_streams
    base = dict(value=round(kv_bytes / dt / 1e9, 4), unit="GB/s", cores=threads, nproc=nproc, kind="oracle",
                sample=("the whole workload" if whole else f"first {n_sample} of {w.n_streams} streams")
                + f" ({kv_bytes / 1e6:.0f} MB of fp16 KV), encode+decode, fp64, {dt:.1f} s wall",
                one_thread=dict(value=round(n_single * stream_bytes / dt1 / 1e9, 4), unit="GB/s", cores=1,
                                sample=f"first {n_single} streams, {dt1:.1f} s wall"))
    # ---- the GPU's artefacts for the sampled streams against the oracle (not timed)
    sym64 = np.concatenate(syms, axis=0)
    u = lambda t, dt_: t.contiguous().cpu().numpy().view(dt_)
    diff, decoded_ok, at = 0, True, 0
    for c in run.codecs():
        take = min(c.n_streams, n_sample - at)
        if take <= 0:
            break
        got = u(c.symbols[:take], np.uint8)
        diff += int((got != sym64[at:at + take]).sum())
        words = u(c.words[:take * c.word_cap], np.uint16)
        back = O.rans_decode(u(c.freq[:take], np.uint16), u(c.states[:take], np.uint32), words,
                             u(c.word_off[:take], np.uint64), u(c.n_words[:take], np.uint32), take, c.N)
        decoded_ok = decoded_ok and bool(np.array_equal(back, got))
        at += take
    check = dict(near_ties_vs_fp64_oracle=dict(count=diff, of=int(sym64.size)),
                 gpu_streams_decoded_by_the_oracle=dict(streams=at, symbols_equal=decoded_ok))
    log(f"  cpu oracle on {run.name}: {base['value']:.4f} GB/s on {threads} threads of {nproc} ({base['sample']}); "
        f"{base['one_thread']['value']:.4f} GB/s on one thread; near-ties {diff} of {sym64.size}; "
        f"oracle decodes the GPU's streams: {decoded_ok}")
    return base, check


def side_paths(run, args, plc, torch, result):
    """Side measurements on the Llama-shaped workload, never part of `value`."""
    import numpy as np
    from paper_2604_15356_amd.codec import KVDeltaCodec
    w, dev = run.w, run.w.cand_k.device
    out_k, out_v, fused, one_kernel = run.out_k, run.out_v, run.fused, run.one_kernel
    codec = run.codec
    E = w.n_streams * w.syms_per_stream
    n_esc = int(codec.esc_cnt.to(torch.int64).sum())
    mk = lambda **kw: KVDeltaCodec(w.S, w.L, w.H, w.n, w.k, w.d, w.delta, w.qmax, device=dev,
                                   cand_stride=w.cand_k.stride()[:5], act_stride=w.act_k.stride()[:4], **kw)
    if run.chunk_syms == 0 and args.also_chunked > 0:
        # Same workload, same step, but every run of `also_chunked` symbols is its own rANS unit (128 B of lane
        # states per chunk): the rANS chains become short and plentiful.  Reported beside the headline, not as it.
        codec2 = mk(chunk_syms=args.also_chunked)

        def step2():
            codec2.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
            codec2.decode(w.cand_k, w.cand_v, w.probs, out_k, out_v, fused=fused)

        for _ in range(args.warmup):
            step2()
        torch.cuda.synchronize()
        timer2 = KernelTimer(plc, torch, args.steps, fused_counts=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            timer2.arm(i)
            step2()
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        timer2.disarm()
        codec2.check_status("chunked steps")
        nw2 = int(codec2.n_words.to(torch.int64).sum())
        bits2 = 16 * nw2 + 16 * n_esc + 32 * 32 * codec2.n_units + (256 * 16 + 3 * 32) * w.n_streams
        ms2 = timer2.mean_ms()
        result["chunked"] = {
            "workload": run.name, "chunk_syms": args.also_chunked, "rans_units": codec2.n_units,
            "value": round(w.kv_bytes / (dt2 / args.steps) / 1e9, 2), "unit": "GB/s",
            "ms_per_step": round(dt2 / args.steps * 1e3, 4),
            "coded_bits_per_token": round(bits2 / (w.S * w.n), 1),
            "roundtrip_symbols_exact": bool(torch.equal(codec2.dec_symbols, codec2.symbols)),
            "kernels_ms": {k: round(v, 4) for k, v in ms2.items()},
        }
        log(f"  with rANS units of {args.also_chunked} symbols: step {dt2 / args.steps * 1e3:.4f} ms "
            f"({result['chunked']['value']} GB/s), rans_encode {ms2['rans_encode']:.4f} ms, rans_decode {ms2['rans_decode']:.4f} ms")
        del codec2
    if not args.no_pipeline:
        # The same steps dealt in turn to a few HIP streams (default priority), each with a codec and output
        # buffers of its own: a step is sequential inside, but the entropy coder keeps only a few wavefronts
        # per compute unit busy, so the neighbouring step's memory-bound kernels run beside it.  What a
        # serving loop that codes independent sessions gets; reported beside the headline, not as it.
        NS = max(2, args.pipeline_streams)
        lanes = [(torch.cuda.Stream(device=dev), codec, out_k, out_v)]
        for _ in range(NS - 1):
            lanes.append((torch.cuda.Stream(device=dev), mk(chunk_syms=run.chunk_syms),
                          torch.zeros_like(out_k), torch.zeros_like(out_v)))

        def run_pipelined(count):
            for st, _, _, _ in lanes:
                st.wait_stream(torch.cuda.current_stream())
            for i in range(count):
                st, cd, ok_, ov_ = lanes[i % NS]
                with torch.cuda.stream(st):
                    cd.encode(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v)
                    cd.decode(w.cand_k, w.cand_v, w.probs, ok_, ov_, fused=fused)
            for st, _, _, _ in lanes:
                torch.cuda.current_stream().wait_stream(st)

        run_pipelined(NS * max(1, args.warmup))
        torch.cuda.synchronize()
        steps_p = ((args.steps + NS - 1) // NS) * NS
        t0 = time.perf_counter()
        run_pipelined(steps_p)
        torch.cuda.synchronize()
        dtp = time.perf_counter() - t0
        same = True
        for _, cd, ok_, ov_ in lanes:
            cd.check_status("pipelined steps")
            same = same and bool(torch.equal(cd.dec_symbols, cd.symbols)) and bool(torch.equal(ok_, out_k)) and \
                bool(torch.equal(ov_, out_v)) and bool(torch.equal(cd.n_words, codec.n_words)) and \
                bool(torch.equal(cd.states, codec.states))
        result["stream_pipeline"] = {
            "workload": run.name, "streams": NS, "steps": steps_p,
            "value": round(w.kv_bytes / (dtp / steps_p) / 1e9, 2), "unit": "GB/s",
            "ms_per_step": round(dtp / steps_p * 1e3, 4), "outputs_identical": same,
        }
        log(f"  steps dealt to {NS} streams: {dtp / steps_p * 1e3:.4f} ms per step "
            f"({result['stream_pipeline']['value']} GB/s), outputs identical: {same}")
        del lanes
    if not args.no_conditional:
        # Token-conditional path on the same workload and in the same format (whole streams unless --chunk-syms):
        # every position is predicted by the candidate of its true token (given, as the serving loop knows it),
        # whose index goes into a per-session stream coded under the model's probabilities.  Per component a
        # position then moves 2 B of one candidate instead of 2k B of all of them: 5 algorithmic bytes.
        codec3 = mk(chunk_syms=run.chunk_syms)
        chosen = w.chosen.to(torch.int32).contiguous()

        def step3():
            codec3.encode_cond(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen=chosen)
            codec3.decode_cond(w.cand_k, w.cand_v, w.probs, out_k, out_v, fused=fused)

        for _ in range(args.warmup):
            step3()
        torch.cuda.synchronize()
        one_kernel3 = one_kernel and (w.n_streams <= 2048 or w.k <= 4)     # the one-call decode's own bound on this path
        timer3 = KernelTimer(plc, torch, args.steps, conditional=True, fused=one_kernel3)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            timer3.arm(i)
            step3()
        torch.cuda.synchronize()
        dt3 = time.perf_counter() - t0
        timer3.disarm()
        codec3.check_status("token-conditional steps")
        nw3 = int(codec3.n_words.to(torch.int64).sum())
        esc3 = int(codec3.esc_cnt.to(torch.int64).sum())
        idx_bits = 16 * int(codec3.idx_n_words.to(torch.int64).sum()) + 32 * 32 * w.S
        bits3 = 16 * nw3 + 16 * esc3 + 32 * 32 * codec3.n_units + (256 * 16 + 3 * 32) * w.n_streams + idx_bits
        err3 = run.max_abs_error()
        ms3 = timer3.mean_ms()
        k3 = {}
        miss_share = float((chosen < 0).float().mean())     # those positions read all k candidates
        cond_bytes = (1.0 - miss_share) * 5.0 + miss_share * (2 * w.k + 3)
        for name in ("predict_residual_cond", "reconstruct_cond"):
            if name not in ms3:     # the reconstruction ran inside the entropy decoder
                continue
            gbs = cond_bytes * E / (ms3[name] * 1e-3) / 1e9
            k3[name] = dict(ms=round(ms3[name], 4), GBs=round(gbs, 1), frac_hbm=round(gbs / HBM_PEAK_GBS, 4))
        result["token_conditional"] = {
            "workload": run.name,
            "value": round(w.kv_bytes / (dt3 / args.steps) / 1e9, 2), "unit": "GB/s",
            "ms_per_step": round(dt3 / args.steps * 1e3, 4), "bytes_per_component": round(cond_bytes, 3),
            "miss_share": round(miss_share, 4),
            "coded_bits_per_token": round(bits3 / (w.S * w.n), 1),
            "payload_bits_per_symbol": round((16 * nw3 + 16 * esc3) / E, 4),
            "index_bits_per_token": round(idx_bits / (w.S * w.n), 3),
            "escape_rate": round(esc3 / E, 6),
            "roundtrip_symbols_exact": bool(torch.equal(codec3.dec_symbols, codec3.symbols)),
            "roundtrip_indices_exact": bool(torch.equal(codec3.dec_chosen, chosen)),
            "max_abs_reconstruction_error": round(err3, 6),
            "kernels": k3, "kernels_ms": {k: round(v, 4) for k, v in ms3.items()},
            "decode": "one kernel (reconstruction inside the entropy decoder)" if one_kernel3 else "two kernels",
        }
        log(f"  token-conditional: step {dt3 / args.steps * 1e3:.4f} ms ({result['token_conditional']['value']} GB/s), "
            f"{result['token_conditional']['payload_bits_per_symbol']} bits/component + "
            f"{result['token_conditional']['index_bits_per_token']} index bits/token; "
            + ", ".join(f"{k} {v['ms']} ms = {100 * v['frac_hbm']:.1f} % of HBM peak" for k, v in k3.items()))
        del codec3
    if not args.no_adaptive and w.d % 16 == 0:
        # Surprisal-adaptive quantiser on the token-conditional path: depth b_i = min(4, max(1, floor(b0 * h_i / hbar)))
        # from the token's coded surprisal (hbar = log2 of the configuration's perplexity), step = range / 2^b_i,
        # one frequency table per depth.  Same format as the headline otherwise (whole streams unless --chunk-syms).
        codec4 = mk(chunk_syms=run.chunk_syms)
        chosen4 = w.chosen.to(torch.int32).contiguous()
        hbar = float(np.log2(np.mean(w.perplexity)))
        thr = plc.plc_surprisal_thresholds(args.adaptive_b0, hbar)

        def step4():
            codec4.encode_adapt(w.cand_k, w.cand_v, w.probs, w.act_k, w.act_v, chosen4, thr, args.adaptive_range)
            codec4.decode_adapt(w.cand_k, w.cand_v, w.probs, out_k, out_v, thr, args.adaptive_range, fused=fused)

        for _ in range(args.warmup):
            step4()
        torch.cuda.synchronize()
        one_kernel4 = one_kernel and w.n_streams <= 512      # the bound of the decoder with one table per depth
        timer4 = KernelTimer(plc, torch, args.steps, conditional=True, fused=one_kernel4)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            timer4.arm(i)
            step4()
        torch.cuda.synchronize()
        dt4 = time.perf_counter() - t0
        timer4.disarm()
        codec4.check_status("surprisal-adaptive steps")
        nw4 = int(codec4.n_words.to(torch.int64).sum())
        esc4 = int(codec4.esc_cnt.to(torch.int64).sum())
        idx4 = 16 * int(codec4.idx_n_words.to(torch.int64).sum()) + 32 * 32 * w.S
        tables = int((codec4.freq_d.to(torch.int32).abs().sum(-1) > 0).sum())          # tables actually used
        bits4 = 16 * nw4 + 16 * esc4 + 32 * 32 * codec4.n_units + 256 * 16 * tables + 3 * 32 * w.n_streams + idx4
        depth = codec4.bits.cpu().numpy()
        sq = 0.0
        for s_ in range(w.S):
            for l_ in range(w.L):
                for got, want in ((out_k, w.act_k), (out_v, w.act_v)):
                    diff = torch.nan_to_num(got[s_, l_].float() - want[s_, l_].float(), nan=0.0, posinf=0.0, neginf=0.0)
                    sq += float((diff.double() ** 2).sum())
        ms4 = timer4.mean_ms()
        result["surprisal_adaptive"] = {
            "workload": run.name,
            "b0": args.adaptive_b0, "hbar": round(hbar, 4), "range": args.adaptive_range, "thresholds": thr[2:],
            "depth_shares": {str(b): round(float((depth == b).mean()), 4) for b in range(1, plc.MAX_BITS + 1)},
            "mean_depth": round(float(depth.mean()), 3),
            "value": round(w.kv_bytes / (dt4 / args.steps) / 1e9, 2), "unit": "GB/s",
            "ms_per_step": round(dt4 / args.steps * 1e3, 4),
            "coded_bits_per_token": round(bits4 / (w.S * w.n), 1),
            "payload_bits_per_symbol": round((16 * nw4 + 16 * esc4) / E, 4),
            "mean_square_error": float(f"{sq / E:.4e}"),
            "fixed_step_mean_square_error": float(f"{float(np.float32(w.delta)) ** 2 / 12:.4e}"),
            "roundtrip_symbols_exact": bool(torch.equal(codec4.dec_symbols, codec4.symbols)),
            "roundtrip_depths_exact": bool(torch.equal(codec4.dec_bits, codec4.bits)),
            "kernels_ms": {k: round(v, 4) for k, v in ms4.items() if k != "histogram"},
            "decode": "one kernel (reconstruction inside the entropy decoder)" if one_kernel4 else "two kernels",
        }
        r4 = result["surprisal_adaptive"]
        log(f"  surprisal-adaptive (b0 {args.adaptive_b0}, range {args.adaptive_range}): step {r4['ms_per_step']} ms "
            f"({r4['value']} GB/s), mean depth {r4['mean_depth']}, {r4['payload_bits_per_symbol']} bits/component, "
            f"mse {r4['mean_square_error']:.3e} (fixed step: {r4['fixed_step_mean_square_error']:.3e}); "
            + ", ".join(f"{k} {ms4[k]:.3f} ms" for k in ("rans_encode", "rans_decode", "rans_decode_reconstruct") if k in ms4))
        del codec4


def linear_path(args, plc, torch, result, chunk_syms):
    """Linear-embedding predictor on a workload of the Llama-shaped KV cache: prediction = c + A * Ebar with
    Ebar = P * E over a 50,016-token vocabulary (embedding dimension 4096), both contractions in fp16 on the
    matrix cores with fp32 accumulation; the expected embedding is recomputed on the decode side."""
    import numpy as np
    from paper_2604_15356_amd.codec import KVDeltaCodec
    from paper_2604_15356_amd.workloads import make_linear_workload
    MFMA_PEAK_TFLOPS = 2500.0           # MI355X dense fp16, published
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    lw = make_linear_workload("llama8b", device=dev)
    torch.cuda.synchronize()
    log(f"  linear-predictor workload: m {lw.m}, V {lw.V} drawn in {time.perf_counter() - t0:.1f} s")
    codec5 = KVDeltaCodec(lw.S, lw.L, lw.H, lw.n, 1, lw.d, lw.delta, lw.qmax, chunk_syms=chunk_syms, device=dev)
    lo_k, lo_v = torch.empty_like(lw.act_k), torch.empty_like(lw.act_v)

    def step5():
        codec5.encode_linear(lw.probs_full, lw.embed_t, lw.A, lw.bias_k, lw.bias_v, lw.act_k, lw.act_v)
        codec5.decode_linear(lw.probs_full, lw.embed_t, lw.A, lw.bias_k, lw.bias_v, lo_k, lo_v)

    lin_steps = max(2, args.steps // 4)
    for _ in range(min(2, args.warmup)):
        step5()
    torch.cuda.synchronize()
    timer5 = KernelTimer(plc, torch, lin_steps, linear=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(lin_steps):
        timer5.arm(i)
        step5()
    torch.cuda.synchronize()
    dt5 = time.perf_counter() - t0
    timer5.disarm()
    codec5.check_status("linear-predictor steps")
    ms5 = timer5.mean_ms()
    rows5 = lw.S * lw.n
    flops = {"expected_embedding": 2.0 * rows5 * lw.m * lw.V,
             "predict_linear": 2.0 * lw.S * lw.L * lw.n * (2 * lw.H * lw.d) * lw.m,
             "reconstruct_linear": 2.0 * lw.S * lw.L * lw.n * (2 * lw.H * lw.d) * lw.m}
    k5 = {}
    for name, fl in flops.items():
        tf = fl / (ms5[name] * 1e-3) / 1e12
        k5[name] = dict(ms=round(ms5[name], 4), TFLOPs=round(tf, 1), frac_mfma=round(tf / MFMA_PEAK_TFLOPS, 4))
    E5 = lw.S * lw.L * lw.H * lw.n * 2 * lw.d
    nw5 = int(codec5.n_words.to(torch.int64).sum())
    esc5 = int(codec5.esc_cnt.to(torch.int64).sum())
    err5 = 0.0
    for l_ in range(lw.L):
        for got, want in ((lo_k, lw.act_k), (lo_v, lw.act_v)):
            diff = (got[0, l_].float() - want[0, l_].float()).abs()
            err5 = max(err5, float(torch.nan_to_num(diff, nan=0.0, posinf=0.0).max()))
    # Context, not part of the step: the first contraction with the vocabulary padded to a multiple of 64
    # tokens (zero probabilities), which makes every row's pitch a whole number of 128-byte lines.
    V64 = (lw.V + 63) // 64 * 64
    padded = None
    if V64 != lw.V and not args.no_padded_vocabulary:
        p64 = torch.zeros((rows5, V64), dtype=torch.float16, device=dev)
        e64 = torch.zeros((lw.m, V64), dtype=torch.float16, device=dev)
        p64[:, :lw.V].copy_(lw.probs_full.reshape(rows5, lw.V))
        e64[:, :lw.V].copy_(lw.embed_t)
        eb64 = torch.empty((rows5, lw.m), dtype=torch.float16, device=dev)
        for _ in range(2):
            plc.plc_expected_embedding(p64, e64, eb64)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(lin_steps):
            plc.plc_expected_embedding(p64, e64, eb64)
        ev1.record()
        torch.cuda.synchronize()
        ms64 = ev0.elapsed_time(ev1) / lin_steps
        eb = torch.empty_like(eb64)
        plc.plc_expected_embedding(lw.probs_full.reshape(rows5, lw.V), lw.embed_t, eb)
        tf64 = flops["expected_embedding"] / (ms64 * 1e-3) / 1e12    # the useful flops: the padding adds none
        padded = dict(V=V64, ms=round(ms64, 4), TFLOPs=round(tf64, 1), frac_mfma=round(tf64 / MFMA_PEAK_TFLOPS, 4),
                      same_result=bool(torch.equal(eb, eb64)))
        del p64, e64, eb64, eb
    dom5 = k5["predict_linear"]
    result["linear_predictor"] = {
        "workload": f"S={lw.S} L={lw.L} H={lw.H} d={lw.d} n={lw.n} m={lw.m} V={lw.V}", "steps": lin_steps,
        "value": round(lw.kv_bytes / (dt5 / lin_steps) / 1e9, 2), "unit": "GB/s",
        "ms_per_step": round(dt5 / lin_steps * 1e3, 4),
        "roofline": dict(bound="mfma", kernel="gemm_nt_direct_kernel<EncodeLinear>", achieved=dom5["TFLOPs"],
                         peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=dom5["frac_mfma"], traffic=None),
        "kernels": k5, "kernels_ms": {k: round(v, 4) for k, v in ms5.items()},
        "payload_bits_per_symbol": round((16 * nw5 + 16 * esc5) / E5, 4),
        "escape_rate": round(esc5 / E5, 6),
        "roundtrip_symbols_exact": bool(torch.equal(codec5.dec_symbols, codec5.symbols)),
        "max_abs_reconstruction_error": round(err5, 6),
        "expected_embedding_padded_vocabulary": padded,
    }
    log(f"  linear predictor: step {result['linear_predictor']['ms_per_step']} ms ({result['linear_predictor']['value']} GB/s); "
        + ", ".join(f"{k} {v['ms']} ms = {v['TFLOPs']} TFLOP/s ({100 * v['frac_mfma']:.1f} % of fp16 MFMA peak)"
                    for k, v in k5.items())
        + (f"; expected embedding with the vocabulary padded to {padded['V']}: {padded['ms']} ms = {padded['TFLOPs']} TFLOP/s" if padded else ""))
    del codec5, lw, lo_k, lo_v
    torch.cuda.empty_cache()


def prefix_index(plc, result):
    """The host-side prefix index in front of the path: 2,000 sessions of 2,048 tokens that share prefixes
    (each continues a random earlier session from a random depth), inserted, looked up and evicted."""
    import numpy as np
    rng = np.random.default_rng(0)
    sessions = []
    for i in range(2000):
        tail = rng.integers(0, 50000, 2048).astype(np.int32)
        if sessions and rng.random() < 0.8:
            base = sessions[int(rng.integers(len(sessions)))]
            cut = int(rng.integers(0, 2048))
            tail[:cut] = base[:cut]
        sessions.append(tail)
    bits = np.full(2048, 3.9, dtype=np.float32)
    trie = plc.PrefixTrie()
    t0 = time.perf_counter()
    for i, sess in enumerate(sessions):
        trie.insert(sess, i, bits)
    t1 = time.perf_counter()
    hits = sum(trie.best_match(sess)[1] == 2048 for sess in sessions)
    t2 = time.perf_counter()
    nodes = trie.nodes
    for i in range(len(sessions)):
        trie.evict(i)
    t3 = time.perf_counter()
    tok = len(sessions) * 2048
    result["prefix_index"] = {"sessions": len(sessions), "tokens_per_session": 2048, "nodes": nodes,
                              "insert_Mtokens_per_s": round(tok / (t1 - t0) / 1e6, 2),
                              "best_match_Mtokens_per_s": round(tok / (t2 - t1) / 1e6, 2),
                              "evict_Mtokens_per_s": round(tok / (t3 - t2) / 1e6, 2),
                              "exact_matches": int(hits), "empty_after_evict": trie.nodes == 1, "threads": 1}
    log(f"  prefix index (host, 1 thread): insert {result['prefix_index']['insert_Mtokens_per_s']} M tokens/s, "
        f"best match {result['prefix_index']['best_match_Mtokens_per_s']}, evict {result['prefix_index']['evict_Mtokens_per_s']}; "
        f"{nodes} nodes for {tok} tokens")
    trie.close()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this path is built and measured on ONE GPU; streams are independent units, so more GPUs "
            "only split the stream list.  Run with --gpus 1.")
        sys.exit(2)
    import torch
    from paper_2604_15356_amd import plc

    plc.lib()                                   # fails loudly if libplc.so is missing
    torch.cuda.set_device(torch.device("cuda:0"))
    headline = args.config
    others = [] if args.no_other_configs else [c for c in ALL_CONFIGS if c != headline]
    sides = {}      # side measurements, all on the Llama-shaped workload
    configs = {}
    cpu_extra = {}

    def llama_extras(run):
        """What is measured on the Llama-shaped workload besides its own step."""
        if not args.no_side_paths:
            side_paths(run, args, plc, torch, sides)
        if not args.no_cpu_baseline and headline != "llama8b":
            base, check = cpu_baseline(run, run.w.n_streams, torch)     # the whole configuration
            cpu_extra["llama8b_whole"] = dict(base, **check)

    # The headline workload first, on a device nothing else has used yet (its 190 GB placed after other workloads
    # were drawn and freed measured up to 8 % slower), then the other configurations, each freed before the next.
    run = Run(headline, args, torch)
    res = time_run(run, args, plc, torch, calibrate=args.calibrate_copy)
    if headline == "llama8b" and not args.sessions:
        llama_extras(run)
    result = {
        "metric": "fp16 KV GB/s delta-coded (encode+decode)", "value": res["value"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    result.update({k: v for k, v in res.items() if k not in ("value", "unit", "ms_per_step")})
    result["paper_context"] = ("theoretical bound 3.3-4.3 bits per token position at perplexity 10-20 (abstract); "
                               "no measured figure")
    base = None
    if not args.no_cpu_baseline:
        w = run.w
        n_cpu = w.n_streams if headline == "llama8b" else \
            (min(w.S, args.cpu_sessions) * w.L * w.H if headline == "batched" else min(args.cpu_streams, w.n_streams))
        base, check = cpu_baseline(run, n_cpu, torch)
        result["cpu_baseline"] = base
        result.update(check)
    run.close()
    if headline == "llama8b" and not args.sessions and not args.no_side_paths and not args.no_linear:
        linear_path(args, plc, torch, sides, args.chunk_syms)

    for name in others:
        run = Run(name, args, torch, layout="lhnkd", chunk_syms=0)
        configs[name] = time_run(run, args, plc, torch)
        if name == "llama8b":
            llama_extras(run)
        run.close()
        if name == "llama8b" and not args.no_side_paths:
            if not args.no_lnkhd:
                # the same workload with the candidates stored [L,n,k,H,d] (heads innermost but one), addressed
                # through the strides of plc_dims: same logical values, same symbols, another memory order
                run = Run(name, args, torch, layout="lnkhd", chunk_syms=0)
                sides["layout_lnkhd"] = time_run(run, args, plc, torch)
                run.close()
            if not args.no_linear:
                linear_path(args, plc, torch, sides, 0)
    if base is not None:
        base.update(cpu_extra)
    if configs:
        result["configs"] = configs
    result.update(sides)
    if not args.no_prefix_index and not args.no_side_paths:
        prefix_index(plc, result)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
