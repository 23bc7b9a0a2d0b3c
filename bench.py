"""Benchmark of the Helix decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gqa_share] [--split-tokens T]

One step = one pass of the whole hot path over one batch of synthetic input already resident in
HBM: the KVP cut of every sequence, the streaming attention over every shard, the merge of the split
records into per-shard (O_i, lse_i), and the LSE combine.  Prints ONE JSON line.  The metric is the
achieved HBM rate of KV streaming: algorithmic KV bytes of the step (Appendix A's numerator for the
workload's shapes) divided by the step time.

The headline (`value`, `config`, `roofline`, `cpu_baseline`) is the workload given by --workload.  With
the default workload the same line also carries, under `configs`, one entry per remaining benchmark
configuration (same K and W, each with its own roofline and a bounded cpu_baseline), under `kv_formats`
the same for the GQA / MLA shares with an e4m3 or MXFP4 cache, and, under
`ceilings`, what the part sustains for a bare streaming read with the GQA launch shape and for an
LDS-fed MFMA loop (the two probes of the library) -- so that every fraction quoted anywhere is on
the clock of this one run.
"""
import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 and fp16
HEADLINE = "gqa_share"
OTHER_CONFIGS = ["tiny_gqa", "mla_share", "gqa_full", "mla_fp8_ragged"]   # the remaining benchmark configurations
# the GQA and MLA shares with the KV cache in the low-precision formats the library also streams (Sec. 3: FP4 KV states)
KV_FORMATS = ["gqa_share_fp8", "gqa_share_mxfp4", "mla_share_mxfp4"]


def kv_bytes_per_step(w, lens) -> int:
    """Algorithmic bytes: every stored K and V element of every token is read exactly once; an MLA
    latent row serves as key and value and counts once; fp8 rows carry one fp32 scale, MXFP4 rows
    half a byte per element plus one scale byte per 32 elements."""
    tokens = int(sum(int(x) for x in lens))
    if w.mla and getattr(w, "fp4", False):
        per_token = w.dk // 2 + w.dk // 32
    elif w.mla:
        per_token = w.dk * (1 if w.fp8 else 2) + (4 if w.fp8 else 0)
    elif getattr(w, "fp4", False):
        per_token = (w.dk + w.dv) // 2 + (w.dk + w.dv) // 32
    elif w.fp8:
        per_token = (w.dk + w.dv) + 4
    else:
        per_token = (w.dk + w.dv) * 2
    return tokens * w.K * per_token


def flops_per_step(w, lens) -> int:
    tokens = int(sum(int(x) for x in lens))
    return 2 * (w.dk + w.dv) * tokens * w.Q


class HipEvents:
    """Raw hipEvent_t pairs from the HIP runtime torch loaded (ctypes)."""

    def __init__(self, n):
        import torch
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        self.hip = ctypes.CDLL(path)
        self.start = [ctypes.c_void_p() for _ in range(n)]
        self.stop = [ctypes.c_void_p() for _ in range(n)]
        for e in self.start + self.stop:
            assert self.hip.hipEventCreate(ctypes.byref(e)) == 0

    def elapsed_ms(self, i) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.start[i], self.stop[i])
        assert rc == 0, f"hipEventElapsedTime -> {rc}"
        return ms.value

    def destroy(self):
        for e in self.start + self.stop:
            self.hip.hipEventDestroy(e)


def cpu_baseline(w, inp, budget_macs=1.5e11):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same
    workload: the first nb sequences with all their heads over their full length, nb chosen so that
    the sample is at most ~budget_macs multiply-adds (10-30 s of CPU work at most)."""
    import numpy as np
    import oracle
    import synth
    lens = inp.lens.numpy()
    if w.fp8 or getattr(w, "fp4", False):
        budget_macs /= 8          # decoding codes element by element is that much slower in the oracle
    per_seq = lens.astype(np.float64) * w.Q * (w.dk + w.dv)
    nb = int(max(1, min(w.B, np.searchsorted(np.cumsum(per_seq), budget_macs, side="right"))))
    q = synth.bits(inp.q[:nb])
    kw = dict(kv_heads=w.K, dv=w.dv)
    if inp.seq_off is not None:                       # packed ragged latent
        hi = int(inp.seq_off[nb])
        k, v = synth.bits(inp.k[:hi]), None
        kw["tok_off"] = inp.seq_off[:nb].numpy()
        if inp.k_mx is not None:
            kw["mx"] = (inp.k_mx[:hi].cpu().numpy(), None)
        if inp.kv_scale is not None:
            kw["kv_scale"] = inp.kv_scale[:hi].cpu().numpy()
    else:
        k = synth.bits(inp.k[:nb])
        v = synth.bits(inp.v[:nb]) if inp.v is not None else None
        if inp.kv_scale is not None:
            kw["kv_scale"] = inp.kv_scale[:nb].cpu().numpy()
        if inp.k_mx is not None:
            kw["mx"] = (inp.k_mx[:nb].cpu().numpy(), None if inp.v_mx is None else inp.v_mx[:nb].cpu().numpy())
    t0 = time.perf_counter()
    oracle.attention(q, k, v, lens[:nb], w.scale, **kw)
    dt = time.perf_counter() - t0
    sample_bytes = kv_bytes_per_step(w, lens[:nb])
    return {"value": sample_bytes / dt / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first {nb} of {w.B} sequences, all {w.Q} heads, {int(lens[:nb].sum())} tokens, fp64, {dt:.1f} s",
            "seconds": dt}


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (the counters
    cannot be read from inside this process; the file names the commands that produced it)."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def kernel_name(w) -> str:
    if w.mla:
        return "mla_decode_kernel<" + ("mxfp4" if getattr(w, "fp4", False) else "e4m3" if w.fp8 else "bf16") + ">"
    shared = "true" if w.Q // w.K > 16 else "false"        # several head tiles per KV head: the variant whose loads stay in the L2
    if getattr(w, "fp4", False):
        return f"gqa_mxfp4_kernel<{shared}>"
    return f"gqa_fp8_kernel<{shared}>" if w.fp8 else f"gqa_decode_kernel<{w.dk}, {shared}>"


def measure(name, args, budget_macs, extras=False):
    """Times workload `name`: K steps of the whole path, then the same K steps through the timed entry
    point (an event pair around the streaming kernel of every step).  Returns the entry of the JSON line."""
    import torch
    import paper_2507_07120_amd as hx
    import synth
    from paper_2507_07120_amd import harness

    dev = "cuda:0"
    w = synth.WORKLOADS[name]
    inp = synth.make_inputs(w, dev)
    prob = harness.problem_for(w, args.split_tokens)
    lens_dev = inp.lens.to(dev)
    seq_base = inp.seq_off[:-1].to(dev) if inp.seq_off is not None else None
    N = w.n_shards
    shard_off = torch.empty((N, w.B), dtype=torch.int64, device=dev)
    shard_len = torch.empty((N, w.B), dtype=torch.int32, device=dev)
    max_len = int(inp.lens.max())
    if inp.k_mx is not None:
        cache = hx.KVShard.from_mxfp4(inp.k, inp.v, inp.k_mx, inp.v_mx, lens_dev, max_len, tok_off=seq_base)
    elif inp.k.dim() == 2:
        cache = hx.KVShard.from_packed(inp.k, lens_dev, max_len, seq_base, kv_scale=inp.kv_scale)
    else:
        cache = hx.KVShard.from_padded(inp.k, inp.v, lens_dev, max_len, kv_scale=inp.kv_scale)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    cache.status = status                     # device word: sequences beyond max_len (bit 0), moved MLA reference exponents (>> 8)
    ws = harness.workspace_for(prob, N, max_len, dev)
    o = torch.empty((w.B, w.Q, w.dv), device=dev)
    lse = torch.empty((w.B, w.Q), device=dev)

    # the explicit shard descriptors (the two-call form of the step, HOP-B, and the plan that is reported)
    ss = harness.make_shards(inp.k, inp.v, lens_dev, N, kv_scale=inp.kv_scale, seq_base=seq_base,
                             mx=None if inp.k_mx is None else (inp.k_mx, inp.v_mx))
    split_tokens, workgroups = hx.helix_attn_plan(prob, ss.max_lens)

    # one step = the whole path over one batch: the KVP cut of every sequence (integer metadata, written
    # out), the per-slice attention fragments, and their combine
    if args.two_call:
        def step(events=None):
            hx.helix_shard_layout(lens_dev, N, shard_off, shard_len, seq_base=seq_base)
            hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    else:
        def step(events=None):
            hx.helix_attn_decode_kvp(prob, inp.q, cache, N, o, ws, lse_out=lse, shard_off=shard_off, shard_len=shard_len,
                                     events=events)

    def timed_step(events):
        # the streaming kernel is the same in both forms of the step; only this entry point takes events
        hx.helix_attn_decode_kvp(prob, inp.q, cache, N, o, ws, lse_out=lse, shard_off=shard_off, shard_len=shard_len, events=events)

    if extras and args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_seconds:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    status.zero_()
    torch.cuda.synchronize()
    # timed region: exactly K steps, nothing else on the stream
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    status_word = int(status.item())
    # the same K steps again with a hipEvent pair recorded around the streaming kernel of every step
    # (the event packets sit between the kernels and cost a few microseconds per step, so they stay
    # out of the region `value` is computed from; that region's own duration is reported alongside)
    ev = HipEvents(args.steps)
    t1 = time.perf_counter()
    for i in range(args.steps):
        timed_step((ev.start[i], ev.stop[i]))
    torch.cuda.synchronize()
    dt_hooked = time.perf_counter() - t1
    kern_ms = sorted(ev.elapsed_ms(i) for i in range(args.steps))
    ev.destroy()
    kern_avg_ms = sum(kern_ms) / len(kern_ms)

    ms_per_step = dt / args.steps * 1e3
    kv_bytes = kv_bytes_per_step(w, inp.lens.tolist())
    flops = flops_per_step(w, inp.lens.tolist())
    value = kv_bytes / (ms_per_step * 1e-3) / 1e9
    hbm_of_kernel = kv_bytes / (kern_avg_ms * 1e-3) / 1e9
    if w.mla:
        achieved = flops / (kern_avg_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": flops}
    else:
        roof = {"bound": "hbm", "achieved": hbm_of_kernel, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_of_kernel / HBM_PEAK_GBS}
    roof["traffic"] = read_traffic(name)
    roof["traffic_source"] = None if roof["traffic"] is None else f"profiles/traffic_{name}.txt (rocprofv3 --pmc, committed)"
    roof["kernel"] = kernel_name(w)
    roof["kernel_us_avg"] = kern_avg_ms * 1e3
    roof["kernel_us_min"] = kern_ms[0] * 1e3
    roof["kernel_timing"] = ("hipEvent pair around the streaming kernel in a second loop of the same K steps "
                             "(helix_attn_decode_kvp_timed); that loop's step time is us_per_step_with_event_hooks")
    if w.mla:
        # (wavefront, tile) events in which a head's reference exponent had to move (see the header), per step
        roof["reference_moves_per_step"] = (status_word >> 8) / args.steps
    roof["status_bits"] = status_word & 0xFF
    roof["algorithmic_bytes"] = kv_bytes
    roof["hbm_gbs_of_kernel"] = hbm_of_kernel
    roof["hbm_frac_of_kernel"] = hbm_of_kernel / HBM_PEAK_GBS
    if name == "tiny_gqa":
        roof["note"] = "2 MiB of KV: launch- and latency-bound and cache-resident; the microseconds are the result"

    entry = {
        "ms_per_step": ms_per_step, "us_per_step": ms_per_step * 1e3,
        "us_per_step_with_event_hooks": dt_hooked / args.steps * 1e6,
        "value": value, "unit": "GB/s", "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        # arithmetic type of the contractions: the e4m3 and MXFP4 latents are widened to fp16 (same MFMA rate as bf16)
        "dtype": "f16" if (w.mla and (w.fp8 or getattr(w, "fp4", False))) else "bf16",
        "config": {"workload": w.name, "B": w.B, "q_heads": w.Q, "kv_heads": w.K, "dk": w.dk, "dv": w.dv,
                   "n_shards": N, "tokens_per_step": int(sum(inp.lens.tolist())) * w.K,
                   "kv_dtype": "e4m3+fp32 scale" if w.fp8 else "mxfp4 (e2m1 + e8m0 per 32)" if getattr(w, "fp4", False) else "bf16",
                   "split_tokens": split_tokens, "workgroups": workgroups,
                   "entry": "helix_shard_layout + helix_attn_decode" if args.two_call else "helix_attn_decode_kvp"},
        "roofline": roof,
    }
    if extras and args.graph > 0:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(args.graph):
                step()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        reps = max(1, args.steps // args.graph)
        tg = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        entry["graph"] = {"steps_per_graph": args.graph, "replays": reps,
                          "us_per_step": (time.perf_counter() - tg) / (reps * args.graph) * 1e6}
    if extras and args.hopb > 0:
        nbytes = hx.helix_attn_hopb_workspace_bytes(prob, N, max(ss.max_lens), args.hopb)
        ws_h = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        bufs = hx.HopbBuffers(prob, N, args.hopb, dev)
        cs, xs = torch.cuda.Stream(), torch.cuda.Stream()

        def timed(exchange_stream):
            for _ in range(args.warmup):
                hx.helix_attn_decode_hopb(prob, inp.q, ss.shards, o, ws_h, bufs, cs, exchange_stream, lse_out=lse)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(args.steps):
                hx.helix_attn_decode_hopb(prob, inp.q, ss.shards, o, ws_h, bufs, cs, exchange_stream, lse_out=lse)
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / args.steps * 1e6
        entry["hopb"] = {"groups": args.hopb, "us_per_step_two_streams": timed(xs), "us_per_step_one_stream": timed(cs),
                         "note": "per-shard attention + device copy of the fragments (stand-in for the All-to-All) + combine; "
                                 "no shard_layout call in these steps"}
    if not args.no_cpu_baseline:
        entry["cpu_baseline"] = cpu_baseline(w, inp, budget_macs)
    return entry


def ceilings(args):
    """The two probes of the library, timed with events on this run's clock: a bare streaming read with the
    GQA kernels' launch shape (256 workgroups of 4 waves, one contiguous chunk each) and 16x16x32 bf16 MFMAs
    fed from LDS, with Gaussian and with all-zero operands (the part's clock depends on the data)."""
    import torch
    import paper_2507_07120_amd as hx
    import synth
    dev = "cuda:0"
    out = {}
    buf = synth.normal_bf16(4242, 1, (1 << 29,), dev)                 # 1 GiB of N(0,1) bf16

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    # untimed, as before every workload: the driver clears memory a process has just given back (the previous
    # workload's tensors) in the background for a second or so, and a read probe started meanwhile measures 4-5 % low
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_seconds:
        for _ in range(20):
            hx.helix_probe_stream_read(buf, 256, True)
        torch.cuda.synchronize()
    for label, nt in (("stream_read_nontemporal", True), ("stream_read_plain", False)):
        nbytes = buf.numel() * 2
        s = timed(lambda: hx.helix_probe_stream_read(buf, 256, nt), max(5, min(args.steps, 50)))
        out[label] = {"GB/s": nbytes / s / 1e9, "us": s * 1e6, "bytes": nbytes, "workgroups": 256,
                      "frac_of_hbm_peak": nbytes / s / 1e9 / HBM_PEAK_GBS}
    iters = 16000
    zeros = torch.zeros(1 << 15, dtype=torch.bfloat16, device=dev)
    for label, operands, stream in (("mfma_lds_gauss", buf, None), ("mfma_lds_gauss_streaming", buf, buf),
                                    ("mfma_lds_zeros", zeros, None)):
        flops = [0.0, 0.0]

        def fn():
            flops[0], flops[1] = hx.helix_probe_mfma_lds(operands, iters, stream)
        s = timed(fn, 3)
        out[label] = {"TFLOP/s": flops[0] / s / 1e12, "ms": s * 1e3, "frac_of_mfma_peak": flops[0] / s / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        if stream is not None:
            out[label]["GB/s"] = flops[1] / s / 1e9
            out[label]["flop_per_byte"] = flops[0] / flops[1]
    out["note"] = ("stream_read_*: helix_probe_stream_read over 1 GiB; mfma_lds_*: helix_probe_mfma_lds, 8 waves per CU, "
                   "A operand from LDS at every MFMA, N(0,1) bf16 or zero operands; *_streaming adds 1 KB of HBM read per wave and 16 MFMAs")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--split-tokens", type=int, default=0)
    ap.add_argument("--settle-seconds", type=float, default=1.0,
                    help="untimed: repeat the step for this long before the warmup steps, so that the part's memory "
                         "and fabric clocks have left their idle state (a fresh process otherwise measures the ramp)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="with the default workload: leave out the other configurations and the ceiling probes")
    ap.add_argument("--two-call", action="store_true",
                    help="time the step as helix_shard_layout + helix_attn_decode (two entry points, one more "
                         "launch) instead of helix_attn_decode_kvp, which cuts the slices inside the kernel")
    ap.add_argument("--hopb", type=int, default=0, metavar="G",
                    help="also time the batch cut into G request groups whose exchange + combine run on a second "
                         "stream under the next group's attention (Sec. 2.1.3), against the same call on one stream")
    ap.add_argument("--graph", type=int, default=0, metavar="G",
                    help="also capture G consecutive steps into one HIP graph and time its replays (launch-bound "
                         "configurations: the library only enqueues kernels, so a step is capturable as it is)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (torch copy_) before the timed loop, so that a "
                         "rocprofv3 --pmc run holds a kernel of known traffic to scale the counters by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all KV shards live on it; there is no collective "
              "path). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2507_07120_amd as hx

    hx.load_library()                       # raises if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"

    head = measure(args.workload, args, budget_macs=1.5e11, extras=True)
    out = {
        "metric": "KV-shard decode attention achieved HBM GB/s (% of peak); us per decode step",
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "us_per_step": head["us_per_step"],
        "us_per_step_with_event_hooks": head["us_per_step_with_event_hooks"],
        "pct_of_hbm_peak": head["pct_of_hbm_peak"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic", "config": head["config"], "roofline": head["roofline"],
    }
    for k in ("graph", "hopb", "cpu_baseline"):
        if k in head:
            out[k] = head[k]
    if args.workload == HEADLINE and not args.headline_only:
        out["configs"] = []
        for name in OTHER_CONFIGS:
            gc.collect()
            torch.cuda.empty_cache()
            # a smaller oracle sample per extra configuration keeps the whole run within a couple of minutes
            out["configs"].append(measure(name, args, budget_macs=4e10))
        out["kv_formats"] = []
        for name in KV_FORMATS:
            gc.collect()
            torch.cuda.empty_cache()
            out["kv_formats"].append(measure(name, args, budget_macs=2e10))
        gc.collect()
        torch.cuda.empty_cache()
        out["ceilings"] = ceilings(args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
