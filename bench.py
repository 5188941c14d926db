#!/usr/bin/env python3
"""Benchmark of the KDA hot path on one MI355X.

A "step" is one pass of the hot path over one batch of synthetic input.  The headline is the
chunkwise prefill (kda_chunk_fwd) on the largest single-GPU workload, the 2^20-token long-context
prefill (cfg3_long_bf16): `value` is its tokens/s, timed over K steps with the inputs resident in
HBM, bracketed by device synchronisation and measured with HIP events on the launch stream.  The
other bf16 prefill workloads (cfg1, cfg2) and the decode workload (cfg4: one kda_recurrent_step
over the 512 MiB state pool) are timed the same way and reported as sub-objects, each with its own
`roofline` and `cpu_baseline`.

Prints ONE JSON line.  Runs on one GPU only.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Published MI355X peaks used for the roofline fractions.
HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0          # dense fp16/bf16 matrix cores

# Algorithmic work per (token, head) at d_k = d_v = 128, C = 64.
FLOP_PER_TOKHEAD = 6 * 128 * 128 + 3 * 64 * 128 + 64 * 64        # paper's FLOPs model: 126976
BYTES_PER_TOKHEAD = (3 * 128 + 128) * 2 + 2 + 128 * 4            # q,k,log_alpha,v,beta bf16 + o fp32: 1538

HEADLINE = "cfg3_long_bf16"
PREFILL_WORKLOADS = ("cfg3_long_bf16", "cfg1_prefill_bf16", "cfg2_varlen_bf16")


def measured_traffic(workload):
    """HBM bytes per launch of the workload's call, from the rocprofv3 counter summary committed
    under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what it reads for a plain copy of
    known size; the file states the command).  Returns (bytes or None, file name or None)."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None, None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
    return (float(m.group(1)) if m else None), os.path.relpath(path, ROOT)


def _time_region(torch, fn, steps):
    """Time `steps` calls of fn() with HIP events on the current stream; returns ms per call."""
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / steps


def make_workload(torch, si, name, dev):
    """Device tensors of one prefill workload: (x, tokens, max_len, config description)."""
    c = si.CONFIGS[name]
    if name == "cfg1_prefill_bf16":
        host = si.make_prefill(c["B"], c["T"], c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], c["h0_std"])
        x = {k_: (v_.to(dev) if isinstance(v_, torch.Tensor) else v_) for k_, v_ in host.items()}
        return x, c["B"] * c["T"], 0, {"workload": name, "B": c["B"], "T": c["T"], "H": c["H"], "dk": c["dk"],
                                      "dv": c["dv"], "chunk": 64}
    if name == "cfg2_varlen_bf16":
        lens = si.varlen_lengths(c["N"], c["len_lo"], c["len_hi"], c["seed"])
        host = si.make_varlen(lens, c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], c["h0_std"])
        x = {k_: (v_.to(dev) if isinstance(v_, torch.Tensor) else v_) for k_, v_ in host.items()}
        return x, int(lens.sum()), int(lens.max()), {"workload": name, "num_seqs": c["N"], "total_tokens": int(lens.sum()),
                                                      "H": c["H"], "dk": c["dk"], "dv": c["dv"], "chunk": 64}
    if name == "cfg3_long_bf16":
        x = si.make_long_on_device(c["T"], c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], dev)
        x["h0"] = None
        x["cu_seqlens"] = None
        return x, c["T"], 0, {"workload": name, "B": 1, "T": c["T"], "H": c["H"], "dk": c["dk"], "dv": c["dv"],
                              "chunk": 64}
    raise SystemExit("unknown workload " + name)


def run_prefill(torch, si, kda, name, steps, warmup, dev, cpu_seconds):
    """Times kda_chunk_fwd on one workload; returns the result object (ms, tokens/s, roofline, cpu_baseline)."""
    c = si.CONFIGS[name]
    x, tokens, max_len, desc = make_workload(torch, si, name, dev)
    H = c["H"]
    tokheads = tokens * H
    dims = kda.kda.make_chunk_dims(x["q"], x["v"], x["cu_seqlens"], 1.0, max_len)
    ws = torch.empty(kda.kda_chunk_fwd_workspace_size(dims), dtype=torch.uint8, device=dev)
    o = torch.empty(x["q"].shape[0], x["q"].shape[1], H, c["dv"], dtype=torch.float32, device=dev)
    hT = torch.empty(dims.num_seqs, H, c["dk"], c["dv"], dtype=torch.float32, device=dev)

    def prefill():
        kda.kda_chunk_fwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], h0=x["h0"],
                          cu_seqlens=x["cu_seqlens"], o=o, hT=hT, workspace=ws, max_seqlen=max_len)

    for _ in range(warmup):
        prefill()
    ms = _time_region(torch, prefill, steps)
    kda.kda_chunk_fwd_check(dims, ws)            # raises if the call reported a failed wait: outputs would be invalid

    alg_bytes = tokheads * BYTES_PER_TOKHEAD + 2 * dims.num_seqs * H * 128 * 128 * 4
    traffic, traffic_file = measured_traffic(name)
    roofline = {
        # one kernel per call (both stages are roles of kda_prefill_kernel), so the kernel's duration is the
        # call's own (HIP events on the launch stream around K calls)
        "kernel": "kda_prefill_kernel",
        "bound": "hbm",
        "achieved": alg_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": traffic, "traffic_source": traffic_file,
        "ms_kernel": ms,
        "algorithmic_bytes": alg_bytes,
        "mfma_frac_model_flops": tokheads * FLOP_PER_TOKHEAD / (ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
        "model_tflops": tokheads * FLOP_PER_TOKHEAD / (ms * 1e-3) / 1e12,
    }
    res = {"metric": "KDA prefill tokens/s", "value": tokens / (ms * 1e-3), "unit": "tokens/s",
           "ms_per_step": ms, "steps": steps, "warmup": warmup, "config": desc,
           "tokheads_per_s": tokheads / (ms * 1e-3), "workspace_bytes": int(ws.numel()), "roofline": roofline}

    if cpu_seconds > 0:
        import oracle
        # bounded sample: a prefix of every (sequence, head), sized so the fp64 recurrence runs for seconds
        n_s = min(16384 if name == HEADLINE else 4096, x["q"].shape[1])
        if x["cu_seqlens"] is None:
            a = {k_: si.to_np32(x[k_][:, :n_s]) for k_ in ("q", "k", "v", "log_alpha", "beta")}
            sample_tokens = x["q"].shape[0] * n_s
            what = "first %d tokens of every sequence" % n_s
            kw = {}
        else:
            import numpy as np
            a = {k_: si.to_np32(x[k_]) for k_ in ("q", "k", "v", "log_alpha", "beta")}
            sample_tokens = tokens
            what = "the whole packed batch"
            kw = {"cu_seqlens": x["cu_seqlens"].cpu().numpy().astype(np.int64)}
        reps, dt = 0, 0.0
        t0 = time.perf_counter()
        while dt < cpu_seconds and reps < 50:
            oracle.kda_forward(a["q"], a["k"], a["v"], a["log_alpha"], a["beta"], want_hT=False, **kw)
            reps += 1
            dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": sample_tokens * reps / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": "%s of %s (x %d heads), %d time(s) over, fp64 per-token recurrence"
                                         % (what, name, H, reps),
                               "seconds": dt}
    del x, ws, o, hT
    torch.cuda.empty_cache()
    return res


def run_decode(torch, si, kda, steps, warmup, dev, cpu_baseline):
    d4 = si.CONFIGS["cfg4_decode_bf16"]
    N4, H4, dk4, dv4 = d4["N"], d4["H"], d4["dk"], d4["dv"]
    S = si.make_state(N4, H4, dk4, dv4, d4["state_std"], d4["seed"]).to(dev)
    tok_host = si.make_decode_tokens(N4, H4, dk4, dv4, d4["dtype"], d4["mu"], d4["seed"], 0)
    tk = {k_: v_.to(dev) for k_, v_ in tok_host.items()}
    o4 = torch.empty(N4, H4, dv4, dtype=torch.float32, device=dev)

    def decode():
        kda.kda_recurrent_step(tk["q"], tk["k"], tk["v"], tk["log_alpha"], tk["beta"], S, o=o4)

    for _ in range(warmup):
        decode()
    ms_decode = _time_region(torch, decode, steps)
    dec_bytes = 2 * N4 * H4 * dk4 * dv4 * 4 + N4 * H4 * ((3 * dk4 + dv4) * 2 + 2) + N4 * H4 * dv4 * 4
    traffic, traffic_file = measured_traffic("cfg4_decode_bf16")
    obj = {
        "metric": "decode-step state GB/s", "value": dec_bytes / (ms_decode * 1e-3) / 1e9, "unit": "GB/s",
        "ms_per_step": ms_decode, "steps": steps,
        "config": {"workload": "cfg4_decode_bf16", "num_seqs": N4, "H": H4, "dk": dk4, "dv": dv4,
                   "state_bytes": N4 * H4 * dk4 * dv4 * 4},
        "roofline": {"kernel": "kda_step_kernel", "bound": "hbm",
                     "achieved": dec_bytes / (ms_decode * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dec_bytes / (ms_decode * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_file, "ms_kernel": ms_decode,
                     "algorithmic_bytes": dec_bytes},
    }

    # pooled multi-token decode: the same 256 x 32 states addressed through a permuted index array,
    # four tokens per sequence and call (state traffic is paid once per call, not once per token)
    Tq = 4
    perm = torch.randperm(N4, generator=torch.Generator().manual_seed(d4["seed"])).to(torch.int32).to(dev)
    mt_host = [si.make_decode_tokens(N4, H4, dk4, dv4, d4["dtype"], d4["mu"], d4["seed"], 1 + t) for t in range(Tq)]
    mt = {k_: torch.stack([t_[k_] for t_ in mt_host], dim=1).contiguous().to(dev) for k_ in mt_host[0]}
    o4m = torch.empty(N4, Tq, H4, dv4, dtype=torch.float32, device=dev)

    def decode_pooled():
        kda.kda_recurrent_steps_pooled(mt["q"], mt["k"], mt["v"], mt["log_alpha"], mt["beta"], S, perm, o=o4m)

    for _ in range(warmup):
        decode_pooled()
    ms_pooled = _time_region(torch, decode_pooled, steps)
    pooled_bytes = 2 * N4 * H4 * dk4 * dv4 * 4 + Tq * (N4 * H4 * ((3 * dk4 + dv4) * 2 + 2) + N4 * H4 * dv4 * 4)
    obj["pooled_multi_token"] = {
        "tokens_per_call": Tq, "ms_per_call": ms_pooled,
        "decode_tokens_per_s": N4 * Tq / (ms_pooled * 1e-3),
        "single_token_decode_tokens_per_s": N4 / (ms_decode * 1e-3),
        "achieved_GBps": pooled_bytes / (ms_pooled * 1e-3) / 1e9,
        "hbm_frac": pooled_bytes / (ms_pooled * 1e-3) / 1e9 / HBM_PEAK_GBS,
    }

    # what a plain device-to-device copy reaches on this GPU (bytes read + written per second)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ms_copy = _time_region(torch, lambda: dst.copy_(src), 10)
    copy_gbs = 2 * src.numel() / (ms_copy * 1e-3) / 1e9
    del src, dst
    obj["roofline"]["measured_copy_GBps"] = copy_gbs
    obj["roofline"]["frac_of_measured_copy"] = obj["value"] / copy_gbs

    # what this device streams with the simplest kernels: 512 MiB (the size of the state pool) read only, written
    # only, and read-modified-written in place, which is the traffic of the decode step
    buf = torch.empty(N4 * H4 * dk4 * dv4, dtype=torch.float32, device=dev)
    rates = {}
    for mode, name in ((0, "read_only"), (1, "write_only"), (2, "read_modify_write_in_place")):
        kda.kda_debug_stream_probe(mode, buf)
        ms = _time_region(torch, lambda: kda.kda_debug_stream_probe(mode, buf), 20)
        rates[name + "_GBps"] = (2 if mode == 2 else 1) * buf.numel() * 4 / (ms * 1e-3) / 1e9
    del buf
    obj["roofline"]["measured_stream"] = rates
    obj["roofline"]["frac_of_measured_read_modify_write"] = obj["value"] / rates["read_modify_write_in_place_GBps"]

    if cpu_baseline:
        import numpy as np
        import oracle
        Sh = S.cpu().numpy().astype(np.float64)
        args = [si.to_np32(tok_host[n_]) for n_ in ("q", "k", "v", "log_alpha", "beta")]
        reps, dt = 0, 0.0
        t0 = time.perf_counter()
        while dt < 5.0 and reps < 50:
            oracle.kda_step(*args, Sh)
            reps += 1
            dt = time.perf_counter() - t0
        obj["cpu_baseline"] = {"value": dec_bytes * reps / dt / 1e9, "unit": "GB/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "one decode step over the whole cfg4 state pool, %d time(s) over, fp64" % reps,
                               "seconds": dt}
    del S
    torch.cuda.empty_cache()
    return obj


def run_extras(torch, si, kda, steps, warmup, dev, cpu_baseline):
    """Other entry points on the cfg1 shape: bf16 outputs, scalar gate, fused stages, backward."""
    name = "cfg1_prefill_bf16"
    c = si.CONFIGS[name]
    x, tokens, _, _ = make_workload(torch, si, name, dev)
    H = c["H"]
    tokheads = tokens * H
    dims = kda.kda.make_chunk_dims(x["q"], x["v"], None, 1.0, 0)
    ws = torch.empty(kda.kda_chunk_fwd_workspace_size(dims), dtype=torch.uint8, device=dev)
    o = torch.empty(c["B"], c["T"], H, c["dv"], dtype=torch.float32, device=dev)
    hT = torch.empty(c["B"], H, c["dk"], c["dv"], dtype=torch.float32, device=dev)
    out = {}

    def timed(fn):
        for _ in range(warmup):
            fn()
        ms = _time_region(torch, fn, steps)
        return {"ms_per_step": ms, "tokens_per_s": tokens / (ms * 1e-3)}

    o16 = torch.empty(o.shape, dtype=torch.bfloat16, device=dev)
    out["prefill_bf16_out"] = dict(what="cfg1 shape, out_dtype bf16 (o rounded once at the store)", **timed(
        lambda: kda.kda_chunk_fwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], h0=x["h0"], o=o16, hT=hT, workspace=ws)))
    del o16
    gh = x["log_alpha"][..., 0].contiguous()
    out["prefill_scalar_gate"] = dict(what="kda_chunk_fwd_scalar_gate on the cfg1 shape (the decay of channel 0 taken for the whole head)", **timed(
        lambda: kda.kda_chunk_fwd_scalar_gate(x["q"], x["k"], x["v"], gh, x["beta"], h0=x["h0"], o=o, hT=hT, workspace=ws)))
    del gh

    rawx = si.make_raw_tokens(c["B"], c["T"], H, c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"])
    rx = {k_: v_.to(dev) for k_, v_ in rawx.items()}
    fused = {"what": "kda_chunk_fwd_fused on the cfg1 shape: (a) input prologue (L2Norm(q), L2Norm(k), Sigmoid(beta), decay "
                     "function) inside the per-chunk kernel; (b) plus the output gate Sigmoid(g) * RMSNorm(o) inside the "
                     "sequential kernel"}
    fused["prologue"] = timed(lambda: kda.kda_chunk_fwd_fused(rx["q_raw"], rx["k_raw"], rx["v"], rx["gate"], rx["beta_logit"],
                                                              h0=x["h0"], o=o, hT=hT, workspace=ws))
    og = torch.randn(c["B"], c["T"], H, c["dv"], generator=torch.Generator().manual_seed(c["seed"])).to(torch.bfloat16).to(dev)
    nw = torch.ones(c["dv"], dtype=torch.float32, device=dev)
    ws_g = torch.empty(kda.kda_chunk_fwd_workspace_size(dims, output_gate=True), dtype=torch.uint8, device=dev)
    fused["prologue_and_output_gate"] = timed(lambda: kda.kda_chunk_fwd_fused(
        rx["q_raw"], rx["k_raw"], rx["v"], rx["gate"], rx["beta_logit"], out_gate=og, norm_weight=nw, h0=x["h0"], o=o, hT=hT,
        workspace=ws_g))
    out["prefill_fused_stages"] = fused
    del ws_g, og, rx

    # the backward pass (kda_chunk_bwd, fp32 throughout): time per call, and its rate against the fp32 vector
    # peak under a FLOP model of the chunkwise backward (per chunk and head: eight C x d x d products, eight
    # half-filled C x C x d ones, the C x C x C chain)
    d_o = torch.randn(o.shape, generator=torch.Generator().manual_seed(c["seed"] + 1)).to(dev)
    ws_b = torch.empty(kda.kda_chunk_bwd_workspace_size(dims), dtype=torch.uint8, device=dev)
    grads = kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], d_o, h0=x["h0"], workspace=ws_b)

    def backward():
        return kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], d_o, h0=x["h0"], workspace=ws_b, out=grads)
    backward()
    steps_b = max(3, min(steps, 10))
    ms_bwd = _time_region(torch, backward, steps_b)
    C_, D_ = 64, c["dk"]
    flop_chunk = 8 * 2 * C_ * D_ * D_ + 8 * C_ * C_ * D_ + 3 * 2 * C_ * C_ * C_
    tflops = tokheads / C_ * flop_chunk / (ms_bwd * 1e-3) / 1e12
    traffic, traffic_file = measured_traffic("backward_cfg1")
    out["backward"] = {"what": "kda_chunk_bwd on the cfg1 shape: gradients of q, k, v, log_alpha, beta, h0 (fp32 arithmetic)",
                       "ms_per_step": ms_bwd, "steps": steps_b, "tokens_per_s": tokens / (ms_bwd * 1e-3),
                       "roofline": {"bound": "alu", "achieved": tflops, "peak": 157.3, "unit": "TFLOP/s",
                                    "frac": tflops / 157.3, "flop_per_chunk_head": flop_chunk, "traffic": traffic,
                                    "traffic_source": traffic_file}}
    del d_o, ws_b, grads, x, ws, o, hT
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true",
                    help="also time the other entry points on the cfg1 shape (bf16 outputs, scalar gate, fused "
                         "stages, backward)")
    ap.add_argument("--only", default=None,
                    help="time just this workload (cfg1_prefill_bf16, cfg2_varlen_bf16, cfg3_long_bf16 or "
                         "cfg4_decode_bf16), with no CPU baseline: what a profiler run wants")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run a plain 1 GiB device copy three times, so that a byte counter collected over "
                         "this run can be scaled by what it reads for a transfer of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as si
    import paper_2510_26692_amd as kda

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = not args.no_cpu_baseline and args.only is None
    results = {}
    for name in PREFILL_WORKLOADS:
        if args.only not in (None, name):
            continue
        # the small workloads take well under a millisecond per step: more steps for a steady figure
        steps = args.steps if name == HEADLINE else max(args.steps, 50)
        warmup = args.warmup if name == HEADLINE else max(args.warmup, 10)
        results[name] = run_prefill(torch, si, kda, name, steps, warmup, dev, 10.0 if cpu else 0.0)
    decode_obj = None
    if args.only in (None, "cfg4_decode_bf16"):
        decode_obj = run_decode(torch, si, kda, max(args.steps, 50), max(args.warmup, 10), dev, cpu)
    extras = run_extras(torch, si, kda, max(args.steps, 50), max(args.warmup, 10), dev, cpu) if args.extras else None

    head = results.get(HEADLINE) or next(iter(results.values()), None) or decode_obj
    if args.only is None:
        # what the matrix cores of this device deliver on the prefill's own instruction, beside the data-sheet peak
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        wgs = 8 * torch.cuda.get_device_properties(0).multi_processor_count
        flops = kda.kda_debug_mfma_probe(sink, wgs, 2000)
        ms_mfma = _time_region(torch, lambda: kda.kda_debug_mfma_probe(sink, wgs, 2000), 5)
        head["roofline"]["measured_mfma_f16_TFLOPs"] = flops / (ms_mfma * 1e-3) / 1e12
        head["roofline"]["mfma_peak_TFLOPs"] = MFMA_PEAK_TFLOPS
        # the data movement of the two-stage design per (chunk, head) and nothing else (64 KiB in, a 72 KiB slot
        # written and read back, 32 KiB out), by a plain kernel on 65 536 items (the item count of a prefill of
        # 2^17 tokens x 32 heads): the level a prefill that is bound by its own traffic is read against
        tbuf = torch.empty(65536 * 172032, dtype=torch.uint8, device=dev)
        items, moved = kda.kda_debug_prefill_traffic_probe(tbuf)
        ms_t = _time_region(torch, lambda: kda.kda_debug_prefill_traffic_probe(tbuf), 5)
        del tbuf
        ns_item = ms_t * 1e6 / items
        head["roofline"]["two_stage_traffic_probe"] = {
            "ns_per_chunk_head": ns_item, "moved_GBps": moved / (ms_t * 1e-3) / 1e9,
            "bytes_per_chunk_head": moved // items}
        for r_ in results.values():
            chunk_heads = r_["tokheads_per_s"] * r_["ms_per_step"] * 1e-3 / 64.0
            r_["roofline"]["probe_time_over_kernel_time"] = ns_item * chunk_heads * 1e-6 / r_["ms_per_step"]
            if r_["roofline"].get("traffic"):
                r_["roofline"]["moved_GBps"] = r_["roofline"]["traffic"] / (r_["ms_per_step"] * 1e-3) / 1e9
    out = {
        "metric": head["metric"], "value": head["value"], "unit": head["unit"],
        "n_gpus": 1, "steps": head["steps"], "warmup": head.get("warmup", args.warmup), "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 matrix-core operands (bf16 inputs), f32 accumulate/state",
        "data": "synthetic",
        "config": head["config"],
        "roofline": head["roofline"],
        "cpu_baseline": head.get("cpu_baseline"),
        "tokheads_per_s": head.get("tokheads_per_s"),
        "workloads": {n_: r_ for n_, r_ in results.items() if r_ is not head},
        "decode": decode_obj if decode_obj is not head else None,
        "extras": extras,
        "error_metric": "max|x-ref|/max|ref| per (sequence, head); parity is gated in tests/",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
