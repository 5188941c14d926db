#!/usr/bin/env python3
"""Benchmark of the KDA hot path on one MI355X.

A "step" is one pass of the hot path over one batch of synthetic input: the
chunkwise prefill (kda_chunk_fwd) on the bf16 prefill workload, and one decode
step (kda_recurrent_step) over the decode workload's state pool.  The two are
timed in separate regions of K steps each, inputs resident in HBM, bracketed
by device synchronisation and measured with HIP events on the launch stream.
`value` is prefill tokens/s; the decode figures are in the `decode` object.

Prints ONE JSON line.  Runs on one GPU only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Published MI355X peaks used for the roofline fractions.
HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0          # dense fp16/bf16 matrix cores

# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (profiles/pmc_traffic_bench_cfg1_cfg4.txt),
# scaled by what the same counters read for a 1 GiB copy.  Counter collection serialises kernels, so the
# prefill figure is that of the two kernels run one after the other (both summed).
MEASURED_TRAFFIC_BYTES = {"cfg1_prefill_bf16": 1007.3e6, "cfg4_decode_bf16": 1086.6e6}
# the same for the five kernels of one backward call on the cfg1 shape (profiles/pmc_traffic_bench_backward_cfg1.txt)
MEASURED_BACKWARD_TRAFFIC_BYTES = 6146.5e6

# Algorithmic work per (token, head) at d_k = d_v = 128, C = 64.
FLOP_PER_TOKHEAD = 6 * 128 * 128 + 3 * 64 * 128 + 64 * 64        # paper's FLOPs model: 126976
BYTES_PER_TOKHEAD = (3 * 128 + 128) * 2 + 2 + 128 * 4            # q,k,log_alpha,v,beta bf16 + o fp32: 1538


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def _time_region(torch, fn, steps):
    """Time `steps` calls of fn() with HIP events on the current stream; returns ms per call."""
    torch.cuda.synchronize()
    a, b = _events(torch)
    a.record()
    for _ in range(steps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true",
                    help="skip the extra serial / single-kernel timing passes (keeps a profile of this "
                         "run down to the launches of the timed configuration)")
    ap.add_argument("--extras", action="store_true",
                    help="with --serial: still run the extra passes (bf16 outputs, scalar gate, fused stages, "
                         "backward), every prefill with its kernels one after the other")
    ap.add_argument("--serial", action="store_true",
                    help="run the two prefill kernels one after the other (needed under tools that serialise "
                         "kernels, e.g. rocprofv3 --pmc); implies --no-breakdown")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run a plain 1 GiB device copy three times, so that a byte counter collected over "
                         "this run can be scaled by what it reads for a transfer of known size")
    ap.add_argument("--workload", default="cfg1_prefill_bf16",
                    help="prefill workload: cfg1_prefill_bf16 (default), cfg2_varlen_bf16, cfg3_long_bf16")
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
    if args.serial:
        args.no_breakdown = not args.extras
        kda.kda_debug_set_overlap(0)
    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ prefill workload
    name = args.workload
    c = si.CONFIGS[name]
    if name == "cfg1_prefill_bf16":
        host = si.make_prefill(c["B"], c["T"], c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"],
                               c["h0_std"])
        x = {k_: (v_.to(dev) if isinstance(v_, torch.Tensor) else v_) for k_, v_ in host.items()}
        tokens = c["B"] * c["T"]
        desc = {"workload": name, "B": c["B"], "T": c["T"], "H": c["H"], "dk": c["dk"], "dv": c["dv"],
                "chunk": 64}
    elif name == "cfg2_varlen_bf16":
        lens = si.varlen_lengths(c["N"], c["len_lo"], c["len_hi"], c["seed"])
        host = si.make_varlen(lens, c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], c["h0_std"])
        x = {k_: (v_.to(dev) if isinstance(v_, torch.Tensor) else v_) for k_, v_ in host.items()}
        tokens = int(lens.sum())
        desc = {"workload": name, "num_seqs": c["N"], "total_tokens": tokens, "H": c["H"], "dk": c["dk"],
                "dv": c["dv"], "chunk": 64}
    elif name == "cfg3_long_bf16":
        host = None
        x = si.make_long_on_device(c["T"], c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], dev)
        x["h0"] = None
        x["cu_seqlens"] = None
        tokens = c["T"]
        desc = {"workload": name, "B": 1, "T": c["T"], "H": c["H"], "dk": c["dk"], "dv": c["dv"], "chunk": 64}
    else:
        raise SystemExit("unknown workload " + name)
    H = c["H"]
    tokheads = tokens * H

    max_len = int(lens.max()) if name == "cfg2_varlen_bf16" else 0
    dims = kda.kda.make_chunk_dims(x["q"], x["v"], x["cu_seqlens"], 1.0, max_len)
    ws_bytes = kda.kda_chunk_fwd_workspace_size(dims)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    o = torch.empty(x["q"].shape[0], x["q"].shape[1], H, c["dv"], dtype=torch.float32, device=dev)
    hT = torch.empty(dims.num_seqs, H, c["dk"], c["dv"], dtype=torch.float32, device=dev)

    def prefill():
        kda.kda_chunk_fwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], h0=x["h0"],
                          cu_seqlens=x["cu_seqlens"], o=o, hT=hT, workspace=ws, max_seqlen=max_len)

    for _ in range(args.warmup):
        prefill()
    ms_prefill = _time_region(torch, prefill, args.steps)
    kda.kda_chunk_fwd_check(dims, ws)            # raises if the sequential kernel ever gave up waiting for a slot
    # The same call with its two kernels strictly one after the other, and each kernel alone
    # (switching one off also switches the overlap off): per-kernel durations.
    ms_serial = ms_intra = ms_scan = None
    if not args.no_breakdown:
        kda.kda_debug_set_overlap(0)
        ms_serial = _time_region(torch, prefill, args.steps)
        kda.kda_debug_set_phase_mask(1)
        ms_intra = _time_region(torch, prefill, args.steps)
        kda.kda_debug_set_phase_mask(2)
        ms_scan = _time_region(torch, prefill, args.steps)
        kda.kda_debug_set_phase_mask(3)
        kda.kda_debug_set_overlap(0 if args.serial else 1)
        prefill()
        torch.cuda.synchronize()

    tok_per_s = tokens / (ms_prefill * 1e-3)
    alg_bytes = tokheads * BYTES_PER_TOKHEAD + 2 * dims.num_seqs * H * 128 * 128 * 4
    streams = dims.num_seqs * H
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    # the library's own rule for running the kernels side by side
    overlapped = 4 * streams <= 3 * cus and not args.serial
    if overlapped or ms_scan is None:
        # kda_scan is launched first and retires last: its duration is the call's, up to the flag
        # reset (a few microseconds) and the launch gaps, which the event pair also brackets
        dom_name, dom_ms = "kda_scan_kernel (kda_intra_kernel runs beside it)", ms_prefill
    else:
        dom_name, dom_ms = ("kda_scan_kernel", ms_scan) if ms_scan >= ms_intra else ("kda_intra_kernel", ms_intra)
    roofline = {
        "kernel": dom_name, "bound": "hbm",
        "achieved": alg_bytes / (dom_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": alg_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": MEASURED_TRAFFIC_BYTES.get(name),
        "ms_kernel": dom_ms,
        "algorithmic_bytes": alg_bytes,
        "kernels_ms_alone": {"kda_intra_kernel": ms_intra, "kda_scan_kernel": ms_scan, "both_serial": ms_serial},
        "whole_call": {
            "hbm_frac": alg_bytes / (ms_prefill * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "mfma_frac_model_flops": tokheads * FLOP_PER_TOKHEAD / (ms_prefill * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
            "model_tflops": tokheads * FLOP_PER_TOKHEAD / (ms_prefill * 1e-3) / 1e12,
        },
    }

    # the same prefill with o stored as bf16 (the headline keeps fp32 o, which parity is stated on)
    bf16_out_obj = None
    if not args.no_breakdown:
        o16 = torch.empty(o.shape, dtype=torch.bfloat16, device=dev)

        def prefill_bf16_out():
            kda.kda_chunk_fwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], h0=x["h0"],
                              cu_seqlens=x["cu_seqlens"], o=o16, hT=hT, workspace=ws, max_seqlen=max_len)
        for _ in range(args.warmup):
            prefill_bf16_out()
        ms_o16 = _time_region(torch, prefill_bf16_out, args.steps)
        kda.kda_chunk_fwd_check(dims, ws)
        bf16_out_obj = {"what": "same workload, out_dtype bf16 (o rounded once at the store)",
                        "ms_per_step": ms_o16, "tokens_per_s": tokens / (ms_o16 * 1e-3)}
        del o16

    # the scalar-gate special case (one decay per token and head) on the same shape: its own entry point
    scalar_obj = None
    if not args.no_breakdown:
        gh = x["log_alpha"][..., 0].contiguous()

        def prefill_scalar_gate():
            kda.kda_chunk_fwd_scalar_gate(x["q"], x["k"], x["v"], gh, x["beta"], h0=x["h0"],
                                          cu_seqlens=x["cu_seqlens"], o=o, hT=hT, workspace=ws, max_seqlen=max_len)
        for _ in range(args.warmup):
            prefill_scalar_gate()
        ms_sg = _time_region(torch, prefill_scalar_gate, args.steps)
        kda.kda_chunk_fwd_check(dims, ws)
        scalar_obj = {"what": "kda_chunk_fwd_scalar_gate on the same shape (the decay of channel 0 taken for the whole head)",
                      "ms_per_step": ms_sg, "tokens_per_s": tokens / (ms_sg * 1e-3)}
        del gh

    # the backward pass (kda_chunk_bwd, fp32 throughout) on the same shape: time per call, and its rate
    # against the fp32 vector peak under a FLOP model of the chunkwise backward (per chunk and head:
    # eight C x d x d products, eight half-filled C x C x d ones, the C x C x C chain)
    backward_obj = None
    if name == "cfg1_prefill_bf16" and not args.no_breakdown:
        d_o = torch.randn(o.shape, generator=torch.Generator().manual_seed(c["seed"] + 1)).to(dev)
        ws_b = torch.empty(kda.kda_chunk_bwd_workspace_size(dims), dtype=torch.uint8, device=dev)

        grads = kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], d_o, h0=x["h0"], workspace=ws_b)

        def backward():
            return kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], d_o, h0=x["h0"],
                                     workspace=ws_b, out=grads)
        backward()
        steps_b = max(3, min(args.steps, 10))
        ms_bwd = _time_region(torch, backward, steps_b)
        C_, D_ = 64, c["dk"]
        flop_chunk = 8 * 2 * C_ * D_ * D_ + 8 * C_ * C_ * D_ + 3 * 2 * C_ * C_ * C_
        chunks_heads = tokheads / C_
        tflops = chunks_heads * flop_chunk / (ms_bwd * 1e-3) / 1e12
        backward_obj = {"what": "kda_chunk_bwd on the same shape: gradients of q, k, v, log_alpha, beta, h0 (fp32 arithmetic)",
                        "ms_per_step": ms_bwd, "steps": steps_b, "tokens_per_s": tokens / (ms_bwd * 1e-3),
                        "roofline": {"bound": "alu", "achieved": tflops, "peak": 157.3, "unit": "TFLOP/s",
                                     "frac": tflops / 157.3, "flop_per_chunk_head": flop_chunk, "traffic": None}}
        if not args.no_cpu_baseline and host is not None:
            import numpy as np
            import oracle
            n_s = 256
            a = {k_: si.to_np32(host[k_][:, :n_s]) for k_ in ("q", "k", "v", "log_alpha", "beta")}
            t0 = time.perf_counter()
            reps = 0
            while time.perf_counter() - t0 < 5.0:
                oracle.kda_backward(a["q"], a["k"], a["v"], a["log_alpha"], a["beta"],
                                    d_o[:, :n_s].cpu().numpy(), h0=host["h0"].numpy().astype(np.float64))
                reps += 1
            dtb = time.perf_counter() - t0
            backward_obj["cpu_baseline"] = {"value": c["B"] * n_s * reps / dtb, "unit": "tokens/s",
                                            "cores": oracle.num_threads(), "kind": "oracle",
                                            "sample": "first %d tokens of every sequence, %d times over, fp64 "
                                                      "token-by-token reverse pass" % (n_s, reps),
                                            "seconds": dtb}
        del d_o, ws_b, grads

    # the same prefill on raw projections (fused input prologue), cfg1 shape only
    fused_obj = None
    if name == "cfg1_prefill_bf16" and not args.no_breakdown:
        rawx = si.make_raw_tokens(c["B"], c["T"], H, c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"])
        rx = {k_: v_.to(dev) for k_, v_ in rawx.items()}

        def prefill_fused():
            # a_scale = 1, dt_bias = 0: the decays then follow the workload's own recipe, -softplus(N(mu, 1))
            kda.kda_chunk_fwd_fused(rx["q_raw"], rx["k_raw"], rx["v"], rx["gate"], rx["beta_logit"],
                                    h0=x["h0"], o=o, hT=hT, workspace=ws)
        for _ in range(args.warmup):
            prefill_fused()
        ms_fused = _time_region(torch, prefill_fused, args.steps)
        kda.kda_chunk_fwd_check(dims, ws)
        og = torch.randn(c["B"], c["T"], H, c["dv"], generator=torch.Generator().manual_seed(c["seed"])).to(torch.bfloat16).to(dev)
        nw = torch.ones(c["dv"], dtype=torch.float32, device=dev)

        # (with the output gate the workspace also holds the re-laid gate logits)
        ws_g = torch.empty(kda.kda_chunk_fwd_workspace_size(dims, output_gate=True), dtype=torch.uint8, device=dev)

        def prefill_fused_both():
            kda.kda_chunk_fwd_fused(rx["q_raw"], rx["k_raw"], rx["v"], rx["gate"], rx["beta_logit"],
                                    out_gate=og, norm_weight=nw, h0=x["h0"], o=o, hT=hT, workspace=ws_g)
        for _ in range(args.warmup):
            prefill_fused_both()
        ms_both = _time_region(torch, prefill_fused_both, args.steps)
        kda.kda_chunk_fwd_check(dims, ws_g)
        del ws_g
        fused_obj = {"what": "kda_chunk_fwd_fused on the cfg1 shape: (a) input prologue (L2Norm(q), L2Norm(k), "
                             "Sigmoid(beta), decay function) inside the per-chunk kernel; (b) plus the output gate "
                             "Sigmoid(g) * RMSNorm(o) inside the sequential kernel",
                     "prologue": {"ms_per_step": ms_fused, "tokens_per_s": tokens / (ms_fused * 1e-3)},
                     "prologue_and_output_gate": {"ms_per_step": ms_both, "tokens_per_s": tokens / (ms_both * 1e-3)}}
        del og
        del rx

    # ------------------------------------------------------------------ decode workload
    d4 = si.CONFIGS["cfg4_decode_bf16"]
    N4, H4, dk4, dv4 = d4["N"], d4["H"], d4["dk"], d4["dv"]
    del ws
    S = si.make_state(N4, H4, dk4, dv4, d4["state_std"], d4["seed"]).to(dev)
    tok_host = si.make_decode_tokens(N4, H4, dk4, dv4, d4["dtype"], d4["mu"], d4["seed"], 0)
    tk = {k_: v_.to(dev) for k_, v_ in tok_host.items()}
    o4 = torch.empty(N4, H4, dv4, dtype=torch.float32, device=dev)

    def decode():
        kda.kda_recurrent_step(tk["q"], tk["k"], tk["v"], tk["log_alpha"], tk["beta"], S, o=o4)

    for _ in range(args.warmup):
        decode()
    ms_decode = _time_region(torch, decode, args.steps)
    dec_bytes = 2 * N4 * H4 * dk4 * dv4 * 4 + N4 * H4 * ((3 * dk4 + dv4) * 2 + 2) + N4 * H4 * dv4 * 4
    decode_obj = {
        "metric": "decode-step state GB/s", "value": dec_bytes / (ms_decode * 1e-3) / 1e9, "unit": "GB/s",
        "ms_per_step": ms_decode, "steps": args.steps,
        "config": {"workload": "cfg4_decode_bf16", "num_seqs": N4, "H": H4, "dk": dk4, "dv": dv4,
                   "state_bytes": N4 * H4 * dk4 * dv4 * 4},
        "roofline": {"kernel": "kda_step_kernel", "bound": "hbm",
                     "achieved": dec_bytes / (ms_decode * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dec_bytes / (ms_decode * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get("cfg4_decode_bf16"),
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

    for _ in range(args.warmup):
        decode_pooled()
    ms_pooled = _time_region(torch, decode_pooled, args.steps)
    pooled_bytes = 2 * N4 * H4 * dk4 * dv4 * 4 + Tq * (N4 * H4 * ((3 * dk4 + dv4) * 2 + 2) + N4 * H4 * dv4 * 4)
    decode_obj["pooled_multi_token"] = {
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
    decode_obj["roofline"]["measured_copy_GBps"] = copy_gbs
    decode_obj["roofline"]["frac_of_measured_copy"] = decode_obj["value"] / copy_gbs

    # ------------------------------------------------------------------ CPU baseline (oracle)
    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        if host is not None and name == "cfg1_prefill_bf16":
            a = {k_: si.to_np32(host[k_]) for k_ in ("q", "k", "v", "log_alpha", "beta")}
            h0 = host["h0"].numpy().astype(np.float64)
            # the whole workload, repeated until about ten seconds of CPU work have gone by
            reps, dt = 0, 0.0
            t0 = time.perf_counter()
            while dt < 10.0 and reps < 200:
                oracle.kda_forward(a["q"], a["k"], a["v"], a["log_alpha"], a["beta"], h0=h0)
                reps += 1
                dt = time.perf_counter() - t0
            sample_tokens = tokens * reps
            sample = "whole %s workload (%d tokens x %d heads) %d times over, fp64 per-token recurrence" % (
                name, tokens, H, reps)
        else:
            # bounded sample: the first 4096 tokens of every head
            n_s = min(4096, tokens)
            a = {k_: si.to_np32(x[k_][:, :n_s]) for k_ in ("q", "k", "v", "log_alpha", "beta")}
            t0 = time.perf_counter()
            oracle.kda_forward(a["q"], a["k"], a["v"], a["log_alpha"], a["beta"])
            dt = time.perf_counter() - t0
            sample_tokens = n_s
            sample = "first %d tokens of %s x %d heads, fp64 per-token recurrence" % (n_s, name, H)
        cpu = {"value": sample_tokens / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": sample, "seconds": dt}
        Sh = S.cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        oracle.kda_step(si.to_np32(tok_host["q"]), si.to_np32(tok_host["k"]), si.to_np32(tok_host["v"]),
                        si.to_np32(tok_host["log_alpha"]), si.to_np32(tok_host["beta"]), Sh)
        dt4 = time.perf_counter() - t0
        decode_obj["cpu_baseline"] = {"value": dec_bytes / dt4 / 1e9, "unit": "GB/s",
                                      "cores": oracle.num_threads(), "kind": "oracle",
                                      "sample": "one decode step over the whole cfg4 state pool, fp64",
                                      "seconds": dt4}

    out = {
        "metric": "KDA prefill tokens/s", "value": tok_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_prefill,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 matrix-core operands (bf16 inputs), f32 accumulate/state",
        "data": "synthetic",
        "config": desc,
        "tokheads_per_s": tokheads / (ms_prefill * 1e-3),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "prefill_bf16_out": bf16_out_obj,
        "prefill_scalar_gate": scalar_obj,
        "prefill_fused_stages": fused_obj,
        "backward": backward_obj,
        "decode": decode_obj,
        "error_metric": "max|x-ref|/max|ref| per (sequence, head); parity is gated in tests/",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
