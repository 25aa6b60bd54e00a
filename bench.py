#!/usr/bin/env python3
"""Benchmark of the DiT attention hot path on one MI355X.

One step = the attention of one DiT block for one request at the 14B-class shape: self-attention
over the 32,760 tokens of a 21x30x52 latent grid (40 heads, head_dim 128, 3-axis RoPE 44/42/42)
followed by cross-attention of the same 32,760 queries over 769 conditioning keys (512 text with a
padding mask + 257 image).  Inputs are seeded synthetic bf16 N(0,1) tensors resident in HBM before
the timed region.  Prints ONE JSON line: whole-step attention TFLOP/s (4*H*Lq*Lk*D flop per
product pair over the keys that attend, RoPE/softmax/mask not counted), a roofline object for the
dominant kernel (the self-attention kernel, timed with HIP events on its stream; beside the published
peak, what an MFMA-only micro-benchmark sustains on the same board) and the CPU fp64 oracle timed on a
bounded row sample as a baseline.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS_16BIT_DENSE = 2500.0  # MI355X published dense bf16/fp16 MFMA peak
PEAK_TFLOPS_8BIT_DENSE = 5000.0   # published dense fp8 MFMA peak

COUNTER_SUMMARY = os.path.join(ROOT, "profiles", "attn_fwd_pipe16_kernel_dit14b_counters.txt")


def traffic_bytes_for(version):
    """HBM bytes per launch of the self-attention kernel at the dit_14b shape with default flags, from the
    FETCH_SIZE / WRITE_SIZE counter runs summarised in COUNTER_SUMMARY (each scaled by a plain copy kernel).
    The summary names the library version it was taken with ("library_version: N") and the figure
    ("traffic_bytes_per_launch: X"); a library of any other version reports null."""
    try:
        text = open(COUNTER_SUMMARY).read()
    except OSError:
        return None
    found = {}
    for line in text.splitlines():
        key, _, val = line.partition(":")
        if key.strip() in ("library_version", "traffic_bytes_per_launch"):
            try:
                found[key.strip()] = float(val.split()[0])
            except (ValueError, IndexError):
                return None
    if int(found.get("library_version", -1)) != int(version):
        return None
    return found.get("traffic_bytes_per_launch")


def measure_mfma_peak(B, torch, launches=3, mfma_per_wavefront=1_200_000, sweep=False):
    """Sustained rate of the matrix cores alone on this board (dit_mfma_probe: two wavefronts per SIMD issuing
    32x32x16 MFMAs back to back from registers), TFLOP/s, for fp16 and bf16 operands, constant and random
    (random = every significand bit of the format in use).  With sweep, also fp16 operands that carry fewer
    significant bits.  Each figure is the mean of `launches` launches of about 50 ms after one warm-up launch."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(2 * cus * 256, dtype=torch.float32, device="cuda")
    cases = [("f16_constant", B.DIT_PROBE_F16, 0, 0), ("f16_random", B.DIT_PROBE_F16, 11, 11),
             ("bf16_constant", B.DIT_PROBE_BF16, 0, 0), ("bf16_random", B.DIT_PROBE_BF16, 8, 8)]
    if sweep:
        cases += [("f16_%d_%d_bits" % (a, b), B.DIT_PROBE_F16, a, b)
                  for a, b in ((10, 10), (9, 9), (8, 8), (6, 6), (4, 4), (11, 8), (8, 11), (11, 0), (0, 11))]
    out = {}
    for name, dt, ba, bb in cases:
        B.dit_mfma_probe(dt, ba, bb, mfma_per_wavefront, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = 0.0
        for _ in range(launches):
            flops += B.dit_mfma_probe(dt, ba, bb, mfma_per_wavefront, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    return out


def mfma_peak_workload(args):
    """Secondary line: the MFMA-only micro-benchmark by itself."""
    import torch

    from paper_2601_20655_amd import binding as B

    B.lib()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    t0 = time.perf_counter()
    rates = measure_mfma_peak(B, torch, launches=max(args.steps, 1), sweep=True)
    dt = time.perf_counter() - t0
    v = rates["f16_random"]
    print(json.dumps({
        "metric": "MFMA-only sustained TFLOP/s (32x32x16, two wavefronts per SIMD, random fp16 operands)",
        "value": v, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": 1,
        "ms_per_step": round(dt * 1e3 / (len(rates) * max(args.steps, 1)), 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "mfma_peak: every SIMD issues MFMAs from registers, nothing else", "rates_tflops": rates},
        "roofline": {"kernel": "mfma_probe_kernel", "bound": "mfma", "achieved": v, "peak": PEAK_TFLOPS_16BIT_DENSE,
                     "unit": "TFLOP/s", "frac": round(v / PEAK_TFLOPS_16BIT_DENSE, 4), "traffic": None},
    }))


class HipEvents:
    """Raw hipEvent_t pairs (ctypes on the HIP runtime) for the library's timing hook."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs:
            assert self.hip.hipEventSynchronize(b) == 0
            ms = ctypes.c_float()
            assert self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
            out.append(ms.value)
        return out

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def time_calls(B, torch, call, steps, warmup):
    """Warm up, then time `steps` calls of call() (one forward through the C ABI each): wall time
    per call bracketed by synchronisations, and the attention kernel's own time from HIP events."""
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    ev = HipEvents(steps)
    t0 = time.perf_counter()
    for i in range(steps):
        B.dit_attn_set_timing_events(*ev.pairs[i])
        call()
        B.dit_attn_set_timing_events(None, None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = ev.elapsed_ms()
    ev.close()
    return (t1 - t0) * 1e3 / steps, sum(kern) / len(kern)


def other_workload(args):
    """Secondary timing lines (not the headline metric): the other shapes and entry points, each as
    one JSON line of the same layout with its own metric name."""
    import numpy as np
    import torch

    from paper_2601_20655_amd import binding as B
    from paper_2601_20655_amd import workloads as wl

    B.lib()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cfg = wl.CONFIGS[args.workload]
    stream = torch.cuda.current_stream()

    def dev(a):
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()

    H, D = cfg.get("H"), cfg.get("D")
    norm = None
    if args.norm and cfg["kind"] in ("self", "cross"):
        gq, gk = wl.norm_weights(cfg)
        norm = (args.norm, 1e-6, torch.from_numpy(gq.reshape(-1)).cuda(), torch.from_numpy(gk.reshape(-1)).cuda())
    if cfg["kind"] == "linear":
        x, w, b = (dev(a) for a in wl.linear_inputs(cfg))
        out = torch.empty((cfg["M"], cfg["N"]), dtype=torch.bfloat16, device="cuda")
        flops = 2.0 * cfg["M"] * cfg["N"] * cfg["K"]
        what = "projection y = x w^T + bias, %d tokens, %d -> %d features" % (cfg["M"], cfg["K"], cfg["N"])
        kernel = "linear_kernel"

        def call():
            B.dit_linear_forward(x, w, b, out=out, stream=stream)
    elif cfg["kind"] == "qkv_attn":
        # q/k/v projection, then self-attention on what it wrote.  Separate: the projection writes [L, 3 H D] bf16
        # rows and the attention call packs its k and v columns into tile images.  --fused-qkv: the projection's
        # epilogue writes the q rows and the tile images itself and the attention call runs on them as they are.
        L = cfg["grid"][0] * cfg["grid"][1] * cfg["grid"][2]
        HD = H * D
        x, w, b = (dev(a) for a in wl.linear_inputs(dict(M=L, N=3 * HD, K=cfg["K"], seed=cfg["seed"])))
        y = torch.empty((L, 3 * HD), dtype=torch.bfloat16, device="cuda")
        yq, yk, yv = (y[:, i * HD:(i + 1) * HD].view(1, L, H, D) for i in range(3))
        q_out = torch.empty((1, L, H, D), dtype=torch.bfloat16, device="cuda")
        out = torch.empty_like(q_out)
        ws = torch.empty(B.dit_attn_workspace_bytes(B.self_attn_params(q_out, q_out, q_out, out, cfg["grid"],
                                                                        cfg["split"], flags=args.flags)),
                         dtype=torch.uint8, device="cuda")
        flops_proj = 2.0 * L * 3 * HD * cfg["K"]
        flops = flops_proj + 4.0 * H * L * L * D
        what = "q/k/v projection (%d tokens, %d -> %d features, %s) + self-attention (grid %dx%dx%d, %d heads, d%d)" % (
            L, cfg["K"], 3 * HD, "epilogue writes the attention's tile images" if args.fused_qkv else
            "separate calls", cfg["grid"][0], cfg["grid"][1], cfg["grid"][2], H, D)
        kernel = "attn_fwd_pipe16_kernel"
        mid = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

        def call():
            mid[0].record(stream)
            if args.fused_qkv:
                B.dit_qkv_proj_forward(x, w, b, cfg["grid"], cfg["split"], H, q_out=q_out, flags=args.flags,
                                       workspace=ws, stream=stream)
                mid[1].record(stream)
                B.dit_attn_forward(q_out, None, None, cfg["grid"], cfg["split"], out=out,
                                   flags=args.flags | B.DIT_FLAG_KV_RESIDENT, workspace=ws, stream=stream)
            else:
                B.dit_linear_forward(x, w, b, out=y, stream=stream)
                mid[1].record(stream)
                B.dit_attn_forward(yq, yk, yv, cfg["grid"], cfg["split"], out=out, flags=args.flags, workspace=ws,
                                   stream=stream)
            mid[2].record(stream)
    elif cfg["kind"] == "self":
        q, k, v = (dev(a) for a in wl.self_attn_inputs(cfg))
        out = torch.empty_like(q)
        ws = torch.empty(B.dit_attn_workspace_bytes(B.self_attn_params(q, k, v, out, cfg["grid"], cfg["split"],
                                                                        flags=args.flags, norm=norm)),
                         dtype=torch.uint8, device="cuda")
        L = q.shape[1]
        flops = 4.0 * cfg["B"] * H * L * L * D
        what = "self-attention, grid %dx%dx%d = %d tokens, %d heads, d%d" % (cfg["grid"] + (L, H, D))
        if norm:
            what += ", q and k RMS-normalised per %s" % args.norm
        kernel = "attn_fwd_pipe16_kernel"

        def call():
            B.dit_attn_forward(q, k, v, cfg["grid"], cfg["split"], out=out, flags=args.flags, workspace=ws,
                               stream=stream, norm=norm)
    elif cfg["kind"] == "varlen":
        q, k, v = (dev(a) for a in wl.varlen_attn_inputs(cfg))
        out = torch.empty_like(q)
        grids = list(cfg["grids"])
        ws = torch.empty(B.dit_attn_varlen_workspace_bytes(B.varlen_attn_params(q, k, v, out, grids, cfg["split"],
                                                                                 flags=args.flags)),
                         dtype=torch.uint8, device="cuda")
        flops = sum(4.0 * H * D * float(t * h * w) ** 2 for t, h, w in grids)
        what = "self-attention over %d packed requests (%d tokens), %d heads, d%d" % (len(grids), q.shape[0], H, D)
        kernel = "attn_fwd_pipe16_varlen_kernel"

        def call():
            B.dit_attn_varlen_forward(q, k, v, grids, cfg["split"], out=out, flags=args.flags, workspace=ws,
                                      stream=stream)
    else:
        qn, kn, vn, valid, text_len = wl.cross_attn_inputs(cfg)
        q, k, v = dev(qn), dev(kn), dev(vn)
        vd = torch.from_numpy(valid).cuda()
        out = torch.empty_like(q)
        split = cfg["n_text"] if args.decoupled else 0
        ws = torch.empty(B.dit_cross_attn_workspace_bytes(B.cross_attn_params(q, k, v, out, flags=args.flags,
                                                                               split=split, norm=norm)),
                         dtype=torch.uint8, device="cuda")
        Lq = q.shape[1]
        flops = 4.0 * H * Lq * D * float(valid.sum())  # keys that attend; padded keys are skipped, not computed
        flops_dense = 4.0 * cfg["B"] * H * Lq * D * float(valid.shape[1])
        # algorithmic bytes: q read and out written once, the attending k and v rows read once
        io_bytes = 2.0 * q.numel() * q.element_size() + 2.0 * float(valid.sum()) * H * D * k.element_size()
        what = "%s cross-attention, B=%d, %d queries x (512 text masked to %s + 257 image) keys, %d heads, d%d" % (
            "decoupled" if split else "joint", cfg["B"], Lq, list(map(int, text_len)), H, D)
        plain = split or args.flags & (B.DIT_FLAG_SIMPLE_SCHEDULE | B.DIT_FLAG_MFMA_32X32 | B.DIT_FLAG_WIDE_QTILE)
        kernel = ("attn_fwd_pipe_kernel" if args.flags & B.DIT_FLAG_PIPELINED_SCHEDULE else
                  "attn_fwd_kernel" if plain else "attn_fwd_pipe16_chain_kernel")
        # --key-counts: the same keys as two counts per request (text keys, image keys) instead of the byte mask
        kv_len = torch.tensor([[int(t), cfg["n_image"]] for t in text_len], dtype=torch.int32, device="cuda")
        if args.key_counts:
            what += ", keys given as counts"
        if norm:
            what += ", q and k RMS-normalised per %s" % args.norm

        def call():
            if args.key_counts:
                B.dit_cross_attn_forward_lengths(q, k, v, kv_len, cfg["n_text"], out=out, flags=args.flags,
                                                 workspace=ws, stream=stream, split=split, norm=norm)
            else:
                B.dit_cross_attn_forward(q, k, v, vd, out=out, flags=args.flags, workspace=ws, stream=stream,
                                         split=split, norm=norm)

    if args.flags & B.DIT_FLAG_KV_RESIDENT:  # the timed calls reuse what one ordinary call packs first
        resident = args.flags
        args.flags = resident & ~B.DIT_FLAG_KV_RESIDENT
        call()
        args.flags = resident
    ms, kern_ms = time_calls(B, torch, call, args.steps, args.warmup)
    achieved = flops / (kern_ms * 1e-3) / 1e12
    extra = {}
    if cfg["kind"] == "linear" and args.vendor_gemm:
        # the vendor's GEMM library on the same tensors and box (context for the projection kernel, never the metric)
        def vendor():
            torch.addmm(b, x, w.t(), out=out)
        for _ in range(args.warmup):
            vendor()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            vendor()
        e1.record()
        torch.cuda.synchronize()
        vms = e0.elapsed_time(e1) / args.steps
        extra = {"vendor_gemm": {"what": "torch.addmm on the same tensors", "ms_per_call": round(vms, 4),
                                 "tflops": round(flops / (vms * 1e-3) / 1e12, 1)}}
    if cfg["kind"] == "qkv_attn":
        # the last timed step's two calls on their own (events on the stream either side of each)
        extra = {"projection_call_ms": round(mid[0].elapsed_time(mid[1]), 4),
                 "attention_call_ms": round(mid[1].elapsed_time(mid[2]), 4),
                 "projection_flops": flops_proj}
        achieved = (flops - flops_proj) / (kern_ms * 1e-3) / 1e12
    if cfg["kind"] == "cross":
        # this shape is close enough to the HBM roofline that the streaming rate is reported beside the flops
        extra = {"tflops_dense_count": round(flops_dense / (ms * 1e-3) / 1e12, 2),
                 "tflops_over_attending_keys": round(flops / (ms * 1e-3) / 1e12, 2),
                 "algorithmic_bytes": io_bytes,
                 "achieved_GBps_whole_call": round(io_bytes / (ms * 1e-3) / 1e9, 1),
                 "achieved_GBps_attn_kernel": round(io_bytes / (kern_ms * 1e-3) / 1e9, 1),
                 "hbm_peak_GBps": 8000.0,
                 "hbm_floor_ms": round(io_bytes / 8e12 * 1e3, 4)}
    fp8 = bool(args.flags & B.DIT_FLAG_QK_FP8)
    # 8-bit scores: half of the flops run at the 8-bit peak, half at the 16-bit peak
    peak = 2.0 / (1.0 / PEAK_TFLOPS_8BIT_DENSE + 1.0 / PEAK_TFLOPS_16BIT_DENSE) if fp8 else PEAK_TFLOPS_16BIT_DENSE
    print(json.dumps({
        "metric": ("projection" if cfg["kind"] == "linear" else "projection + attention" if cfg["kind"] == "qkv_attn"
                   else "attention") + " TFLOP/s, %s" % args.workload
                  + (" (decoupled)" if args.decoupled else "")
                  + (" (8-bit score operands: outside the 16-bit parity contract)" if fp8 else ""),
        "value": round(flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["kind"] == "linear" else "fp8 scores, f16 PV" if fp8
                 else "f16" if not (args.flags & B.DIT_FLAG_QK_BF16) else "bf16",
        "data": "synthetic",
        "config": dict({"workload": what, "flags": args.flags, "attn_kernel_ms": round(kern_ms, 4),
                        "flops_per_step": flops}, **extra),
        "roofline": {"kernel": kernel, "bound": "mfma", "achieved": round(achieved, 2),
                     "peak": round(peak, 1), "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--flags", type=int, default=0, help="DIT_FLAG_* bits for both calls (0 = library defaults)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-mfma-peak", action="store_true", help="skip the MFMA-only micro-benchmark leg")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy before the timed region, so that a "
                         "counter run (FETCH_SIZE / WRITE_SIZE) holds a kernel of known traffic to scale by")
    ap.add_argument("--workload", default="step",
                    help="'step' (default: the headline metric) or one of the other shapes for a secondary "
                         "timing line: dit_1p3b, dit_14b, dit_14b_hires, cross_14b, varlen_14b, qkv_proj_14b, out_proj_14b, "
                         "qkv_attn_14b (projection, then self-attention on its output), mfma_peak (the MFMA-only micro-benchmark)")
    ap.add_argument("--decoupled", action="store_true", help="cross_14b: one softmax per conditioning sequence")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="qkv_proj_14b / out_proj_14b: also time the vendor GEMM library (torch.addmm) on the same tensors")
    ap.add_argument("--fused-qkv", action="store_true",
                    help="qkv_attn_14b: dit_qkv_proj_forward (the projection writes the attention's tile images) and "
                         "the attention call on them, instead of two separate calls")
    ap.add_argument("--norm", choices=["head", "token"], default=None,
                    help="self- and cross-attention workloads: fused RMS normalisation of q and k (weights 1 + 0.25 N(0,1))")
    ap.add_argument("--key-counts", action="store_true",
                    help="cross_14b: dit_cross_attn_forward_lengths (two key counts per request) instead of the byte mask")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on ONE GPU (all heads of one request on one MI355X, no "
                 "collectives); --gpus %d is not supported" % args.gpus)
    if args.workload == "mfma_peak":
        return mfma_peak_workload(args)
    if args.workload != "step":
        return other_workload(args)
    if args.flags & (1 << 12):
        sys.exit("bench.py: the headline step is the 16-bit contract; time the 8-bit score path as a secondary "
                 "line, e.g. --workload dit_14b --flags 4096")

    import numpy as np
    import torch

    from paper_2601_20655_amd import binding as B
    from paper_2601_20655_amd import workloads as wl

    B.lib()  # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    cfg = wl.CONFIGS["dit_14b"]
    ccfg = dict(wl.CONFIGS["cross_14b"], B=1)
    q, k, v = wl.self_attn_inputs(cfg)
    cq, ck, cv, cvalid, text_len = wl.cross_attn_inputs(ccfg)

    def dev(a):
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()

    qd, kd, vd = dev(q), dev(k), dev(v)
    ckd, cvd = dev(ck), dev(cv)
    cvalid_d = torch.from_numpy(cvalid).cuda()
    Bsz, L, H, D = qd.shape
    Lk = ckd.shape[1]
    out = torch.empty_like(qd)
    cout = torch.empty_like(qd)
    ps = B.self_attn_params(qd, kd, vd, out, cfg["grid"], cfg["split"], flags=args.flags)
    pc = B.cross_attn_params(out, ckd, cvd, cout, flags=args.flags & ~(B.DIT_FLAG_KV_FUSED | B.DIT_FLAG_KV_PREPACK))
    ws = torch.empty(max(B.dit_attn_workspace_bytes(ps), B.dit_cross_attn_workspace_bytes(pc), 256),
                     dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        # the cross-attention consumes the self-attention output as its queries, as in a DiT block
        B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], out=out, flags=args.flags, workspace=ws,
                           stream=stream)
        B.dit_cross_attn_forward(out, ckd, cvd, cvalid_d, out=cout, flags=pc.flags, workspace=ws, stream=stream)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # one copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    ev = HipEvents(args.steps)
    # the whole self-attention call (rotation table, pre-pack pass, attention kernel) is bracketed too
    call_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        a, b = ev.pairs[i]
        call_ev[i][0].record(stream)
        B.dit_attn_set_timing_events(a, b)
        B.dit_attn_forward(qd, kd, vd, cfg["grid"], cfg["split"], out=out, flags=args.flags, workspace=ws,
                           stream=stream)
        B.dit_attn_set_timing_events(None, None)
        call_ev[i][1].record(stream)
        B.dit_cross_attn_forward(out, ckd, cvd, cvalid_d, out=cout, flags=pc.flags, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern_ms = ev.elapsed_ms()
    ev.close()
    self_call_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in call_ev]))

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops_self = 4.0 * Bsz * H * L * L * D
    # cross-attention: padded keys are skipped, not computed, so only the keys that attend count
    n_attend = float(cvalid.sum())
    flops_cross = 4.0 * H * L * D * n_attend
    tflops = (flops_self + flops_cross) / (ms_per_step * 1e-3) / 1e12
    kern_avg_ms = float(np.mean(kern_ms))
    achieved = flops_self / (kern_avg_ms * 1e-3) / 1e12
    qk_name = "bf16" if args.flags & B.DIT_FLAG_QK_BF16 else "fp16"
    pv_name = "bf16" if args.flags & B.DIT_FLAG_PV_BF16 else "fp16"

    result = {
        "metric": "attention TFLOP/s + % bf16 MFMA peak at 32,760 tokens x 40 heads x d128",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if qk_name == "fp16" else "bf16",
        "data": "synthetic",
        "config": {
            "workload": "dit_14b self-attention (B=1, grid 21x30x52 = 32,760 tokens, 40 heads, d128, RoPE 44/42/42) "
                        "+ cross-attention of the same queries over 769 keys (512 text masked to %d, 257 image: "
                        "%d keys attend)" % (int(text_len[0]), int(n_attend)),
            "io": "bf16 in, bf16 out; fp32 accumulate",
            "mfma_operands": "q', k': %s; P, V: %s (the metric names bf16: fp16 has the same matrix rate and three "
                             "more significand bits; the all-bf16 kernel is DIT_FLAG_QK_BF16|DIT_FLAG_PV_BF16 = "
                             "--flags 5 and does not meet the 2e-2 parity bar)" % (qk_name, pv_name),
            "flags": args.flags,
            "pct_of_16bit_mfma_peak": round(100.0 * tflops / PEAK_TFLOPS_16BIT_DENSE, 2),
            "self_attn_kernel_ms": round(kern_avg_ms, 4),
            # the metric's own number: the self-attention call alone, rotation table and pre-pack pass included
            "self_attn_call_ms": round(self_call_ms, 4),
            "self_attn_tflops": round(flops_self / (self_call_ms * 1e-3) / 1e12, 2),
            "self_attn_pct_of_16bit_mfma_peak": round(100.0 * flops_self / (self_call_ms * 1e-3) / 1e12
                                                      / PEAK_TFLOPS_16BIT_DENSE, 2),
            "cross_attn_flops_counted": "over the %d attending keys (dense count over 769: %.4g)" % (
                int(n_attend), 4.0 * H * L * D * Lk),
            "flops_per_step": flops_self + flops_cross,
        },
        "roofline": {
            "kernel": "attn_fwd_pipe16_kernel (self-attention, 32,760 x 32,760 x 40 heads)",
            "bound": "mfma",
            "achieved": round(achieved, 2),
            "peak": PEAK_TFLOPS_16BIT_DENSE,
            "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_TFLOPS_16BIT_DENSE, 4),
            "traffic": traffic_bytes_for(B.dit_attn_version()) if args.flags == 0 else None,
        },
    }
    if not args.no_mfma_peak:
        # what the matrix cores alone sustain on THIS board, beside the published peak the fraction is quoted on
        rates = measure_mfma_peak(B, torch)
        key = "%s_random" % ("bf16" if qk_name == "bf16" and pv_name == "bf16" else "f16")
        result["roofline"]["measured_mfma_peak"] = dict(rates, unit="TFLOP/s",
                                                        what="MFMA-only micro-benchmark, two wavefronts per SIMD")
        result["roofline"]["frac_of_measured_%s" % key] = round(achieved / rates[key], 4)

    if not args.no_cpu_baseline:
        import oracle

        rows = wl.sample_rows(L, cfg["seed"], edge=64, n_random=1920)  # about 15 s of fp64 work on 16 cores
        t0 = time.perf_counter()
        ref = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], rows=rows)
        dt = time.perf_counter() - t0
        got = out[:, torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        rms = float(np.sqrt(np.mean(ref * ref)))
        result["cpu_baseline"] = {
            "value": round(4.0 * Bsz * H * len(rows) * L * D / dt / 1e12, 5),
            "unit": "TFLOP/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "%d query rows x %d heads x all %d keys of the same self-attention (fp64, %.1f s); "
                      "extrapolated full problem %.0f s" % (len(rows), H, L, dt, dt * L / len(rows)),
            "gpu_vs_oracle_max_err_over_rms": round(float(np.abs(got - ref).max() / rms), 5),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
