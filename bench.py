#!/usr/bin/env python3
"""Benchmark of the hot path: causal linear attention forward + backward on one MI355X.

A step is one pass of the whole hot path -- chela_linattn_fwd followed by chela_linattn_bwd -- over one batch of
synthetic, seeded input that is already resident in HBM.  Default workload: the LM-shaped configuration the headline
metric is quoted on (B=4, H=12, N=16384, dk=dv=64, bf16 I/O, fp32 accumulation).  Prints one JSON line.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MFMA_F32_PEAK_TFLOPS = 157.3    # dense fp32


def algorithmic_bytes_per_token_head(dk, dv, es=2):
    """Each I/O tensor moved once, states stay on chip: fwd reads Q,K,V writes O; bwd reads Q,K,V,dO writes dQ,dK,dV."""
    fwd = es * (2 * dk + 2 * dv)
    bwd = es * (2 * dk + 2 * dv + 2 * dk + dv)
    return fwd, bwd


def flops_per_token_head(dk, dv, C):
    """Full-tile count of matrix-core work: fwd 2C(dk+dv) + 4 dk dv; bwd 6C dk + 4C dv + 10 dk dv."""
    return 2 * C * (dk + dv) + 4 * dk * dv, 6 * C * dk + 4 * C * dv + 10 * dk * dv


def read_profile(path, sources_hash):
    """The `key: value` lines of a committed rocprofv3 summary (profiles/*.txt, written by
    paper_2406_08128_amd/profile_summary.py) and where they come from.  Counter figures cannot be measured by an
    ordinary run, so the line quotes the committed ones -- but only while the summary was taken on the kernel
    sources this tree holds (its kernel_sources_sha256 equals the tree's) and, where the repository's history is at
    hand, its commit is an ancestor of HEAD.  Returns (values or None, source description)."""
    src = {"file": os.path.relpath(path, ROOT)}
    try:
        txt = open(path).read()
    except OSError:
        src["status"] = "absent"
        return None, src
    kv = dict(re.findall(r"^([A-Za-z_][A-Za-z0-9_\[\]]*):\s*(.+?)\s*$", txt, flags=re.M))
    src["commit"] = kv.get("commit", "unknown").split()[0]
    src["kernel_sources_sha256"] = kv.get("kernel_sources_sha256", "unknown")
    if src["kernel_sources_sha256"] != sources_hash:
        src["status"] = "stale: taken on other kernel sources than this tree's (%s); not quoted" % sources_hash
        return None, src
    if os.path.isdir(os.path.join(ROOT, ".git")) and re.fullmatch(r"[0-9a-f]{40}", src["commit"]):
        import subprocess
        r = subprocess.run(["git", "-C", ROOT, "merge-base", "--is-ancestor", src["commit"], "HEAD"],
                           stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        if r.returncode != 0:
            src["status"] = "stale: its commit is not an ancestor of HEAD; not quoted"
            return None, src
    src["status"] = "current"
    return kv, src


def bench_decode(args, w, torch, binding):
    """Single-token decode steps (S += k v^T; o = S^T q) for `decode_batch` sequences x H heads of the workload's width."""
    B, H, dk, dv = args.decode_batch, w.H, w.dk, w.dv
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    q = (torch.randn(B, H, dk, device="cuda", generator=g) / 8).to(torch.bfloat16)
    k = (torch.randn(B, H, dk, device="cuda", generator=g) / 8).to(torch.bfloat16)
    v = torch.randn(B, H, dv, device="cuda", generator=g).to(torch.bfloat16)
    S = torch.zeros(B, H, dk, dv, device="cuda")
    o = torch.empty(B, H, dv, device="cuda", dtype=torch.bfloat16)
    for _ in range(args.warmup):
        binding.chela_linattn_step(q, k, v, S, o=o)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        binding.chela_linattn_step(q, k, v, S, o=o)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    binding.chela_profile_reset()
    binding.chela_profile_enable(True)
    for _ in range(args.steps):
        binding.chela_linattn_step(q, k, v, S, o=o)
    torch.cuda.synchronize()
    prof = binding.chela_profile_read()
    binding.chela_profile_enable(False)
    binding.chela_profile_reset()
    n, tot = prof["bf16_step_kernel"]
    us = tot * 1e3 / n
    alg = B * H * (2 * dk * dv * 4 + 2 * (2 * dk + 2 * dv))     # state read + written in fp32, q,k,v,o in bf16
    achieved = alg / (us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "causal linear-attn decode tokens/s", "value": round(B / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "decode: %d sequences x H%d dk%d dv%d, one token each per step, fp32 state" % (B, H, dk, dv)},
        "roofline": {"bound": "hbm", "kernel": "bf16_step_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": alg, "avg_launch_us": round(us, 2)},
        "cpu_baseline": None}))


def bench_n_sweep(args, w, torch, binding):
    """The workload's shape at sequence lengths 2048 ... 65536 (B, H, widths fixed): time per token must not depend on
    N once the GPU is full (the linear-cost claim of Sec. 1 and of the ablation on hardware efficiency)."""
    from paper_2406_08128_amd.workloads import make_inputs, shrink
    rows = []
    for N in (2048, 4096, 8192, 16384, 32768, 65536):
        wn = shrink(w, N=N)
        d = {k: v.cuda() for k, v in make_inputs(wn, with_dO=True).items()}
        O = torch.empty_like(d["V"])
        dQ, dK, dV = torch.empty_like(d["Q"]), torch.empty_like(d["K"]), torch.empty_like(d["V"])

        def step():
            binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], O=O, chunk=args.chunk)
            binding.chela_linattn_bwd(d["Q"], d["K"], d["V"], d["dO"], dQ=dQ, dK=dK, dV=dV, chunk=args.chunk)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        rows.append({"N": N, "ms_per_step": round(ms, 4), "ns_per_token_head": round(ms * 1e6 / (wn.B * wn.H * N), 4),
                     "tokens_per_s": round(wn.B * N / (ms * 1e-3), 1)})
        del d, O, dQ, dK, dV
    ref = [r for r in rows if r["N"] == 16384][0]["ns_per_token_head"]
    for r in rows:
        r["vs_N16384"] = round(r["ns_per_token_head"] / ref, 3)
    print(json.dumps({
        "metric": "causal linear-attn fwd+bwd time per token-head over sequence length", "unit": "ns/token-head",
        "value": ref, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s shape (B%d H%d dk%d dv%d), N swept, fwd+bwd, chunk %d"
                               % (w.name, w.B, w.H, w.dk, w.dv, args.chunk)},
        "sweep": rows, "cpu_baseline": None}))


def bench_conv(args, w, torch, binding):
    """Short-long convolution Z = K_l(silu(K_s(X))) at the workload's width: B sequences x (H*dk) channels x N steps."""
    from paper_2406_08128_amd.workloads import make_conv_inputs, to_f64_numpy
    B, d, L, m = w.B, w.H * w.dk, w.N, 9
    dt = "bf16" if w.dtype == "bf16" else "f32"
    es = 2 if dt == "bf16" else 4
    x = make_conv_inputs(B, d, L, m, w.seed, dt)
    dev = {k: v.cuda() for k, v in x.items()}
    spec = binding.chela_longconv_spectrum(dev["k_long"])
    Z = torch.empty_like(dev["X"])

    train = args.mode == "conv_train"
    if train:
        g = torch.Generator(device="cuda")
        g.manual_seed(11)
        dZ = torch.randn(B, d, L, device="cuda", generator=g).to(dev["X"].dtype)

        def step():
            binding.chela_shortlong_conv_fwd(dev["X"], dev["w_short"], spec, Z=Z)
            binding.chela_shortlong_conv_bwd(dev["X"], dev["w_short"], spec, dZ)
    else:
        def step():
            binding.chela_shortlong_conv_fwd(dev["X"], dev["w_short"], spec, Z=Z)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    binding.chela_profile_reset()
    binding.chela_profile_enable(True)
    for _ in range(args.steps):
        step()
    binding.chela_longconv_spectrum(dev["k_long"])
    torch.cuda.synchronize()
    prof = binding.chela_profile_read()
    binding.chela_profile_enable(False)
    binding.chela_profile_reset()
    kernels = {k: {"launches": n, "avg_us": round(t * 1e3 / n, 2)} for k, (n, t) in prof.items()}
    us = kernels["shortlong_conv_kernel"]["avg_us"]      # (with the backward: mean over its two kinds of launch)
    M = 256 if L <= 256 else 1024 if L <= 1024 else 4096 if L <= 4096 else 16384
    nb = (L + 16383) // 16384 if L > 16384 else 0     # beyond 16384 steps: blocks of 16384, nb (nb + 1) / 2 block pairs
    if nb:
        M = 1 << (L - 1).bit_length()                 # the flop model stays the method's: one transform of 2 M >= 2 L points
    # ALU model per sequence: two complex FFTs of length M at 5 M log2 M flops + 20 flops per spectrum pair + short kernel
    import math
    flops = B * d * (2 * 5 * M * math.log2(M) + 20 * M / 2 + 2 * m * L)       # one launch of the forward kernel
    alg = B * d * L * es * 2 + d * ((nb * 8193) if nb else (M // 2 + 1)) * 16   # X in, Z out, the kernel spectrum once
    achieved = flops / (us * 1e-6) / 1e12
    # bf16 I/O at 4096 < L <= 16384 (L a multiple of 8) runs the transforms on the matrix cores: 1280 instructions of
    # 32768 flop per pair of sequences and forward call, fp16 operands, fp32 sums
    matrix = dt == "bf16" and 4096 < L <= 16384 and L % 8 == 0 and os.environ.get("CHELA_CONV_MATRIX", "1") != "0"
    mfma_flop = d * ((B + 1) // 2) * 1280 * 32768 if matrix else 0
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import conv as oracle_conv
        # bounded sample: the direct sum is O(L^2) per sequence (512 channels at 16384 steps, fewer beyond)
        nch = min(d, 512, max(16, int(7e10 / (L * L / 2))))
        Xn = to_f64_numpy(x["X"][:1, :nch]); wn = to_f64_numpy(x["w_short"][:nch]); kn = to_f64_numpy(x["k_long"][:nch])
        import oracle
        c0 = time.perf_counter()
        oracle_conv.short_long_conv(Xn, wn, kn)
        if train:
            oracle_conv.short_long_conv_bwd(Xn, wn, kn, to_f64_numpy(dZ[:1, :nch]))
        c1 = time.perf_counter()
        cpu = {"value": round(L * nch / d / (c1 - c0), 2), "unit": "tokens/s", "cores": min(oracle.num_threads(), nch),
               "kind": "oracle", "seconds": round(c1 - c0, 3),
               "cpu_seconds": round((c1 - c0) * min(oracle.num_threads(), nch), 1),
               "sample": "fp64 direct-sum oracle on %d of the %d (batch, channel) sequences; tokens/s = L / (seconds "
                         "scaled to all %d channels of one batch entry)" % (nch, B * d, d)}
    print(json.dumps({
        "metric": "short-long convolution %s tokens/s" % ("fwd+bwd" if train else "fwd"), "value": round(B * L / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16" if matrix else "f32", "data": "synthetic",
        "config": {"workload": "conv at %s width: B%d d%d L%d, short kernel %d taps + silu + long kernel of L taps, %s I/O, %s"
                               % (w.name, B, d, L, m, dt, "transforms on the matrix cores (fp16 operands, fp32 sums), the "
                                  "rest fp32" if matrix else "fp32 arithmetic" + (", %d blocks of 16384 steps (%d forward "
                                  "block transforms and %d inverse ones per sequence)" % (nb, nb * (nb + 1) // 2, nb)
                                  if nb else ""))},
        "roofline": {"bound": "alu", "kernel": "shortlong_conv_kernel", "achieved": round(achieved, 2), "peak": 157.3,
                     "unit": "TFLOP/s", "frac": round(achieved / 157.3, 4), "traffic": None,
                     "flop_model_per_launch": flops, "avg_launch_us": us,
                     "hbm_GBs_algorithmic": round(alg / (us * 1e-6) / 1e9, 1),
                     "note": "flop model of the method (5 M log2 M per transform), whatever executes it"
                             + ("; the matrix cores execute %.3g flop per launch = %.0f TFLOP/s (%.3f of the 2.5 PFLOP/s "
                                "fp16 peak): the kernel is bound by the vector ALU work around them (rotations, "
                                "conversions, short kernel and activation)"
                                % (mfma_flop, mfma_flop / (us * 1e-6) / 1e12, mfma_flop / (us * 1e-6) / 2.5e15)
                                if matrix else "")},
        "kernels": kernels, "cpu_baseline": cpu}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (defaults: the GPU needs some 60-100 steps of this size, 20-30 ms, before its clocks have settled -- the first
    # fifty steps after an idle moment average 0.34 ms, every later block of ten 0.311-0.313 ms; 100 + 200 steps of
    # the headline workload are still under a tenth of a second of GPU time)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="lm_bf16")
    ap.add_argument("--chunk", type=int, default=64)
    ap.add_argument("--mode", default="train", choices=["train", "train_saved", "train_state", "train_bnhd", "train_z", "train_z_saved", "noncausal", "decode",
                             "conv", "conv_train", "gated", "gated_unfused", "train_layer", "train_layer_unfused", "n_sweep", "nc_gated", "nc_gated_unfused"],
                    help="train: fwd+bwd (the headline); train_saved: the same step through chela_linattn_fwd_save / "
                         "_bwd_saved (the forward leaves the boundary states, the backward skips its pass over K, V); "
                         "train_state: the same through the carried-state entry points "
                         "(S_in, S_out, dS_out, dS_in all live); train_z: queries and keys formed on chip from one tensor Z "
                         "(chela_linattn_zfwd / zbwd: three forward and five backward HBM streams); noncausal: O = Q (K^T V) "
                         "without a mask (the classification models' form); conv: the short-long convolution of "
                         "Sec. 4.2 at the workload's width (B x H*dk channels x N steps); decode: single-token steps of the recurrent form")
    ap.add_argument("--decode-batch", type=int, default=256, help="sequences decoded together in --mode decode")
    ap.add_argument("--io-dtype", default="workload", choices=["workload", "f32"],
                    help="f32: run the workload's shape through the fp32 I/O entry points (--mode train only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph (caller-owned scratch) and time replays of it instead of "
                         "eager launches")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run the library's plain copy kernel on a buffer of this many MiB (3 launches): the "
                         "kernel of known size that rocprofv3 byte counters are calibrated against")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "bwd_sweep_lm_bf16_pmc.txt"))
    ap.add_argument("--mfma-file", default=os.path.join(ROOT, "profiles", "mfma_counters_lm_bf16.txt"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X per box); --gpus %d is not supported. "
              "(b,h) pairs are independent, so N GPUs would each run this same kernel on B*H/N of them."
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_08128_amd import binding
    from paper_2406_08128_amd.workloads import WORKLOADS, make_gate_inputs, make_inputs, make_z_inputs, to_f64_numpy

    w = WORKLOADS[args.workload]
    if args.io_dtype == "f32" and w.dtype != "f32":
        assert args.mode == "train", "--io-dtype f32 goes with --mode train"
        from paper_2406_08128_amd.workloads import shrink
        w = shrink(w, dtype="f32", name=w.name + " shape with fp32 I/O")
    torch.cuda.set_device(0)
    if args.mode == "decode":
        return bench_decode(args, w, torch, binding)
    if args.mode in ("conv", "conv_train"):
        return bench_conv(args, w, torch, binding)
    if args.mode == "n_sweep":
        return bench_n_sweep(args, w, torch, binding)
    has_bwd = w.backward          # the headline workload runs forward + backward; forward-only workloads time the forward
    if args.mode in ("gated", "gated_unfused", "nc_gated", "nc_gated_unfused"):
        has_bwd = False           # Eq. 9 at inference
    elif args.mode in ("train_layer", "train_layer_unfused"):
        has_bwd = True
    es = 2 if w.dtype == "bf16" else 4
    x = make_inputs(w, with_dO=has_bwd)
    d = {k: v.cuda() for k, v in x.items()}
    O = torch.empty_like(d["V"])
    dQ, dK, dV = (torch.empty_like(d["Q"]), torch.empty_like(d["K"]), torch.empty_like(d["V"])) if has_bwd else (None,) * 3
    chunk = args.chunk

    if args.mode == "train_state":
        assert has_bwd and w.dtype == "bf16", "--mode train_state needs a bf16 forward+backward workload"
        g = torch.Generator(device="cuda")
        g.manual_seed(7)
        S_in = torch.randn(w.B, w.H, w.dk, w.dv, device="cuda", generator=g)
        dS_out = torch.randn(w.B, w.H, w.dk, w.dv, device="cuda", generator=g)
        S_out = torch.empty_like(S_in)

        def step():
            binding.chela_linattn_fwd_state(d["Q"], d["K"], d["V"], S_in=S_in, O=O, S_out=S_out, chunk=chunk)
            binding.chela_linattn_bwd_state(d["Q"], d["K"], d["V"], d["dO"], S_in=S_in, dS_out=dS_out, chunk=chunk)
    elif args.mode == "train_saved":
        assert has_bwd and w.dtype == "bf16", "--mode train_saved needs a bf16 forward+backward workload"
        saved = torch.empty(max(binding.chela_linattn_saved_bytes(w.B, w.H, w.N, w.dk, w.dv, chunk), 16) // 4,
                            dtype=torch.float32, device="cuda")

        def step():
            binding.chela_linattn_fwd_save(d["Q"], d["K"], d["V"], O=O, saved=saved, chunk=chunk)
            binding.chela_linattn_bwd_saved(d["Q"], d["K"], d["V"], d["dO"], saved, dQ=dQ, dK=dK, dV=dV, chunk=chunk)
    elif args.mode == "train_bnhd":
        assert w.dtype == "bf16", "--mode train_bnhd needs a bf16 workload"
        t = {k: v.transpose(1, 2).contiguous() for k, v in d.items()}          # [B,N,H,d]
        Ot = torch.empty_like(t["V"])
        if has_bwd:
            def step():
                binding.chela_linattn_fwd_bnhd(t["Q"], t["K"], t["V"], O=Ot)
                binding.chela_linattn_bwd_bnhd(t["Q"], t["K"], t["V"], t["dO"])
        else:
            def step():
                binding.chela_linattn_fwd_bnhd(t["Q"], t["K"], t["V"], O=Ot)
    elif args.mode == "noncausal":
        assert w.dtype == "bf16", "--mode noncausal needs a bf16 workload"
        if has_bwd:
            def step():
                binding.chela_linattn_noncausal_fwd(d["Q"], d["K"], d["V"], O=O)
                binding.chela_linattn_noncausal_bwd(d["Q"], d["K"], d["V"], d["dO"])
        else:
            def step():
                binding.chela_linattn_noncausal_fwd(d["Q"], d["K"], d["V"], O=O)
    elif args.mode in ("nc_gated", "nc_gated_unfused"):
        # the non-causal form with the Eq. 9 epilogue (what a classifier runs at inference)
        assert w.dtype == "bf16", "--mode nc_gated needs a bf16 workload"
        gate = make_gate_inputs(w)["G"].cuda()
        Y = torch.empty_like(O)
        if args.mode == "nc_gated":
            def step():
                binding.chela_linattn_noncausal_fwd_gated(d["Q"], d["K"], d["V"], gate, 1e-5, Y=Y)
        else:
            def step():
                binding.chela_linattn_noncausal_fwd(d["Q"], d["K"], d["V"], O=O)
                binding.chela_gate_norm_fwd(O, gate, 1e-5, Y=Y)
    elif args.mode in ("gated", "gated_unfused"):
        # Eq. 9 at inference: Y = Norm(O) * G; fused into the forward, or as a second pass over a stored O
        assert w.dtype == "bf16", "--mode gated needs a bf16 workload"
        gate = make_gate_inputs(w)["G"].cuda()
        Y = torch.empty_like(O)
        if args.mode == "gated":
            def step():
                binding.chela_linattn_fwd_gated(d["Q"], d["K"], d["V"], gate, 1e-5, Y=Y)
        else:
            def step():
                binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], O=O, chunk=chunk)
                binding.chela_gate_norm_fwd(O, gate, 1e-5, Y=Y)
    elif args.mode in ("train_layer", "train_layer_unfused"):
        # the layer's attention core in training: Z, V, G -> Y, then dY -> dZ, d_affine, dV, dG
        assert w.dtype == "bf16", "--mode train_layer needs a bf16 workload"
        dz = {k: v.cuda() for k, v in make_z_inputs(w, with_dO=False).items()}
        gi = {k: v.cuda() for k, v in make_gate_inputs(w).items()}
        Y, dOb, dG = torch.empty_like(O), torch.empty_like(O), torch.empty_like(O)
        saved = torch.empty(max(binding.chela_linattn_saved_bytes(w.B, w.H, w.N, w.dk, w.dv, 64), 16) // 4,
                            dtype=torch.float32, device="cuda")
        if args.mode == "train_layer":
            def step():
                binding.chela_linattn_zfwd_gated(dz["Z"], dz["affine"], dz["V"], gi["G"], 1e-5, Y=Y, O=O, saved=saved)
                binding.chela_gate_norm_bwd(O, gi["G"], gi["dY"], 1e-5, dO=dOb, dG=dG)
                binding.chela_linattn_zbwd_saved(dz["Z"], dz["affine"], dz["V"], dOb, saved)
        else:
            def step():
                binding.chela_linattn_zfwd_save(dz["Z"], dz["affine"], dz["V"], O=O, saved=saved)
                binding.chela_gate_norm_fwd(O, gi["G"], 1e-5, Y=Y)
                binding.chela_gate_norm_bwd(O, gi["G"], gi["dY"], 1e-5, dO=dOb, dG=dG)
                binding.chela_linattn_zbwd_saved(dz["Z"], dz["affine"], dz["V"], dOb, saved)
    elif args.mode in ("train_z", "train_z_saved"):
        assert w.dtype == "bf16", "--mode train_z needs a bf16 workload"
        xz = make_z_inputs(w, with_dO=has_bwd)
        dz = {k: v.cuda() for k, v in xz.items()}
        if args.mode == "train_z_saved":
            assert has_bwd, "--mode train_z_saved needs a forward+backward workload"
            saved = torch.empty(max(binding.chela_linattn_saved_bytes(w.B, w.H, w.N, w.dk, w.dv, 64), 16) // 4,
                                dtype=torch.float32, device="cuda")

            def step():
                binding.chela_linattn_zfwd_save(dz["Z"], dz["affine"], dz["V"], O=O, saved=saved)
                binding.chela_linattn_zbwd_saved(dz["Z"], dz["affine"], dz["V"], dz["dO"], saved)
        elif has_bwd:
            def step():
                binding.chela_linattn_zfwd(dz["Z"], dz["affine"], dz["V"], O=O)
                binding.chela_linattn_zbwd(dz["Z"], dz["affine"], dz["V"], dz["dO"])
        else:
            def step():
                binding.chela_linattn_zfwd(dz["Z"], dz["affine"], dz["V"], O=O)
    elif has_bwd:
        def step():
            binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], O=O, chunk=chunk)
            binding.chela_linattn_bwd(d["Q"], d["K"], d["V"], d["dO"], dQ=dQ, dK=dK, dV=dV, chunk=chunk)
    else:
        def step():
            binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], O=O, chunk=chunk)

    if args.copy_probe_mib > 0:
        src = torch.zeros(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            binding.chela_copy_probe(src, dst)
        torch.cuda.synchronize()
        del src, dst

    eager_step = step
    if args.graph:
        # nothing may be allocated while capturing: hand the library a scratch buffer of the size a first eager step
        # made it allocate, then record the step once
        step()
        torch.cuda.synchronize()
        ws_buf = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        binding.chela_set_workspace(ws_buf)
        cap_stream = torch.cuda.Stream()
        with torch.cuda.stream(cap_stream):
            step()
        cap_stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap_stream):
            step()
        step = graph.replay
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.tokens / (ms_per_step * 1e-3)

    # Per-kernel durations: the same steps again with the library's HIP-event brackets switched on (events are
    # recorded on the launch stream around each kernel).  Kept out of the region that `value` is computed from.
    binding.chela_profile_reset()
    binding.chela_profile_enable(True)
    for _ in range(args.steps):
        eager_step()
    torch.cuda.synchronize()
    prof = binding.chela_profile_read()
    binding.chela_profile_enable(False)
    binding.chela_profile_reset()
    kernels = {k: {"launches": n, "avg_us": ms * 1e3 / n} for k, (n, ms) in prof.items()}

    fwd_b, bwd_b = algorithmic_bytes_per_token_head(w.dk, w.dv, es)
    if args.mode in ("train_z", "train_z_saved"):     # Z replaces Q and K on the way in, dZ replaces dQ and dK on the way out
        fwd_b, bwd_b = es * (w.dk + 2 * w.dv), es * (w.dk + 2 * w.dv + w.dk + w.dv)
    elif args.mode in ("gated", "gated_unfused"):     # the gate comes in as a fifth tensor; unfused: O out, O and G in, Y out
        fwd_b = es * (2 * w.dk + 3 * w.dv) if args.mode == "gated" else es * (2 * w.dk + 5 * w.dv)
    elif args.mode in ("train_layer", "train_layer_unfused"):
        # forward Z,V,G -> Y,O; epilogue gradient O,G,dY -> dO,dG; backward Z,V,dO -> dZ,dV
        fwd_b = es * (w.dk + 4 * w.dv) + (0 if args.mode == "train_layer" else es * 2 * w.dv)
        bwd_b = es * (5 * w.dv) + es * (2 * w.dk + 3 * w.dv)
    fwd_f, bwd_f = flops_per_token_head(w.dk, w.dv, chunk)
    th = w.token_heads
    if args.mode == "noncausal":    # the apply kernel reads one tensor and writes one; forward: Q in, O out
        dom, dom_b = "bf16_apply_state_kernel", es * (w.dk + w.dv)
    elif args.mode in ("nc_gated", "nc_gated_unfused"):
        dom, dom_b = "bf16_apply_state_kernel", es * (w.dk + (2 if args.mode == "nc_gated" else 1) * w.dv)
        fwd_b = es * (2 * w.dk + (3 if args.mode == "nc_gated" else 5) * w.dv)
    elif w.dtype != "bf16":
        dom, dom_b = "f32_sweep_kernel", fwd_b
    elif args.mode in ("train_layer", "train_layer_unfused"):
        dom, dom_b = "bf16_bwd_sweep_kernel", es * (2 * w.dk + 3 * w.dv)
    elif args.mode == "gated_unfused":
        dom, dom_b = "bf16_fwd_sweep_kernel", es * (2 * w.dk + 2 * w.dv)
    elif has_bwd:
        dom, dom_b = "bf16_bwd_sweep_kernel", bwd_b
    else:
        dom, dom_b = "bf16_fwd_sweep_kernel", fwd_b
    dom_us = kernels[dom]["avg_us"]
    achieved = dom_b * th / (dom_us * 1e-6) / 1e9
    sources_hash = binding.kernel_sources_sha256()
    headline = args.workload == "lm_bf16" and chunk == 64 and w.dtype == "bf16" and args.mode == "train"
    traffic, traffic_src, mfma_counted = None, None, None
    if headline:
        # counters of the dominant kernel, from the committed summaries of rocprofv3 --pmc runs of this same command
        kv, traffic_src = read_profile(args.traffic_file, sources_hash)
        if kv and "traffic_bytes_per_launch" in kv:
            traffic = float(kv["traffic_bytes_per_launch"])
        kv, mfma_src = read_profile(args.mfma_file, sources_hash)
        mfma_counted = {"source": mfma_src}
        if kv and "mfma_flop_per_launch" in kv:
            fl = float(kv["mfma_flop_per_launch"])
            mfma_counted.update({"flop_per_launch": fl, "TFLOPs": round(fl / (dom_us * 1e-6) / 1e12, 1),
                                 "frac_of_peak": round(fl / (dom_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                 "pipe_busy_frac": float(kv["mfma_busy_frac"]) if "mfma_busy_frac" in kv else None})
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": dom_b * th, "avg_launch_us": round(dom_us, 2)}
    if traffic_src is not None:
        roofline["traffic_source"] = traffic_src
    if mfma_counted is not None:
        roofline["mfma_counted"] = mfma_counted
    # What the GPU delivers for the dominant kernel's mix of streams when nothing but streaming is asked of it: the
    # library's plain grid-stride kernel on as many read and written arrays, of the same total size.
    if dom == "bf16_bwd_sweep_kernel":
        n_rd, n_wr = (3, 2) if args.mode in ("train_z", "train_z_saved", "train_layer", "train_layer_unfused") else (4, 3)
    elif dom == "bf16_apply_state_kernel":
        n_rd, n_wr = (2, 1) if args.mode == "nc_gated" else (1, 1)
    else:
        n_rd, n_wr = (4, 1) if args.mode == "gated" else (3, 1)
    each = (dom_b * th // (n_rd + n_wr)) // 16 * 16
    # (enough sets of arrays, used in turn, that a launch never finds its arrays in the 256 MB memory-side cache)
    n_sets = min(8, max(1, -(-(1 << 30) // max(1, each * (n_rd + n_wr)))))
    sets = [[torch.empty(each, dtype=torch.uint8, device="cuda") for _ in range(n_rd + n_wr)] for _ in range(n_sets)]
    for bufs in sets:
        for b in bufs[:n_rd]:
            b.zero_()
    for i in range(3):
        binding.chela_stream_probe(sets[i % n_sets][:n_rd], sets[i % n_sets][n_rd:])
    torch.cuda.synchronize()
    binding.chela_profile_reset()
    binding.chela_profile_enable(True)
    for i in range(20):
        binding.chela_stream_probe(sets[i % n_sets][:n_rd], sets[i % n_sets][n_rd:])
    torch.cuda.synchronize()
    sp = binding.chela_profile_read()["stream_probe_kernel"]
    binding.chela_profile_enable(False)
    binding.chela_profile_reset()
    del sets, bufs
    sp_us = sp[1] * 1e3 / sp[0]
    sp_gbs = each * (n_rd + n_wr) / (sp_us * 1e-6) / 1e9
    roofline["stream_mix"] = {"reads": n_rd, "writes": n_wr, "bytes_per_launch": each * (n_rd + n_wr),
                              "avg_launch_us": round(sp_us, 2), "GB/s": round(sp_gbs, 1)}
    roofline["frac_of_stream_mix"] = round(achieved / sp_gbs, 4)
    # The matrix rate the GPU delivers when nothing but matrix instructions are asked of it (registers only).
    mf_blocks, mf_iters = 256 * 8, 1024
    mf_out = torch.empty(mf_blocks * 256, dtype=torch.float32, device="cuda")
    for _ in range(2):
        binding.chela_mfma_probe(mf_out, mf_blocks, mf_iters)
    torch.cuda.synchronize()
    binding.chela_profile_reset()
    binding.chela_profile_enable(True)
    for _ in range(5):
        mf_flop = binding.chela_mfma_probe(mf_out, mf_blocks, mf_iters)
    torch.cuda.synchronize()
    mp = binding.chela_profile_read()["mfma_probe_kernel"]
    binding.chela_profile_enable(False)
    binding.chela_profile_reset()
    del mf_out
    mfma_measured = mf_flop / (mp[1] / mp[0] * 1e-3) / 1e12
    measured_peaks = {"mfma_bf16_TFLOPs": round(mfma_measured, 1),
                      "mfma_bf16_frac_of_published": round(mfma_measured / MFMA_BF16_PEAK_TFLOPS, 4),
                      "stream_mix_GBs": round(sp_gbs, 1),
                      "note": "plain kernels of this library: matrix instructions on registers only; a grid-stride "
                              "stream over as many read and written arrays as the dominant kernel moves"}

    # Forward and backward on their own (outside the region `value` is computed from).
    phases = None
    if has_bwd and args.mode == "train" and not args.graph:
        def time_loop(fn):
            for _ in range(max(2, args.warmup // 2)):
                fn()
            torch.cuda.synchronize()
            a = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - a) * 1e3 / args.steps
        f_ms = time_loop(lambda: binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], O=O, chunk=chunk))
        b_ms = time_loop(lambda: binding.chela_linattn_bwd(d["Q"], d["K"], d["V"], d["dO"], dQ=dQ, dK=dK, dV=dV,
                                                           chunk=chunk))
        phases = {"fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                  "note": "each call timed in a loop of its own: what a kernel finds in the memory-side cache "
                          "differs from the alternating step, so the two need not add up to ms_per_step"}

    # The same step through the training pair (the forward leaves the boundary states, the backward's pre-pass then
    # reads Q and dO only): what a training loop that calls both would use.  Outside the region `value` comes from.
    training_pair = None
    if phases is not None and w.dtype == "bf16":
        sv = torch.empty(max(binding.chela_linattn_saved_bytes(w.B, w.H, w.N, w.dk, w.dv, chunk), 16) // 4,
                         dtype=torch.float32, device="cuda")

        def pair_step():
            binding.chela_linattn_fwd_save(d["Q"], d["K"], d["V"], O=O, saved=sv, chunk=chunk)
            binding.chela_linattn_bwd_saved(d["Q"], d["K"], d["V"], d["dO"], sv, dQ=dQ, dK=dK, dV=dV, chunk=chunk)
        p_ms = time_loop(pair_step)
        training_pair = {"entry_points": "chela_linattn_fwd_save + chela_linattn_bwd_saved",
                         "ms_per_step": round(p_ms, 4), "tokens_per_s": round(w.tokens / (p_ms * 1e-3), 1),
                         "vs_plain_pair": round(p_ms / ms_per_step, 4)}
        del sv

    # The same step over three sets of tensors used in turn (outside the region `value` comes from): no call then finds
    # its inputs in the 256 MB memory-side cache because the step before touched them, which a loop over one set of
    # tensors allows and a model, whose next call works on other tensors, does not.
    rotating = None
    if args.mode == "train" and w.dtype == "bf16" and not args.graph:
        n_rot = 3
        rsets = [(d, O, dQ, dK, dV)]
        for _ in range(n_rot - 1):
            dd = {k: v.clone() for k, v in d.items()}
            rsets.append((dd, torch.empty_like(O)) + tuple(torch.empty_like(t) if t is not None else None
                                                            for t in (dQ, dK, dV)))

        def rot_step(i):
            dd, o_, dq_, dk_, dv_ = rsets[i % n_rot]
            binding.chela_linattn_fwd(dd["Q"], dd["K"], dd["V"], O=o_, chunk=chunk)
            if has_bwd:
                binding.chela_linattn_bwd(dd["Q"], dd["K"], dd["V"], dd["dO"], dQ=dq_, dK=dk_, dV=dv_, chunk=chunk)
        for i in range(max(6, args.warmup // 2)):
            rot_step(i)
        torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(args.steps):
            rot_step(i)
        torch.cuda.synchronize()
        r_ms = (time.perf_counter() - a) * 1e3 / args.steps
        rotating = {"sets": n_rot, "ms_per_step": round(r_ms, 4), "tokens_per_s": round(w.tokens / (r_ms * 1e-3), 1),
                    "vs_one_set": round(r_ms / ms_per_step, 4)}
        del rsets

    # What plain streaming kernels need for the bytes this step's kernels HAVE to move in the three-launch structure
    # (every input once per pass that needs it, every output once; states left out): the pre-pass of the forward call
    # reads K, V of all but the last segment, its sweep reads Q, K, V and writes O, the backward's pre-pass reads
    # Q, K, V, dO, its sweep reads them again and writes dQ, dK, dV.  Each line is the stream probe on as many arrays
    # of the tensors' size (widths differ: arrays of the mean width, same total bytes).
    stream_floor = None
    if args.mode == "train" and w.dtype == "bf16" and not args.graph:
        def probe_us(n_rd, n_wr, total_bytes):
            each = (int(total_bytes) // (n_rd + n_wr)) // 16 * 16
            n_sets = min(8, max(2, -(-(1 << 30) // max(1, each * (n_rd + n_wr)))))
            sets = [[torch.zeros(each, dtype=torch.uint8, device="cuda") for _ in range(n_rd + n_wr)] for _ in range(n_sets)]
            for i in range(3):
                binding.chela_stream_probe(sets[i % n_sets][:n_rd], sets[i % n_sets][n_rd:])
            torch.cuda.synchronize()
            binding.chela_profile_reset()
            binding.chela_profile_enable(True)
            for i in range(16):
                binding.chela_stream_probe(sets[i % n_sets][:n_rd], sets[i % n_sets][n_rd:])
            torch.cuda.synchronize()
            r = binding.chela_profile_read()["stream_probe_kernel"]
            binding.chela_profile_enable(False)
            binding.chela_profile_reset()
            return r[1] * 1e3 / r[0]
        tb_k, tb_v = th * w.dk * es, th * w.dv * es
        # segments per sequence of the forward call's plan (one: no pre-pass at all)
        n_seg = max(1, binding.chela_linattn_workspace_bytes(w.B, w.H, w.N, w.dk, w.dv, chunk, False, binding.DTYPE_BF16)
                    // (w.B * w.H * w.dk * w.dv * 4))
        seg_frac = (n_seg - 1) / n_seg
        parts = {}
        if n_seg > 1:
            parts["fwd_prepass_2r"] = probe_us(2, 0, seg_frac * (tb_k + tb_v))
        parts["fwd_sweep_3r_1w"] = probe_us(3, 1, 2 * tb_k + 2 * tb_v)
        if has_bwd:
            parts["bwd_prepass_4r"] = probe_us(4, 0, 2 * tb_k + 2 * tb_v)
            parts["bwd_sweep_4r_3w"] = probe_us(4, 3, 4 * tb_k + 3 * tb_v)
        tot = sum(parts.values())
        stream_floor = {"us_per_part": {k: round(v, 1) for k, v in parts.items()}, "us": round(tot, 1),
                        "bytes": int((seg_frac * (tb_k + tb_v) if n_seg > 1 else 0) + (2 * tb_k + 2 * tb_v)
                                     + ((2 * tb_k + 2 * tb_v) + 4 * tb_k + 3 * tb_v if has_bwd else 0)),
                        "segments_per_sequence": n_seg,
                        "step_over_floor": round(ms_per_step * 1e3 / tot, 3),
                        "note": "plain grid-stride kernels moving what the pre-passes and sweeps of this step must "
                                "move, each on arrays that nothing has touched just before (kernel time only, no "
                                "launch gaps).  A step below this (step_over_floor < 1) has found part of what it "
                                "reads in the 256 MB memory-side cache: a sweep re-reads what its pre-pass has just "
                                "read, and the outputs leave as streaming stores so that they do not push those "
                                "lines out; rotating_sets gives the step when at least no call finds its inputs "
                                "there because the step before used the same tensors"}

    step_bytes = (fwd_b + (bwd_b if has_bwd else 0)) * th
    step_flops = (fwd_f + (bwd_f if has_bwd else 0)) * th
    whole = {"hbm_GBs_algorithmic": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
             "hbm_frac": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
             "mfma_TFLOPs_full_tile_model": round(step_flops / (ms_per_step * 1e-3) / 1e12, 1),
             "mfma_frac": round(step_flops / (ms_per_step * 1e-3) / 1e12
                                / (MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS), 4)}
    if w.dtype == "bf16":
        whole["mfma_frac_of_measured_peak"] = round(step_flops / (ms_per_step * 1e-3) / 1e12 / mfma_measured, 4)
    whole["hbm_frac_of_stream_mix"] = round(step_bytes / (ms_per_step * 1e-3) / 1e9 / sp_gbs, 4)
    if stream_floor is not None:
        whole["stream_floor"] = stream_floor
    target = None
    if headline:
        target = {"north_star": ">= 50 % of peak bf16 MFMA at B4 H12 N16384 d64, as shown by rocprof",
                  "met": False,
                  "mfma_frac_whole_step_full_tile_model": whole["mfma_frac"],
                  "mfma_frac_dominant_kernel_counted": (mfma_counted or {}).get("frac_of_peak"),
                  "why": "the path is HBM-bound: 1408 B and 114688 FLOP per token-head at chunk 64 = 81 FLOP/B against "
                         "a ridge of 312 FLOP/B; even at the 8 TB/s floor (138 us per step) chunk 64 would be 26 % of "
                         "peak.  The primary roofline is the HBM one (roofline.frac, whole_step.hbm_frac)."}

    cpu = None
    cpu_reps = 1
    parity_rel_l2 = None
    if not args.no_cpu_baseline:
        import oracle
        if args.mode in ("nc_gated", "nc_gated_unfused"):
            from oracle import layer as oracle_layer
            Qn, Kn, Vn, Gg = (to_f64_numpy(t) for t in (x["Q"], x["K"], x["V"], gate))
            c0 = time.perf_counter()
            oracle_layer.gate_norm_fwd(oracle_layer.noncausal_fwd(Qn, Kn, Vn), Gg, 1e-5)
            c1 = time.perf_counter()
        elif args.mode == "noncausal":
            from oracle import layer as oracle_layer
            Qn, Kn, Vn = (to_f64_numpy(x[n]) for n in ("Q", "K", "V"))
            Gn = to_f64_numpy(x["dO"]) if has_bwd else None
            c0 = time.perf_counter()
            oracle_layer.noncausal_fwd(Qn, Kn, Vn)
            if has_bwd:
                oracle_layer.noncausal_bwd(Qn, Kn, Vn, Gn)
            c1 = time.perf_counter()
        elif args.mode in ("gated", "gated_unfused"):
            from oracle import layer as oracle_layer
            Qn, Kn, Vn, Gg = (to_f64_numpy(t) for t in (x["Q"], x["K"], x["V"], gate))
            c0 = time.perf_counter()
            oracle_layer.gated_fwd(Qn, Kn, Vn, Gg, 1e-5)
            c1 = time.perf_counter()
        elif args.mode in ("train_layer", "train_layer_unfused"):
            from oracle import layer as oracle_layer
            Zn, An, Vn, Gg, dYn = (to_f64_numpy(t) for t in (dz["Z"], dz["affine"], dz["V"], gi["G"], gi["dY"]))
            c0 = time.perf_counter()
            Qn, Kn = oracle_layer.qk_from_z(Zn, An)
            On, _ = oracle_layer.gated_fwd(Qn, Kn, Vn, Gg, 1e-5)
            dOn, _ = oracle_layer.gate_norm_bwd(On, Gg, dYn, 1e-5)
            oracle_layer.zqk_bwd(Zn, An, Vn, dOn)
            c1 = time.perf_counter()
        elif args.mode in ("train_z", "train_z_saved"):
            from oracle import layer as oracle_layer
            Zn, An, Vn = (to_f64_numpy(xz[n]) for n in ("Z", "affine", "V"))
            Gn = to_f64_numpy(xz["dO"]) if has_bwd else None
            c0 = time.perf_counter()
            oracle_layer.zqk_fwd(Zn, An, Vn)
            if has_bwd:
                oracle_layer.zqk_bwd(Zn, An, Vn, Gn)
            c1 = time.perf_counter()
        else:
            Qn, Kn, Vn = (to_f64_numpy(x[n]) for n in ("Q", "K", "V"))
            Gn = to_f64_numpy(x["dO"]) if has_bwd else None
            cpu_reps = 0
            c0 = time.perf_counter()
            while True:           # whole passes over the workload until about a second of wall time on all threads
                oracle.fwd_recurrent(Qn, Kn, Vn)
                if has_bwd:
                    oracle.bwd_recurrent(Qn, Kn, Vn, Gn)
                cpu_reps += 1
                c1 = time.perf_counter()
                if c1 - c0 >= 1.0 or cpu_reps >= 8:
                    break
        if args.mode == "train" and w.dtype in ("bf16", "f32"):
            # rel-L2 of every output against the oracle on a sample of (b,h) pairs (outside every timed region)
            O_s = binding.chela_linattn_fwd(d["Q"], d["K"], d["V"], chunk=chunk)
            outs = [O_s] + (list(binding.chela_linattn_bwd(d["Q"], d["K"], d["V"], d["dO"], chunk=chunk)) if has_bwd else [])
            torch.cuda.synchronize()
            bh = w.B * w.H
            pick = sorted({0, bh // 3, bh - 1})
            sel = lambda t: t.reshape(1, bh, w.N, -1)[:, pick]
            Qs, Ks, Vs = (to_f64_numpy(sel(x[n])) for n in ("Q", "K", "V"))
            refs = [oracle.fwd_recurrent(Qs, Ks, Vs)]
            if has_bwd:
                refs += list(oracle.bwd_recurrent(Qs, Ks, Vs, to_f64_numpy(sel(x["dO"]))))
            parity_rel_l2 = {n: float("%.3e" % oracle.rel_l2(to_f64_numpy(sel(g)), r))
                             for n, g, r in zip(("O", "dQ", "dK", "dV"), outs, refs)}
            parity_rel_l2["sample"] = "(b,h) pairs %s of %d, every token; bar %s" % (pick, bh, "2e-2" if w.dtype == "bf16" else "1e-5")
        cpu = {"value": round(cpu_reps * w.tokens / (c1 - c0), 1), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle", "seconds": round(c1 - c0, 3),
               "cpu_seconds": round((c1 - c0) * oracle.num_threads(), 1),       # wall time x threads: the CPU work done
               "sample": "fp64 oracle, %s, all %d (b,h) pairs of the workload, %d repetition%s"
                         % ("fwd+bwd" if has_bwd else "fwd", w.B * w.H, cpu_reps, "" if cpu_reps == 1 else "s")}

    out = {
        "metric": "%s linear-attn %s tokens/s" % ("non-causal" if args.mode in ("noncausal", "nc_gated", "nc_gated_unfused") else "causal",
                                                  "fwd+bwd" if has_bwd else "fwd")
                  + (" (carried-state entry points)" if args.mode == "train_state" else "")
                  + (" (forward saves the boundary states)" if args.mode == "train_saved" else "")
                  + (" ([B,N,H,d] tensors)" if args.mode == "train_bnhd" else "")
                  + (" (Q, K formed on chip from Z)" if args.mode == "train_z" else "")
                  + (" (Q, K formed on chip from Z; forward saves the boundary states)" if args.mode == "train_z_saved" else "")
                  + (" (Y = Norm(O) * G inside the forward)" if args.mode in ("gated", "nc_gated") else "")
                  + (" (Y = Norm(O) * G as a second pass)" if args.mode == "nc_gated_unfused" else "")
                  + (" (Y = Norm(O) * G as a second pass)" if args.mode == "gated_unfused" else "")
                  + (" (layer core: Z, V, G -> Y and all gradients, prologue and epilogue fused)" if args.mode == "train_layer" else "")
                  + (" (layer core: Z, V, G -> Y and all gradients, epilogue as a separate pass)" if args.mode == "train_layer_unfused" else ""),
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: B%d H%d N%d dk%d dv%d %s, %s, chunk %d"
                               % (w.name, w.B, w.H, w.N, w.dk, w.dv,
                                  "bf16 I/O fp32 accumulate" if w.dtype == "bf16" else "fp32 I/O",
                                  "fwd+bwd" if has_bwd else "fwd", chunk),
                   "tokens_per_step": w.tokens, "token_heads_per_step": th},
        "roofline": roofline,
        "whole_step": whole,
        "measured_peaks": measured_peaks,
        "kernels": {k: {"launches": v["launches"], "avg_us": round(v["avg_us"], 2)} for k, v in kernels.items()},
        "cpu_baseline": cpu,
        "build": {"kernel_sources_sha256": sources_hash},
    }
    if phases is not None:
        out["phases"] = phases
    if training_pair is not None:
        out["training_pair"] = training_pair
    if rotating is not None:
        out["rotating_sets"] = rotating
    if parity_rel_l2 is not None:
        out["parity_rel_l2"] = parity_rel_l2
    if target is not None:
        out["target"] = target
    print(json.dumps(out))


if __name__ == "__main__":
    main()
