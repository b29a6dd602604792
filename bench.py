"""Benchmark of the GKA layer forward hot path (libgka) on one MI355X.

One step = one gka_forward over the single-layer bf16 workload (B=4, H=16, T=4096, d=128, chunk 64,
n_iter=10), inputs resident in HBM. Prints one JSON line: layer tokens/s, the roofline of the dominant
kernel (the fused chunk-walk kernel, bf16 MFMA bound) from HIP-event timings taken on the launch stream,
and the fp64 CPU oracle timed on this machine's host cores on the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
HBM_PEAK_GBS = 8000.0              # MI355X HBM3E peak
N_INPUT_SETS = 3                   # rotated so that the 256 MiB of q,k,v,o do not sit in the last-level cache
# An idle GPU needs tens of milliseconds of work before its clocks settle; a step is a third of a millisecond. These
# untimed forward passes run before the W warm-up steps whatever W is (reported as "clock_ramp_steps").
CLOCK_RAMP_STEPS = 300
FUSED_KERNEL = "gka::fused_forward_kernel<false, false>(gka::FusedArgs)"
TWO_PHASE_SOLVE_KERNEL = "gka::chunk_solve_kernel_bf16<gka::IOBF16, 128, false>(gka::SolveArgs)"


def committed_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summaries (profiles/*.md, lines of the
    form `traffic_bytes_per_launch <kernel>: <bytes>`), or None: counters are collected in runs of their own, not here."""
    pdir = os.path.join(ROOT, "profiles")
    try:
        for name in sorted(os.listdir(pdir)):
            if not name.endswith(".md"):
                continue
            with open(os.path.join(pdir, name)) as f:
                for line in f:
                    if line.startswith("traffic_bytes_per_launch ") and kernel in line:
                        return int(line.rsplit(":", 1)[1].strip())
    except OSError:
        pass
    return None


def algorithmic_flops_per_chunk(d, C, r):
    """Causal algorithmic FLOPs of one (pair, chunk): S2 chunk deltas, S4 Frobenius, S5 r Chebyshev
    passes, S6 readout. delta = number of causal (j <= c) pairs."""
    delta = C * (C + 1) // 2
    f_s2 = 4 * C * d * d
    f_s4 = 2 * C * d * d + 2 * delta * d + 2 * C * delta
    f_s5 = r * (2 * C * d * d + 4 * delta * d)
    f_s6 = 2 * C * d * d + 4 * delta * d
    return f_s2, f_s4, f_s5, f_s6


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step is about half a millisecond; the clocks of an idle GPU take tens of milliseconds of work to settle
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--n-iter", type=int, default=None,
                    help="profiling aid: another number of Chebyshev passes than the workload's 10 (the difference "
                         "between two counts isolates the passes); the JSON line then describes that variant")
    ap.add_argument("--path", choices=["auto", "two-phase"], default="auto",
                    help="profiling aid: time the two-phase kernels (chunk states through the workspace) instead of "
                         "the library's choice, the fused kernels; the JSON line then describes that variant")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-backward", action="store_true")
    ap.add_argument("--no-sketch", action="store_true")
    ap.add_argument("--no-head-dims", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); every (batch, head) pair is independent, "
              "so more GPUs would shard pairs with no communication.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_21016_amd import binding, synth
    from gka_testutil import pair_rel_err, to_host, upload_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU available", file=sys.stderr)
        sys.exit(1)
    binding.load_library()          # fails loudly when the HIP library has not been built

    w = synth.CFG2 if args.n_iter is None else synth.CFG2.scaled(n_iter=args.n_iter)
    sets_host = [synth.make_inputs(w.scaled(seed=w.seed + 100 * i)) for i in range(N_INPUT_SETS)]
    sets = [upload_inputs(x, w.dtype) for x in sets_host]
    two_phase = args.path == "two-phase"
    params = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_BF16,
                                 path=binding.GKA_PATH_TWO_PHASE if two_phase else binding.GKA_PATH_AUTO)
    ws = torch.empty(binding.forward_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    outs = [torch.empty_like(s["v"]) for s in sets]

    # raw device addresses, marshalled once: a step is then a single C call that enqueues the kernels
    stream = torch.cuda.current_stream().cuda_stream
    ptrs = [tuple(s[name].data_ptr() for name in ("q", "k", "v", "gate", "lam")) + (o.data_ptr(),)
            for s, o in zip(sets, outs)]
    ws_ptr, ws_bytes = ws.data_ptr(), ws.numel()

    def step(i):
        q, k, v, gate, lam, o = ptrs[i % N_INPUT_SETS]
        st = binding.forward_raw(params, q, k, v, gate, lam, o, workspace=ws_ptr, workspace_bytes=ws_bytes,
                                 stream=stream)
        if st != binding.GKA_OK:
            raise binding.GkaError(st, binding.status_string(st))

    # A plain 1 GiB device copy, untimed: under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` it calibrates the counters.
    calib_src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    del calib_src, calib_dst

    for i in range(CLOCK_RAMP_STEPS):
        step(i)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K whole forward passes
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps

    # ---- per-kernel timing: the library brackets its launches with HIP events on the same stream
    ms_states = ms_solve = 0.0
    n_launches = 1
    for i in range(args.steps):
        q, k, v, gate, lam, o = ptrs[i % N_INPUT_SETS]
        st, a, b, n_launches = binding.forward_profile_raw(params, q, k, v, gate, lam, o, ws_ptr, ws_bytes, stream)
        if st != binding.GKA_OK:
            raise binding.GkaError(st, binding.status_string(st))
        ms_states += a / args.steps
        ms_solve += b / args.steps
    ms_solve_launch = ms_solve / n_launches

    n_chunks = w.B * w.H * (w.T // w.chunk)
    f_s2, f_s4, f_s5, f_s6 = algorithmic_flops_per_chunk(w.d, w.chunk, w.n_iter)
    flops_total = n_chunks * (f_s2 + f_s4 + f_s5 + f_s6)
    tokens = w.B * w.T
    tflops_total = flops_total / (ms_per_step * 1e-3) / 1e12
    # the fused kernel does all of S1-S6 for every chunk (the summary launch before it repeats part of S2 and is
    # not counted as algorithmic work)
    tflops_solve = flops_total / (ms_solve_launch * 1e-3) / 1e12
    phase_names = ("segment_summaries", "chunk_walk")
    kernel = FUSED_KERNEL
    if two_phase:
        # the solve kernel does S4-S6 and the in-chunk part of S1; the state pass before it does S2 and S3
        tflops_solve = n_chunks * (f_s4 + f_s5 + f_s6) / (ms_solve_launch * 1e-3) / 1e12
        phase_names = ("chunk_states", "chunk_solve")
        kernel = TWO_PHASE_SOLVE_KERNEL

    result = {
        "metric": "GKA layer forward tokens/sec + % bf16 MFMA peak (H=16,d=128,T=4096)",
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "T": w.T, "d": w.d, "chunk": w.chunk,
                   "n_iter": w.n_iter, "input_sets_rotated": N_INPUT_SETS, "clock_ramp_steps": CLOCK_RAMP_STEPS},
        "head_tokens_per_s": tokens * w.H / (ms_per_step * 1e-3),
        "tflops_algorithmic": tflops_total,
        "frac_bf16_mfma_peak": tflops_total / MFMA_BF16_PEAK_TFLOPS,
        "phase_ms": {phase_names[0]: ms_states, phase_names[1]: ms_solve,
                     phase_names[1] + "_launches_per_step": n_launches,
                     phase_names[1] + "_ms_per_launch": ms_solve_launch},
        "roofline": {"kernel": kernel, "bound": "mfma",
                     "achieved": tflops_solve, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops_solve / MFMA_BF16_PEAK_TFLOPS, "traffic": committed_traffic(kernel)},
    }
    if two_phase:
        result["config"]["path"] = "two-phase kernels (profiling aid; not the library's choice for this workload)"

    # ---- the other forward configurations (extra information): long context and the ill-conditioned stress
    if not args.no_other_configs:
        other = {}
        # (configuration 4 needs more than single bf16 operands: see tests/test_gpu_configs.py)
        for wo, compute, label in ((synth.CFG3, binding.GKA_COMPUTE_BF16, "bf16 operands"),
                                   (synth.CFG4, binding.GKA_COMPUTE_BF16_SPLIT, "bf16 value + remainder operands"),
                                   (synth.CFG4, binding.GKA_COMPUTE_F32, "fp32 operands")):
            xo = upload_inputs(synth.make_inputs(wo), wo.dtype)
            po = binding.make_params(wo.B, wo.H, wo.T, wo.d, wo.n_iter, binding.GKA_BF16, compute)
            wso = torch.empty(binding.forward_workspace_bytes(po), dtype=torch.uint8, device="cuda")
            oo = torch.empty_like(xo["v"])
            call = lambda: binding.gka_forward(xo["q"], xo["k"], xo["v"], xo["gate"], xo["lam"], wo.n_iter,
                                               compute=compute, workspace=wso, out=oo)
            for _ in range(10):
                call()
            torch.cuda.synchronize()
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record()
            for _ in range(20):
                call()
            c1.record()
            torch.cuda.synchronize()
            ms = c0.elapsed_time(c1) / 20
            other[f"{wo.name} ({label})"] = {"ms_per_step": ms, "tokens_per_s": wo.B * wo.T / (ms * 1e-3)}
            del xo, wso, oo
        result["other_configs"] = other

    # ---- recurrent decode, configuration 5: 256 sequences x 32 heads, d = 128, states prefilled from 2048 tokens by
    # gka_forward, then 1024 single-token steps timed end to end (no host synchronisation inside). HBM bound: 256 KiB
    # of fp32 state read + written per (sequence, head) per step. Extra information, not the headline metric. The
    # tokens are drawn on the device (same distributions as configuration 2; the parity tests use the host generator).
    if not args.no_decode:
        w5 = synth.CFG5
        dB, dH, dd, d_steps = w5.B, w5.H, w5.d, synth.CFG5_DECODE_STEPS
        gen = torch.Generator(device="cuda").manual_seed(5)

        def draw(*lead):
            qq = torch.nn.functional.normalize(torch.randn((*lead, dH, dd), device="cuda", generator=gen), dim=-1).bfloat16()
            kk = torch.nn.functional.normalize(torch.randn((*lead, dH, dd), device="cuda", generator=gen), dim=-1).bfloat16()
            vv = torch.randn((*lead, dH, dd), device="cuda", generator=gen).bfloat16()
            gg = torch.sigmoid(torch.randn((*lead, dH), device="cuda", generator=gen) + w5.gate_mean)
            ll = torch.nn.functional.softplus(torch.randn((*lead, dH), device="cuda", generator=gen)) + w5.lambda_add
            return qq, kk, vv, gg, ll

        qp, kp, vp, gp, lp = draw(dB, w5.T)
        op, exs = binding.gka_forward(qp, kp, vp, gp, lp, w5.n_iter, return_state=True)
        torch.cuda.synchronize()
        t0 = time.time()
        binding.gka_forward(qp, kp, vp, gp, lp, w5.n_iter, out=op)
        torch.cuda.synchronize()
        ms_prefill = (time.time() - t0) * 1e3
        Hs, Us = exs["H_final"], exs["U_final"]
        del qp, kp, vp, gp, lp, op
        qs, ks, vs, gs, ls = draw(d_steps, dB)
        od = torch.empty((dB, dH, dd), dtype=torch.bfloat16, device="cuda")
        qd, kd, vd, gd, ld = qs[0], ks[0], vs[0], gs[0], ls[0]
        for i in range(5):
            binding.gka_decode_step(Hs, Us, qs[i], ks[i], vs[i], gs[i], ls[i], w5.n_iter, out=od)
        torch.cuda.synchronize()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for i in range(d_steps):
            binding.gka_decode_step(Hs, Us, qs[i], ks[i], vs[i], gs[i], ls[i], w5.n_iter, out=od)
        d1.record()
        torch.cuda.synchronize()
        ms_decode = d0.elapsed_time(d1) / d_steps
        state_bytes = dB * dH * 2 * dd * dd * 4 * 2          # H and U, read and written
        dk = "decode_step_kernel<IOBF16,128,false,false,true>"
        result["decode"] = {"workload": f"{w5.name}: {dB} seq x {dH} heads, d={dd}, n_iter={w5.n_iter}, states prefilled "
                                        f"from {w5.T} tokens by gka_forward ({ms_prefill:.1f} ms), {d_steps} steps",
                            "ms_per_step": ms_decode, "sequence_tokens_per_s": dB / (ms_decode * 1e-3),
                            "prefill_ms": ms_prefill, "prefill_tokens_per_s": dB * w5.T / (ms_prefill * 1e-3),
                            "roofline": {"kernel": dk, "bound": "hbm",
                                         "achieved": state_bytes / (ms_decode * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                                         "unit": "GB/s", "frac": state_bytes / (ms_decode * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                         "traffic": committed_traffic(dk)}}
        d_steps = 50
        # the decode cache in the reduced layout of H (only the 32 x 32 blocks on and below the block diagonal are
        # read and written: 10 of 16 blocks at d = 128)
        for _ in range(5):
            binding.gka_decode_step(Hs, Us, qd, kd, vd, gd, ld, 10, out=od,
                                    state_layout=binding.GKA_STATE_H_LOWER_BLOCKS)
        torch.cuda.synchronize()
        d0.record()
        for _ in range(d_steps):
            binding.gka_decode_step(Hs, Us, qd, kd, vd, gd, ld, 10, out=od,
                                    state_layout=binding.GKA_STATE_H_LOWER_BLOCKS)
        d1.record()
        torch.cuda.synchronize()
        ms_lower = d0.elapsed_time(d1) / d_steps
        lower_bytes = dB * dH * (dd * dd + 10 * 32 * 32) * 4 * 2
        result["decode"]["h_lower_blocks"] = {
            "ms_per_step": ms_lower, "sequence_tokens_per_s": dB / (ms_lower * 1e-3),
            "roofline": {"kernel": "decode_step_kernel<IOBF16,128,false,true,true>", "bound": "hbm",
                         "achieved": lower_bytes / (ms_lower * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": lower_bytes / (ms_lower * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": committed_traffic("decode_step_kernel<IOBF16,128,false,true,true>")}}
        # several tokens per call (gka_decode_tokens): the states still cross HBM once per call
        multi = {}
        for nt in (4, 8):
            qm = torch.nn.functional.normalize(torch.randn((dB, nt, dH, dd), device="cuda", generator=gen),
                                               dim=-1).bfloat16()
            km = torch.nn.functional.normalize(torch.randn((dB, nt, dH, dd), device="cuda", generator=gen),
                                               dim=-1).bfloat16()
            vm = torch.randn((dB, nt, dH, dd), device="cuda", generator=gen).bfloat16()
            gm = torch.sigmoid(torch.randn((dB, nt, dH), device="cuda", generator=gen) + 3.0)
            lm = torch.nn.functional.softplus(torch.randn((dB, nt, dH), device="cuda", generator=gen)) + 1e-2
            om = torch.empty_like(vm)
            for _ in range(3):
                binding.gka_decode_tokens(Hs, Us, qm, km, vm, gm, lm, 10, out=om)
            torch.cuda.synchronize()
            d0.record()
            for _ in range(20):
                binding.gka_decode_tokens(Hs, Us, qm, km, vm, gm, lm, 10, out=om)
            d1.record()
            torch.cuda.synchronize()
            ms = d0.elapsed_time(d1) / 20
            multi[f"tokens_per_call_{nt}"] = {"ms_per_call": ms, "sequence_tokens_per_s": dB * nt / (ms * 1e-3)}
        result["decode"]["multi_token"] = multi

    # ---- backward pass on the same workload (extra information, not the headline metric): a composition of forward
    # kernels, see the header of gka_backward
    if not args.no_backward:
        xs = sets[0]
        dyb = torch.randn_like(xs["v"])
        bparams = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_BF16)
        bws = torch.empty(binding.backward_workspace_bytes(bparams), dtype=torch.uint8, device="cuda")

        def time_backward(lam, lambda_scale):
            call = lambda: binding.gka_backward(xs["q"], xs["k"], xs["v"], xs["gate"], lam, dyb, w.n_iter,
                                                lambda_scale=lambda_scale, workspace=bws)
            for _ in range(3):
                call()
            torch.cuda.synchronize()
            b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            b0.record()
            for _ in range(10):
                call()
            b1.record()
            torch.cuda.synchronize()
            return b0.elapsed_time(b1) / 10

        ms_bwd = time_backward(xs["lam"], 0.0)
        ms_rule = time_backward(None, 0.02)                 # lambda_t = 0.02 ||H_t||_F (Section 4.1)
        result["backward"] = {"ms_per_call": ms_bwd, "tokens_per_s": tokens / (ms_bwd * 1e-3),
                              "times_forward": ms_bwd / ms_per_step, "workspace_bytes": bws.numel(),
                              "frobenius_rule_ms_per_call": ms_rule}
        del bws, dyb

    # ---- latent sketching on the same workload (extra information): sketch dimension 32, one Gaussian sketch per head
    if not args.no_sketch:
        xs = sets[0]
        d_s = 32
        gen = torch.Generator(device="cuda").manual_seed(7)
        S = torch.randn((w.H, d_s, w.d), generator=gen, device="cuda", dtype=torch.float32) / w.d ** 0.5
        sparams = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_BF16)
        sws = torch.empty(binding.forward_sketched_workspace_bytes(sparams, d_s), dtype=torch.uint8, device="cuda")
        so = torch.empty_like(xs["v"])
        call = lambda: binding.gka_forward_sketched(xs["q"], xs["k"], xs["v"], xs["gate"], xs["lam"], S, w.n_iter,
                                                    workspace=sws, out=so)
        for _ in range(20):
            call()
        torch.cuda.synchronize()
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for _ in range(50):
            call()
        s1.record()
        torch.cuda.synchronize()
        ms_sk = s0.elapsed_time(s1) / 50
        result["latent_sketching"] = {"sketch_dim": d_s, "ms_per_step": ms_sk, "tokens_per_s": tokens / (ms_sk * 1e-3),
                                      "times_forward": ms_sk / ms_per_step, "workspace_bytes": sws.numel()}
        del sws, so, S

    # ---- other head dimensions (extra information): the token-by-token path of gka_forward, synthetic inputs of the
    # workload's distributions. d = 16 on the shape of a vision model (Appendix L: 197 tokens, many short sequences);
    # d = 256 at the model width of the headline workload.
    if not args.no_head_dims:
        result["other_head_dims"] = {}
        rec = binding.GKA_PATH_RECURRENT
        for name, shape, path, kernel in (
                ("d16_197_tokens", dict(B=256, H=24, T=197, d=16), binding.GKA_PATH_AUTO, "small_solve_kernel (chunk-wise, d <= 32)"),
                ("d16_197_tokens_recurrent", dict(B=256, H=24, T=197, d=16), rec, "decode_step_kernel_d16 (path recurrent)"),
                ("d256", dict(B=4, H=8, T=1024, d=256), binding.GKA_PATH_AUTO, "decode_step_kernel (path recurrent)")):
            wd = w.scaled(seed=w.seed + 50, **shape)
            xd = upload_inputs(synth.make_inputs(wd), "bf16")
            od = torch.empty_like(xd["v"])
            pd = binding.make_params(wd.B, wd.H, wd.T, wd.d, wd.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_BF16,
                                     path=path)
            wsd = torch.empty(binding.forward_workspace_bytes(pd), dtype=torch.uint8, device="cuda")
            call = lambda: binding.gka_forward(xd["q"], xd["k"], xd["v"], xd["gate"], xd["lam"], wd.n_iter,
                                               workspace=wsd, out=od, path=path)
            call()
            torch.cuda.synchronize()
            d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            d0.record()
            for _ in range(3):
                call()
            d1.record()
            torch.cuda.synchronize()
            ms_d = d0.elapsed_time(d1) / 3
            result["other_head_dims"][name] = {"B": wd.B, "H": wd.H, "T": wd.T, "d": wd.d, "ms_per_step": ms_d,
                                               "tokens_per_s": wd.B * wd.H * wd.T / (ms_d * 1e-3),
                                               "kernel": kernel}
            del xd, od, wsd

    if not args.no_cpu_baseline:
        import oracle
        x = sets_host[0]
        t0 = time.time()
        ref = oracle.forward(x["q"], x["k"], x["v"], x["gate"], x["lam"], w.n_iter)
        dt = time.time() - t0
        result["cpu_baseline"] = {"value": tokens / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"the whole workload once ({w.B * w.H} pairs x {w.T} tokens), {dt:.1f} s"}
        step(0)
        torch.cuda.synchronize()
        result["max_rel_err_vs_oracle"] = pair_rel_err(to_host(outs[0]), ref)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
