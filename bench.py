"""Benchmark of the whole hot path on one MI355X.

A step is one complete pass of Algorithm 1 (enumerate, featurize, V(s), argmin, commit
for every layer) over one batch of synthetic scheduling problems.  Default workload:
a batch of ResNet-18-shaped 20-stage pipelines, 4096 candidate ids per decision, 256
features, MLP 256-512-512-1 in bf16 with fp32 accumulation.  Prints ONE JSON line.

Next to the headline the line carries, under "workloads", the other four synthetic
configurations (tiny conv+ReLU greedy in fp32, raw scoring of 1,048,576 vectors through
MLP 256-1024-1024-1024-1, the recurrent V(s) on 16,384 sequences of 50 steps, the greedy
schedule of the 100-stage MobileNet-V2-shaped pipeline), each timed with HIP events
outside the headline's timed region and with the CPU checker's rate on a bounded sample
(all cores and one thread).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
HBM_PROFILE = os.path.join(ROOT, "profiles", "k_whole_and_k_featurize_resnet18_batch256_hbm_counters.txt")


def kernel_sources_sha256():
    """Hash of the HIP sources: HBM counters taken for other sources say nothing about these."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2011_14486_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def measured_traffic(kernel, batch):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary (FETCH_SIZE
    and WRITE_SIZE runs, scaled by a plain copy) - or None when the summary was taken for other
    kernel sources or another batch than the ones being timed."""
    try:
        text = open(HBM_PROFILE).read()
    except OSError:
        return None
    m = re.search(r"^# csrc_sha256: (\w+)", text, re.M)
    b = re.search(r"^# batch: (\d+)", text, re.M)
    t = re.search(rf"^# traffic_bytes_per_launch {re.escape(kernel)}: (\d+)", text, re.M)
    if not (m and b and t) or m.group(1) != kernel_sources_sha256() or int(b.group(1)) != batch:
        return None
    return int(t.group(1))


def mlp_flops(dims):
    return 2 * sum(dims[k] * dims[k + 1] for k in range(len(dims) - 1))


def fused_mlp_flops(dims):
    """Flops per candidate the fused step executes on the matrix cores: of the input rows only
    16..55 and 59 differ between the candidates of a decision; the first layer's product with
    all the others is computed once per decision (a bias), and the candidates' contraction runs
    over rows 16..63: three k-steps of 16."""
    d = list(dims)
    if d[0] in (64, 256):
        d[0] = 48
    return mlp_flops(d)


def timed_cpu(fn, threads_all):
    """fn() -> units of work; timed with all threads, then (fn(single=True)) with one."""
    from oracle import ovf
    out = {}
    for label, nthr in (("all_cores", threads_all), ("single_thread", 1)):
        ovf.set_num_threads(nthr)
        t0 = time.perf_counter()
        units, what = fn(label == "single_thread")
        dt = time.perf_counter() - t0
        out[label] = {"value": units / dt, "cores": nthr, "seconds": dt, "sample": what}
    ovf.set_num_threads(threads_all)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=250)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--batch", type=int, default=256, help="independent pipelines per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="headline workload only")
    ap.add_argument("--only", default="", help="comma-separated subset of the other workloads: "
                    "c1,c3,c4,c5,rollouts,lstm_search,single")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy a few times (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    only = set(filter(None, args.only.split(",")))

    def wanted(name):
        return not args.no_latency and (not only or name in only)

    import numpy as np
    import torch
    import paper_2011_14486_amd as pkg
    from paper_2011_14486_amd import inputs as I
    vf = pkg.load()
    cpu = not args.no_cpu_baseline
    if cpu:
        from oracle import ovf
        ncores = ovf.num_threads()

    B = args.batch
    dims = [256, 512, 512, 1]
    pipes = I.resnet18_batch(B, seed=2)
    space = I.resnet18_space()
    S, M = pipes.shape[1], I.space_dense_count(space)
    w = I.mlp_weights(dims, 0)
    model = I.model_record(I.MLP, dims, I.BF16)

    ctx = vf.vf_create(0)
    vf.vf_set_space(ctx, space)
    vf.vf_set_pipeline(ctx, pipes)
    vf.vf_set_model(ctx, model, w)
    out = (ctx.empty((B, S, 16), torch.int32), ctx.empty((B, S), torch.int32), ctx.empty((B, S), torch.float32))

    def step():
        vf.vf_reset_state(ctx)
        vf.vf_greedy_schedule(ctx, 0, S - 1, out=out)

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    vf.vf_profile_enable(ctx, True)
    for k in (0, 1, 2):
        vf.vf_profile_read(ctx, k)
    vf.vf_profile_counts(ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    vf.vf_profile_enable(ctx, False)
    ms_feat, n_feat = vf.vf_profile_read(ctx, vf.VF_PROF_FEATURIZE)
    ms_score, n_score = vf.vf_profile_read(ctx, vf.VF_PROF_SCORE)
    ms_commit, n_commit = vf.vf_profile_read(ctx, vf.VF_PROF_COMMIT)
    vf.vf_sync_status(ctx)     # raises if a whole-schedule launch gave up a wait between workgroups
    cids = out[1].cpu().numpy()
    assert (cids >= 0).all(), "a schedule ended early"

    # Algorithm 1 evaluates V on the candidates of each layer: `value` counts the valid
    # candidates.  The dense id space is larger (ids whose digits break a validity rule);
    # runs of ids closed by the compute_at / store_at digits alone never reach the
    # network, the other invalid ids share a tile with valid ones and do.
    scored, valid = vf.vf_profile_counts(ctx)
    ids_per_step = B * S * M
    valid_per_step = valid / args.steps
    scored_per_step = scored / args.steps
    value = valid / dt

    # dominant kernel: the fused MLP scorer (dense contraction -> MFMA roofline); the
    # flops are those of the ids that went through the network
    flops_per_launch = fused_mlp_flops(dims) * scored / max(n_score, 1)
    score_ms = ms_score / max(n_score, 1)
    achieved = flops_per_launch / (score_ms * 1e-3) / 1e12
    traffic = measured_traffic("k_whole", B)
    roofline = {"bound": "mfma", "kernel": "k_whole<128,2,4> (Algorithm 1 per problem in one workgroup: enumerate+featurize+MLP+argmin+commit)", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                "traffic_source": os.path.relpath(HBM_PROFILE, ROOT) if traffic is not None else
                "none: the committed counter summary was taken for other kernel sources or another batch",
                "flops_per_candidate_executed": fused_mlp_flops(dims), "flops_per_candidate_model": mlp_flops(dims),
                "launch_ms": score_ms, "launches": n_score}
    # the materialising featurizer (vf_featurize) on the same batch: in the step above the
    # features are produced inside the scoring kernel and never written to HBM, so the
    # HBM-bound kernel is timed on its own, at the state the schedules ended in
    feat_buf = ctx.empty((B, 256, vf.vf_padded_count(ctx)), torch.int32)
    for _ in range(2):
        vf.vf_featurize(ctx, S - 1, out=feat_buf)
    torch.cuda.synchronize()
    vf.vf_profile_enable(ctx, True)
    for j in range(10):
        vf.vf_featurize(ctx, S - 1 - (j % 4), out=feat_buf)
    vf.vf_profile_enable(ctx, False)
    ms_featk, n_featk = vf.vf_profile_read(ctx, vf.VF_PROF_FEATURIZE)
    del feat_buf
    feat_bytes = 4 * 256 * B * M
    feat_ms = ms_featk / max(n_featk, 1)
    feat_gbs = feat_bytes / (feat_ms * 1e-3) / 1e9
    roofline_feat = {"bound": "hbm", "kernel": "k_featurize", "achieved": feat_gbs, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": feat_gbs / PEAK_HBM_GBS, "traffic": measured_traffic("k_featurize", B),
                     "launch_ms": feat_ms, "launches": n_featk,
                     "note": "vf_featurize alone, 10 launches after the timed region"}

    def greedy_ms(sp, pp, mdl, wts, reps, warm=3):
        """Wall time per vf_greedy_schedule of one context (reset included), milliseconds."""
        c = vf.vf_create(0)
        vf.vf_set_space(c, sp); vf.vf_set_pipeline(c, pp); vf.vf_set_model(c, mdl, wts)
        for _ in range(warm):
            vf.vf_reset_state(c); vf.vf_greedy_schedule(c)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(reps):
            vf.vf_reset_state(c); vf.vf_greedy_schedule(c)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t1) / reps * 1e3
        vf.vf_profile_enable(c, True); vf.vf_profile_counts(c)
        vf.vf_reset_state(c); vf.vf_greedy_schedule(c)
        _, nvalid = vf.vf_profile_counts(c)
        vf.vf_profile_enable(c, False)
        vf.vf_destroy(c)
        return ms, nvalid

    workloads = {}

    # ---- tiny conv3x3 + ReLU, 6000 ids per decision, MLP 64-128-128-1 in fp32, 2 decisions
    if wanted("c1"):
        p1, s1 = I.tiny_conv_relu(), I.tiny_space()
        d1 = [64, 128, 128, 1]
        w1, m1 = I.mlp_weights(d1, 0), I.model_record(I.MLP, d1, I.FP32)
        ms1, _ = greedy_ms(s1, p1, m1, w1, reps=50)
        ref1 = None
        e = {"workload": "conv3x3 (8->8 ch, 16x16) + ReLU, 6000 candidate ids per decision, F=64, MLP 64-128-128-1 fp32, "
                         "2 decisions", "dtype": "f32", "greedy_ms": ms1, "flops_per_candidate": mlp_flops(d1)}
        if cpu:
            def f1(single):
                r = ovf.greedy(p1, s1, m1, w1)
                return r["n_evals"], "the whole workload (2 decisions)"
            e["cpu_oracle"] = dict(timed_cpu(f1, ncores), unit="candidates/s")
            ref1 = ovf.greedy(p1, s1, m1, w1)
            e["valid_candidates"] = ref1["n_evals"]
            e["candidates_per_s"] = ref1["n_evals"] / (ms1 * 1e-3)
        workloads["tiny_conv_relu_fp32"] = e

    # ---- single pipelines: the latency half of the metric (one launch per layer)
    if wanted("single"):
        ms2, nv2 = greedy_ms(space, pipes[0], model, w, reps=20)
        workloads["resnet18_single_pipeline"] = {
            "workload": f"one ResNet-18-shaped pipeline, {S} stages, {M} candidate ids per decision, MLP 256-512-512-1 bf16",
            "greedy_ms": ms2, "valid_candidates": nv2, "candidates_per_s": nv2 / (ms2 * 1e-3)}
    if wanted("c5"):
        p5, s5 = I.mobilenetv2_shaped(), I.mobilenetv2_space()
        ms5, nv5 = greedy_ms(s5, p5, model, w, reps=10)
        e = {"workload": "one MobileNet-V2-shaped pipeline, 100 stages, 16384 candidate ids per decision, MLP 256-512-512-1 bf16",
             "greedy_ms": ms5, "valid_candidates": nv5, "candidates_per_s": nv5 / (ms5 * 1e-3),
             "mfma_frac": nv5 * fused_mlp_flops(dims) / (ms5 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        if cpu:
            def f5(single):
                last = 0 if single else 3
                r = ovf.greedy(p5, s5, model, w, last=last)
                return r["n_evals"], f"decisions 0..{last} of the 100 (16384 ids each: features and V(s) for every id)"
            e["cpu_oracle"] = dict(timed_cpu(f5, ncores), unit="candidates/s")
        workloads["mobilenetv2_100_stages"] = e

    # ---- raw scoring: 1,048,576 feature vectors, MLP 256-1024-1024-1024-1 bf16, argmin per 4096
    if wanted("c3"):
        d3 = [256, 1024, 1024, 1024, 1]
        G, group = 256, 4096
        w3, m3 = I.mlp_weights(d3, 0), I.model_record(I.MLP, d3, I.BF16)
        x3 = torch.from_numpy(I.raw_feature_matrix(G, 256, group, seed=3)).cuda()
        c3 = vf.vf_create(0)
        vf.vf_set_model(c3, m3, w3)
        for _ in range(5):
            vf.vf_score(c3, x3, vf.VF_X_RAW_I32, group=group, want_scores=False)
        torch.cuda.synchronize()
        vf.vf_profile_enable(c3, True); vf.vf_profile_read(c3, vf.VF_PROF_SCORE)
        t1 = time.perf_counter()
        for _ in range(50):
            vf.vf_score(c3, x3, vf.VF_X_RAW_I32, group=group, want_scores=False)
        torch.cuda.synchronize()
        wall3 = (time.perf_counter() - t1) / 50 * 1e3
        ms3, n3 = vf.vf_profile_read(c3, vf.VF_PROF_SCORE)
        vf.vf_profile_enable(c3, False)
        vf.vf_destroy(c3)
        del x3
        k3 = ms3 / max(n3, 1)
        tf3 = G * group * mlp_flops(d3) / (k3 * 1e-3) / 1e12
        e = {"workload": "1,048,576 raw feature vectors (F=256, values floor(2^u), u~U[0,20)), MLP 256-1024-1024-1024-1 "
                         "bf16, fused argmin per group of 4096; inputs resident in HBM (1 GiB int32)",
             "kernel_ms": k3, "launches": n3, "wall_ms_per_call": wall3, "candidates_per_s": G * group / (k3 * 1e-3),
             "flops_per_candidate": mlp_flops(d3),
             "roofline": {"bound": "mfma", "achieved": tf3, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                          "frac": tf3 / PEAK_BF16_TFLOPS},
             "hbm_read_gbs": 4 * 256 * G * group / (k3 * 1e-3) / 1e9}
        # the other design for this width, as a ceiling: one library GEMM per layer (the three
        # contractions alone, bf16 in and out, with nothing of what the fused kernel also does:
        # quantisation, bias, ReLU, output dot, argmin)
        def library_gemm_ms(K):
            a = torch.randn(G * group, K, device="cuda", dtype=torch.bfloat16)
            wt = torch.randn(1024, K, device="cuda", dtype=torch.bfloat16) * 0.03
            out = torch.empty(G * group, 1024, device="cuda", dtype=torch.bfloat16)
            for _ in range(3):
                torch.matmul(a, wt.t(), out=out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                torch.matmul(a, wt.t(), out=out)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / 10
        g256, g1024 = library_gemm_ms(256), library_gemm_ms(1024)
        gsum = g256 + 2 * g1024
        e["per_layer_library_gemm"] = {
            "what": "torch.matmul (the vendor GEMM library) on [1048576, K] x [K, 1024] bf16: the first layer's "
                    "contraction (K = 256) and the two hidden ones (K = 1024), contractions only",
            "ms_k256": g256, "ms_k1024": g1024, "ms_three_contractions": gsum,
            "frac_of_peak": G * group * 2.0 * (256 * 1024 + 2 * 1024 * 1024) / (gsum * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "fused_kernel_ms": k3}
        if cpu:
            def f3(single):
                n = 256 if single else 4096
                blk = I.raw_feature_group(0, 256, group, seed=3)[:, :n].copy()
                ovf.score_mlp(m3, w3, blk)
                return n, f"the first {n} vectors of group 0"
            e["cpu_oracle"] = dict(timed_cpu(f3, ncores), unit="candidates/s")
        workloads["raw_scoring_1M"] = e

    # ---- recurrent V(s) of Sec. 3.2: 16,384 sequences, T = 50, LSTM 128 -> 256, head summed
    if wanted("c4"):
        F4, H4, T4, B4 = 128, 256, 50, 16384
        w4, m4 = I.lstm_weights(F4, H4, seed=0), I.model_record(I.LSTM, [F4, H4, 1], I.BF16)
        xb = I.feature_sequences(0, B4, T=T4, F=F4, seed=4)
        x4 = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        c4 = vf.vf_create(0)
        vf.vf_set_model(c4, m4, w4)
        for _ in range(5):
            vf.vf_score(c4, x4, vf.VF_X_SEQ_BF16, want_scores=False)
        torch.cuda.synchronize()
        vf.vf_profile_enable(c4, True); vf.vf_profile_read(c4, vf.VF_PROF_SCORE)
        t1 = time.perf_counter()
        for _ in range(100):
            vf.vf_score(c4, x4, vf.VF_X_SEQ_BF16, want_scores=False)
        torch.cuda.synchronize()
        wall4 = (time.perf_counter() - t1) / 100 * 1e3
        ms4, n4 = vf.vf_profile_read(c4, vf.VF_PROF_SCORE)
        vf.vf_profile_enable(c4, False)
        vf.vf_destroy(c4)
        del x4
        k4 = ms4 / max(n4, 1)
        fl4 = T4 * (2 * 4 * H4 * (F4 + H4) + 2 * H4)
        tf4 = B4 * fl4 / (k4 * 1e-3) / 1e12
        e = {"workload": "16,384 feature sequences [50][128] bf16, LSTM 128->256 + linear 256->1 summed over the 50 "
                         "steps, bf16 weights, fp32 gates and cell; inputs resident in HBM (210 MB)",
             "kernel_ms": k4, "launches": n4, "wall_ms_per_call": wall4, "candidates_per_s": B4 / (k4 * 1e-3),
             "flops_per_candidate": fl4,
             "roofline": {"bound": "mfma", "achieved": tf4, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                          "frac": tf4 / PEAK_BF16_TFLOPS}}
        if cpu:
            def f4(single):
                n = 32 if single else 512
                ovf.score_lstm(m4, w4, xb[:n])
                return n, f"the first {n} sequences"
            e["cpu_oracle"] = dict(timed_cpu(f4, ncores), unit="candidates/s")
        workloads["lstm_16384x50"] = e

    # Algorithm 2's use of the scan: 100 noisy rollouts of one network (Sec. 3.1), here the
    # 100-stage pipeline: a batch of 100 copies with different noise
    rollouts = None
    if wanted("rollouts"):
        ctxr = vf.vf_create(0)
        vf.vf_set_space(ctxr, I.mobilenetv2_space())
        vf.vf_set_pipeline(ctxr, np.repeat(I.mobilenetv2_shaped()[None], 100, axis=0))
        vf.vf_set_model(ctxr, model, w)
        vf.vf_set_noise(ctxr, 0.3, 7)
        vf.vf_profile_enable(ctxr, True)
        for _ in range(2):
            vf.vf_reset_state(ctxr); vf.vf_greedy_schedule(ctxr)
        torch.cuda.synchronize()
        vf.vf_profile_counts(ctxr)
        t1 = time.perf_counter()
        for _ in range(5):
            vf.vf_reset_state(ctxr); vf.vf_greedy_schedule(ctxr)
        torch.cuda.synchronize()
        dtr = (time.perf_counter() - t1) / 5
        _, valid_r = vf.vf_profile_counts(ctxr)
        vf.vf_profile_enable(ctxr, False)
        for k in (0, 1, 2):
            vf.vf_profile_read(ctxr, k)
        rollouts = {"workload": "100 noisy rollouts (eps 0.3) of the MobileNet-V2-shaped pipeline, 100 stages, "
                                "16384 candidate ids per decision", "ms_per_batch": dtr * 1e3,
                    "valid_candidates_per_s": valid_r / 5 / dtr,
                    "mfma_frac": valid_r / 5 * fused_mlp_flops(dims) / dtr / 1e12 / PEAK_BF16_TFLOPS}
        vf.vf_destroy(ctxr)

    # the paper's own kind of V (Sec. 3.2): LSTM 64 -> 256 over one timestep per stage, head
    # summed, guiding the same greedy scan on a smaller batch of the same pipelines
    lstm = None
    if wanted("lstm_search"):
        Bl, H = min(B, 64), 256
        ctxl = vf.vf_create(0)
        vf.vf_set_space(ctxl, space); vf.vf_set_pipeline(ctxl, pipes[:Bl])
        vf.vf_set_model(ctxl, I.model_record(I.LSTM, [64, H, 1], I.BF16), I.lstm_weights(64, H, 0))
        vf.vf_profile_enable(ctxl, True); vf.vf_profile_counts(ctxl)
        flops_l, valid_l = 0, 0
        for i in range(S):     # per-layer counts: a candidate of layer i costs S - i cell steps
            vf.vf_argmin_step(ctxl, i, True)
            sc_i, va_i = vf.vf_profile_counts(ctxl)
            flops_l += sc_i * (2 * 4 * H * 64 + (S - 1 - i) * 2 * 4 * H * H)
            valid_l += va_i
        vf.vf_profile_enable(ctxl, False)
        for k in (0, 1, 2):
            vf.vf_profile_read(ctxl, k)
        vf.vf_reset_state(ctxl); vf.vf_greedy_schedule(ctxl)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(3):
            vf.vf_reset_state(ctxl); vf.vf_greedy_schedule(ctxl)
        torch.cuda.synchronize()
        dtl = (time.perf_counter() - t1) / 3
        lstm = {"model": f"LSTM 64-{H}-1 bf16 over {S} timesteps", "batch": Bl, "ms_per_step": dtl * 1e3,
                "valid_candidates_per_s": valid_l / dtl, "mfma_tflops": flops_l / dtl / 1e12,
                "mfma_frac": flops_l / dtl / 1e12 / PEAK_BF16_TFLOPS}
        vf.vf_destroy(ctxl)

    line = {
        "metric": "candidate schedules scored/sec (V(s) eval) + end-to-end greedy schedule ms",
        "value": value, "unit": "candidates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-18-shaped pipelines, {S} stages, {M} candidate ids per decision, F=256, "
                               f"MLP 256-512-512-1 bf16 weights/activations with fp32 accumulation; batch of {B} "
                               "independent pipelines per step (problem 0 has the standard shapes, the others "
                               "seeded width/resolution variants)",
                   "batch": B, "stages": S, "candidate_ids_per_decision": M, "candidate_ids_per_step": ids_per_step,
                   "valid_candidates_per_step": valid_per_step, "ids_through_network_per_step": scored_per_step},
        "timed_region_s": dt,
        "candidate_ids_per_s": ids_per_step * args.steps / dt,
        "workloads": workloads,
        "noisy_rollouts_100": rollouts,
        "greedy_with_recurrent_network": lstm,
        "kernel_ms_per_step": {"featurize": ms_feat / args.steps, "score": ms_score / args.steps,
                               "commit": ms_commit / args.steps},
        "roofline": roofline,
        "roofline_featurize": roofline_feat,
    }
    if cpu:
        def f2(single):
            last = 1 if single else S - 1
            r = ovf.greedy(pipes[0], space, model, w, last=last)
            return r["n_evals"], (f"problem 0 of the batch, decisions 0..{last} ({M} candidate ids each: features and "
                                  "V(s) for every id, argmin over the valid ones)")
        both = timed_cpu(f2, ncores)
        line["cpu_baseline"] = {"value": both["all_cores"]["value"], "unit": "candidates/s", "cores": ncores,
                                "kind": "oracle", "sample": f"{both['all_cores']['sample']}, {both['all_cores']['seconds']:.1f} s",
                                "single_thread": both["single_thread"]}
    vf.vf_destroy(ctx)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
