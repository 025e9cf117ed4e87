"""Benchmark of the whole hot path on one MI355X.

A step is one complete pass of Algorithm 1 (enumerate, featurize, V(s), argmin, commit
for every layer) over one batch of synthetic scheduling problems.  Default workload:
a batch of ResNet-18-shaped 20-stage pipelines, 4096 candidates per decision, 256
features, MLP 256-512-512-1 in bf16 with fp32 accumulation.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE at batch 256, scaled by a
# plain 1 GiB copy (profiles/*_hbm_counters.txt); only valid for the default batch, and to be
# set to None whenever the kernel changes without the counters being taken again
TRAFFIC_SCORE_BYTES = {256: 8827.5 * 1024 * 2.0 + 50885.0 * 1024}
TRAFFIC_FEATURIZE_BYTES = {256: 945.0 * 1024 * 2.0 + 1073741824.0}


def mlp_flops(dims):
    return 2 * sum(dims[k] * dims[k + 1] for k in range(len(dims) - 1))


def fused_mlp_flops(dims):
    """Flops per candidate the fused step executes on the matrix cores: of the 256 input
    rows only the 64 core rows differ between the candidates of a decision; the first
    layer's product with the other 192 is computed once per decision (a bias)."""
    d = list(dims)
    if d[0] == 256:
        d[0] = 64
    return mlp_flops(d)


def cpu_baseline(I, pipe, space, model, w, dims):
    """The CPU checker, as it stands, on one pipeline of the batch (bounded sample)."""
    from oracle import ovf
    S = len(pipe)
    M = ovf.dense_count(space)
    t0 = time.perf_counter()
    r = ovf.greedy(pipe, space, model, w)
    dt = time.perf_counter() - t0
    return {"value": r["n_evals"] / dt, "unit": "candidates/s", "cores": ovf.num_threads(), "kind": "oracle",
            "candidate_ids_per_s": S * M / dt,
            "sample": f"one pipeline of the batch (problem 0: {S} decisions x {M} candidate ids, of which "
                      f"{r['n_evals']} are valid candidates; features and V(s) for every id, argmin over the "
                      f"valid ones), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=256, help="independent pipelines per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="skip the single-pipeline latency measurement")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy a few times (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2011_14486_amd as pkg
    from paper_2011_14486_amd import inputs as I
    vf = pkg.load()

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
    roofline = {"bound": "mfma", "kernel": "k_whole<128,2,4> (Algorithm 1 per problem in one workgroup: enumerate+featurize+MLP+argmin+commit)", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_SCORE_BYTES.get(B),
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
                     "unit": "GB/s", "frac": feat_gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_FEATURIZE_BYTES.get(B),
                     "launch_ms": feat_ms, "launches": n_featk,
                     "note": "vf_featurize alone, 10 launches after the timed region"}

    # latency of one pipeline alone (the single-network case of Algorithm 1)
    single_ms = None
    if not args.no_latency:
        ctx1 = vf.vf_create(0)
        vf.vf_set_space(ctx1, space); vf.vf_set_pipeline(ctx1, pipes[0]); vf.vf_set_model(ctx1, model, w)
        for _ in range(3):
            vf.vf_reset_state(ctx1); vf.vf_greedy_schedule(ctx1)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        reps = 10
        for _ in range(reps):
            vf.vf_reset_state(ctx1); vf.vf_greedy_schedule(ctx1)
        torch.cuda.synchronize()
        single_ms = (time.perf_counter() - t1) / reps * 1e3
        vf.vf_destroy(ctx1)

    # end-to-end greedy schedule of the 100-stage MobileNet-V2-shaped pipeline, 16384
    # candidates per decision, same value network (latency of a single large problem)
    mb_ms = None
    if not args.no_latency:
        ctx5 = vf.vf_create(0)
        vf.vf_set_space(ctx5, I.mobilenetv2_space()); vf.vf_set_pipeline(ctx5, I.mobilenetv2_shaped())
        vf.vf_set_model(ctx5, model, w)
        for _ in range(2):
            vf.vf_reset_state(ctx5); vf.vf_greedy_schedule(ctx5)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(5):
            vf.vf_reset_state(ctx5); vf.vf_greedy_schedule(ctx5)
        torch.cuda.synchronize()
        mb_ms = (time.perf_counter() - t1) / 5 * 1e3
        vf.vf_destroy(ctx5)

    # Algorithm 2's use of the scan: 100 noisy rollouts of one network (Sec. 3.1), here the
    # 100-stage pipeline: a batch of 100 copies with different noise
    rollouts = None
    if not args.no_latency:
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
        for _ in range(3):
            vf.vf_reset_state(ctxr); vf.vf_greedy_schedule(ctxr)
        torch.cuda.synchronize()
        dtr = (time.perf_counter() - t1) / 3
        _, valid_r = vf.vf_profile_counts(ctxr)
        vf.vf_profile_enable(ctxr, False)
        for k in (0, 1, 2):
            vf.vf_profile_read(ctxr, k)
        rollouts = {"workload": "100 noisy rollouts (eps 0.3) of the MobileNet-V2-shaped pipeline, 100 stages, "
                                "16384 candidate ids per decision", "ms_per_batch": dtr * 1e3,
                    "valid_candidates_per_s": valid_r / 3 / dtr}
        vf.vf_destroy(ctxr)

    # the paper's own kind of V (Sec. 3.2): LSTM 64 -> 256 over one timestep per stage, head
    # summed, guiding the same greedy scan on a smaller batch of the same pipelines
    lstm = None
    if not args.no_latency:
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
        "candidate_ids_per_s": ids_per_step * args.steps / dt,
        "greedy_ms_single_pipeline": single_ms,
        "greedy_ms_mobilenetv2_100_stages_16384_candidates": mb_ms,
        "noisy_rollouts_100": rollouts,
        "greedy_with_recurrent_network": lstm,
        "kernel_ms_per_step": {"featurize": ms_feat / args.steps, "score": ms_score / args.steps,
                               "commit": ms_commit / args.steps},
        "roofline": roofline,
        "roofline_featurize": roofline_feat,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(I, pipes[0], space, model, w, dims)
    vf.vf_destroy(ctx)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
