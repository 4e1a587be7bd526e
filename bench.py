#!/usr/bin/env python3
"""Benchmark of the GRPO scoring hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic batch already
resident in HBM: group advantages, then the fused LM-head + log-softmax + GRPO
loss forward and backward (dH, dW).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--full-length]
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

METRIC = "scored tokens/sec, fused LM-head+logsoftmax+GRPO fwd+bwd; % bf16 MFMA peak"
MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(batch, sp, rows_T=256):
    """Times the CPU oracle (as it stands) on a bounded sample of the same workload: the first
    prompt's rollouts truncated to their first `rows_T` tokens, at full V and d, once with all the
    threads NumPy's BLAS takes on this host and once confined to a single thread (on the first
    eighth of those tokens: the oracle's cost is linear in the rows)."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info, threadpool_limits

    from oracle import mrl_oracle as orc
    from tests import util

    T = batch["T"]
    k = sp.k_own + sp.k_peer
    W = util.to_f64(batch["W"])
    rewards = util.to_f64(batch["rewards_all"][:k])
    gid = np.zeros(k, dtype=np.int64)
    cfg = util.cfg_dict(sp)

    def timed(t_sub):
        rows = (np.arange(k)[:, None] * T + np.arange(t_sub)[None, :]).reshape(-1)
        ridx = torch.tensor(rows, device=batch["H"].device)
        H = util.to_f64(batch["H"][ridx])
        y = batch["targets"][ridx].cpu().numpy()
        mask = batch["mask"].reshape(-1)[ridx].cpu().numpy().reshape(k, t_sub)
        behav, ref = util.to_f64(batch["behav"][ridx]), util.to_f64(batch["ref"][ridx])
        t0 = time.perf_counter()
        adv, *_ = orc.group_advantages(rewards, gid, 1)
        out = orc.grpo_loss_fwd_bwd(H, W, y, mask, behav, ref, adv, gid, None, k, t_sub, 1, cfg)
        dt = time.perf_counter() - t0
        assert np.isfinite(out["loss_total"])
        return int(mask.sum()), dt

    t_all = min(rows_T, T)
    n_tok, dt = timed(t_all)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    t_one = max(1, t_all // 8)
    with threadpool_limits(limits=1):
        n_tok1, dt1 = timed(t_one)
    return dict(value=n_tok / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"{k} sequences x first {t_all} tokens ({n_tok} scored rows) at full V={sp.V}, d={sp.d}; "
                       f"fp64 NumPy, {dt:.1f} s",
                single_thread=dict(value=n_tok1 / dt1, unit="tokens/s", cores=1,
                                   sample=f"{k} sequences x first {t_one} tokens ({n_tok1} scored rows), {dt1:.1f} s"),
                host_cpus=os.cpu_count())


def thl_alignment_leg(mrl, synth, torch, with_cpu, B=2048, S_src=1180, S_tgt=1536, reps=20):
    """The word-level trace alignment of the pooled peer rollouts (a pass of its own, before the
    scoring step, not part of `value`): achieved GB/s on algorithmic bytes, oracle on a sample."""
    b = synth.make_thl(B, S_src, S_tgt)
    call = lambda: mrl.thl_word_align(b["src_logp"], b["src_mask"], b["src_word_map"], b["src_map_len"],
                                      b["tgt_mask"], b["tgt_word_map"], b["tgt_map_len"], b["max_words"],
                                      want_bad_count=False)
    call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    # log-prob, mask byte and map entry per source position; mask byte, map entry and output per target position
    nbytes = B * (S_src * 9 + S_tgt * 9)
    n_tok = int(b["tgt_mask"].sum().item())
    leg = dict(workload=f"{B} peer rollouts, source grid {S_src}, target grid {S_tgt} (configuration 3 lengths)",
               ms_per_launch=round(ms, 4), algorithmic_MB=round(nbytes / 1e6, 2),
               achieved_GBps=round(nbytes / (ms * 1e-3) / 1e9, 1), peak_GBps=8000.0,
               target_tokens_per_s=round(n_tok / (ms * 1e-3), 1))
    if with_cpu:
        from oracle import thl_oracle
        n = 64
        c = {k: (v[:n].cpu().numpy() if isinstance(v, torch.Tensor) else v) for k, v in b.items()}
        t0 = time.perf_counter()
        thl_oracle.word_align_logprobs(c["src_logp"].astype("float64"), c["src_mask"], c["src_word_map"], c["src_map_len"],
                                       c["tgt_mask"], c["tgt_word_map"], c["tgt_map_len"], -100.0)
        dt = time.perf_counter() - t0
        leg["cpu_oracle"] = dict(target_tokens_per_s=round(int(c["tgt_mask"].sum()) / dt, 1), cores=1,
                                 sample=f"first {n} sequences, pure Python, {dt:.2f} s")
    return leg


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration index (2..5)")
    ap.add_argument("--full-length", action="store_true", help="score every slot (no padding)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-rows", type=int, default=0)
    ap.add_argument("--prompts", type=int, default=0, help="override the number of prompts (debug)")
    ap.add_argument("--hidden", type=int, default=0, help="override the hidden width d (debug)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the legs that are not part of `value` (alignment pass, forward-only scoring pass); "
                         "used for kernel profiles so that only the step's launches are in the trace")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (calibration of the HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1")

    import torch

    import paper_2605_07244_amd as mrl
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    mrl.lib()

    over = {}
    if args.full_length:
        over["len_dist"] = "full"
    if args.prompts:
        over["n_prompts"] = args.prompts
    if args.hidden:
        over["d"] = args.hidden
    sp = synth.spec(args.config, **over)
    log(f"generating workload {sp.name}: V={sp.V} d={sp.d} prompts={sp.n_prompts} T={sp.T}")
    batch = synth.make(sp, "cuda")
    B, T, G, N, V, d = (batch[k] for k in ("B", "T", "G", "N", "V", "d"))
    n_scored = int(batch["mask"].sum().item())
    mask = batch["mask"].reshape(-1)
    cfg = mrl.LossConfig(clip_eps_low=sp.clip_eps, clip_eps_high=sp.clip_eps, kl_beta=sp.kl_beta,
                         sgt_lambda=sp.sgt_lambda, dh_dtype=mrl.BF16, chunk_rows=args.chunk_rows,
                         scored_rows_hint=n_scored)
    ws_bytes = mrl.grpo_loss_workspace(B, T, d, V, mrl.BF16, cfg)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    out_logp = torch.empty(N, dtype=torch.float32, device="cuda")
    out_dH = torch.empty((N, d), dtype=torch.bfloat16, device="cuda")
    out_dW = torch.empty((V, d), dtype=torch.float32, device="cuda")
    out_stats = torch.empty(mrl.binding.STATS_BYTES, dtype=torch.uint8, device="cuda")
    log(f"N={N} slots, {n_scored} scored, workspace {ws_bytes / 1e9:.2f} GB")

    def step():
        adv, _, _, _ = mrl.group_advantages(batch["rewards_all"], batch["group_all"], G, batch["in_stats"],
                                            batch["scored"], batch["is_own"])
        seq_adv = adv if adv.numel() == B else synth.seq_adv_from(adv, batch)
        return mrl.grpo_loss_fwd_bwd(batch["H"], batch["W"], batch["targets"], mask, batch["behav"], batch["ref"],
                                     seq_adv, batch["seq_group"], batch["seq_kind"], B, T, G, cfg,
                                     out_dH=out_dH, out_dW=out_dW, workspace=ws, out_logp=out_logp,
                                     out_stats=out_stats)

    for i in range(args.warmup):
        step()
        torch.cuda.synchronize()
        log(f"warmup {i + 1}/{args.warmup} done")
    mrl.profile_enable(True)
    mrl.profile_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = mrl.profile_collect()
    mrl.profile_enable(False)
    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    stats = mrl.read_stats(out_stats)
    assert stats["n_scored_tokens"] == n_scored and stats["n_unprocessed_rows"] == 0, stats

    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = n_scored * args.steps / elapsed
    flop_per_token = 6.0 * d * V
    pct_peak = 100.0 * tokens_per_s * flop_per_token / (MFMA_BF16_PEAK_TFLOPS * 1e12)

    # roofline of the dominant kernel class: algorithmic flops of its launches / their duration
    gemm = {k: prof[k] for k in ("gemm_fwd", "gemm_dh", "gemm_dw")}
    dom = max(gemm, key=lambda k: gemm[k][0])
    dom_ms, dom_launches = gemm[dom]
    flops_per_launch = 2.0 * n_scored * d * V * args.steps / max(dom_launches, 1)
    avg_launch_ms = dom_ms / max(dom_launches, 1)
    achieved = flops_per_launch / (avg_launch_ms * 1e-3) / 1e12 if avg_launch_ms > 0 else 0.0
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tfile):
        try:
            rec = json.load(open(tfile)).get(f"{dom}:config{args.config}")
            traffic = rec["fetch_bytes"] + rec["write_bytes"] if rec else None
        except Exception:
            traffic = None
    roofline = dict(bound="mfma", kernel=dom, achieved=round(achieved, 2), peak=MFMA_BF16_PEAK_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), traffic=traffic,
                    avg_launch_ms=round(avg_launch_ms, 3), launches=int(dom_launches),
                    flops_per_launch=flops_per_launch)
    classes = {k: dict(ms_per_step=round(v[0] / args.steps, 3), launches_per_step=v[1] / args.steps)
               for k, v in prof.items()}
    # HBM-bound passes: algorithmic bytes per step / measured time of the class
    Vp = (V + 255) // 256 * 256
    dp = (d + 127) // 128 * 128
    n_part = 2 * (Vp // 256)
    alg_bytes = dict(
        # mask + target scans (count, fill, sequence lengths), row index, zero fill of the unscored
        # slots' dH rows and log-probs, target logits (one H row and one W row per scored token)
        prep=3 * N * 5 + 4 * n_scored + (N - n_scored) * (2 * d + 4) + n_scored * (4 * d + 12),
        adv=B * 22 + G * 9,
        # partial sums of the forward launches, the per-token inputs / outputs of Eq. (1), the row
        # scale and the patched target column of the stash
        row_epilogue=n_scored * (4 * n_part + 36),
        # gathered copy of each pass's hidden rows, their scaled transpose for the dW launch, and
        # (once per step) the transpose of W for the dH launch
        operand_prep=n_scored * (2 * d + 2 * dp) + n_scored * 4 * dp + V * d * 2 + Vp * dp * 2)
    hbm_passes = {k: dict(algorithmic_GB=round(b / 1e9, 3),
                          achieved_GBps=round(b * args.steps / (prof[k][0] * 1e-3) / 1e9, 1) if prof[k][0] > 0 else None,
                          peak_GBps=8000.0, source="HIP events over the class's launches; counters in profiles/")
                  for k, b in alg_bytes.items()}

    # what the matrix cores sustain on this machine with no memory traffic: clock-limited (constant
    # operands) and power-limited (random-mantissa operands, like the workload's tensors)
    measured_peak = dict(unit="TFLOP/s", instruction="v_mfma_f32_16x16x32_bf16, registers only, 0.5 s each",
                         constant_operands=round(mrl.probe_mfma_rate(False, 0.5), 1),
                         random_operands=round(mrl.probe_mfma_rate(True, 0.5), 1))
    measured_peak["pct_of_random_operand_rate"] = round(
        100.0 * tokens_per_s * flop_per_token / (measured_peak["random_operands"] * 1e12), 2)

    thl_leg = None if args.no_extras else thl_alignment_leg(mrl, synth, torch, with_cpu=not args.no_cpu_baseline)

    fwd_leg = None
    if not args.no_extras:
        # forward-only scoring pass (behaviour / reference traces, re-scoring of pooled peer rollouts):
        # log-probs + entropy of the same batch, 2 N d V FLOP
        ws_f = torch.empty(mrl.lib().mrl_token_scores_workspace(N, d, V, mrl.BF16), dtype=torch.uint8, device="cuda")
        mrl.token_scores(batch["H"], batch["W"], batch["targets"], mask, workspace=ws_f)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(2):
            mrl.token_scores(batch["H"], batch["W"], batch["targets"], mask, workspace=ws_f)
        torch.cuda.synchronize()
        dt_f = (time.perf_counter() - t0) / 2
        del ws_f
        fwd_leg = dict(outputs="logp, lse, entropy", ms_per_call=round(1e3 * dt_f, 2),
                       tokens_per_s=round(n_scored / dt_f, 1),
                       pct_bf16_mfma_peak=round(100.0 * 2.0 * n_scored * d * V / dt_f / (MFMA_BF16_PEAK_TFLOPS * 1e12), 2))

    base = None
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        base = cpu_baseline(batch, sp)

    line = dict(metric=METRIC, value=round(tokens_per_s, 1), unit="tokens/s", n_gpus=1, steps=args.steps,
                warmup=args.warmup, ms_per_step=round(ms_per_step, 3), higher_is_better=True, scaling="weak",
                vs_baseline=None, dtype="bf16", data="synthetic",
                config=dict(workload=f"config{args.config}:{sp.name}" + (":full-length" if args.full_length else ""),
                            V=V, d=d, B=B, T=T, slots=N, scored_tokens=n_scored, prompts=sp.n_prompts,
                            rollouts_per_prompt=sp.k_own + sp.k_peer),
                pct_bf16_mfma_peak=round(pct_peak, 2), flop_per_token=flop_per_token,
                roofline=roofline, measured_mfma_peak=measured_peak, kernel_classes=classes,
                hbm_passes=hbm_passes, thl_word_align=thl_leg, scoring_forward_only=fwd_leg, cpu_baseline=base,
                loss=dict(total=stats["loss_total"], clip_frac=stats["n_clipped_tokens"] / max(n_scored, 1),
                          mean_ratio=stats["mean_ratio"]))
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
