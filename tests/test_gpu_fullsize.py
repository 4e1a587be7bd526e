"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The CPU oracle cannot run N x V = 10^11 logits, so it computes, from the inputs alone,
(i) the log-prob, (ii) dL/dl and (iii) the dH row of SAMPLED scored tokens (one row of
logits each, fp64), and the whole-batch quantities that need no vocabulary work
(weights, counts).  The O(N) part of the step (Eq. 1 / Eq. 2 terms, statistics) is recomputed by
the oracle for ALL rows from the log-probs the GPU returned (validated on the sampled rows), and
SAMPLED VOCABULARY ROWS of dW are recomputed by the oracle's formula over all scored rows, with
each row's log-sum-exp taken as (fp64 target logit) - (that validated log-prob).
Everything else is checked through properties that hold at any size:
  * <dH, H> = <dW, W>  (both equal sum_n,v dz[n,v] z[n,v]),
  * sum_v dW[v, :] = 0 (each dz row sums to zero),
  * unscored slots have zero log-prob and zero dH rows,
  * loss_total = loss_pg + beta * loss_kl + lambda * loss_sgt, counts match the mask.
"""
import numpy as np
import pytest
import torch

from oracle import mrl_oracle as orc
from tests import util

pytestmark = pytest.mark.gpu

N_SAMPLES = 48
KINK_MARGIN = 5e-3


def _run_full(idx, **over):
    import paper_2605_07244_amd as mrl
    from workloads import synth
    sp = synth.spec(idx, **over)
    b = synth.make(sp, "cuda")
    B, T, G, N, V, d = (b[k] for k in ("B", "T", "G", "N", "V", "d"))
    adv, _, _, flags = mrl.group_advantages(b["rewards_all"], b["group_all"], G, b["in_stats"], b["scored"], b["is_own"])
    adv_o, _, _, flags_o = util.oracle_advantages(b)
    assert np.array_equal(flags.cpu().numpy(), flags_o)
    assert np.allclose(adv.cpu().numpy(), adv_o, rtol=2e-6, atol=1e-7)
    seq_adv = synth.seq_adv_from(adv, b)
    n_scored = int(b["mask"].sum())
    lc = mrl.LossConfig(clip_eps_low=sp.clip_eps, clip_eps_high=sp.clip_eps, kl_beta=sp.kl_beta,
                        sgt_lambda=sp.sgt_lambda, scored_rows_hint=n_scored)       # as bench.py
    out = mrl.grpo_loss_fwd_bwd(b["H"], b["W"], b["targets"], b["mask"].reshape(-1), b["behav"], b["ref"], seq_adv,
                                b["seq_group"], b["seq_kind"], B, T, G, lc)
    torch.cuda.synchronize()
    st = mrl.read_stats(out["stats"])
    return mrl, sp, b, seq_adv, out, st, n_scored


def _check_sampled(sp, b, seq_adv, out, st, n_scored):
    B, T, G, N, V, d = (b[k] for k in ("B", "T", "G", "N", "V", "d"))
    mask_np = b["mask"].cpu().numpy().astype(bool)
    mflat = mask_np.reshape(-1)
    cfg = util.cfg_dict(sp)
    # whole-batch weights from the masks alone
    c, c_sgt = orc.sequence_weights(mask_np, b["seq_group"].cpu().numpy(), b["seq_kind"].cpu().numpy(), G)
    c, c_sgt = c.reshape(-1), c_sgt.reshape(-1)
    rng = np.random.default_rng(1234 + sp.index)
    scored_idx = np.nonzero(mflat)[0]
    rows = np.sort(rng.choice(scored_idx, size=N_SAMPLES, replace=False))
    # always include first / last scored rows (pass boundaries) and an auxiliary row if there is one
    rows[0], rows[-1] = scored_idx[0], scored_idx[-1]
    aux = np.nonzero(mflat & np.repeat(b["seq_kind"].cpu().numpy() == 1, T))[0]
    if aux.size:
        rows[1] = aux[aux.size // 2]
    rows = np.unique(rows)
    ridx = torch.tensor(rows, device="cuda")
    Hs = util.to_f64(b["H"][ridx])
    W = util.to_f64(b["W"])
    ys = b["targets"][ridx].cpu().numpy()
    logp_o, lse_o = orc.token_logprobs(Hs, W, ys)
    logp_g = out["logp"][ridx].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(logp_g - logp_o)) <= util.LOGP_TOL
    # dL/dl of the sampled rows from the oracle's own log-probs
    beh = util.to_f64(b["behav"][ridx]); ref = util.to_f64(b["ref"][ridx])
    A = seq_adv.cpu().numpy().astype(np.float64)[rows // T]
    kind = b["seq_kind"].cpu().numpy()[rows // T]
    w, s1, s2, J, dJ, k3, dk3 = orc.token_terms(logp_o, beh, ref, A, cfg["clip_eps_low"], cfg["clip_eps_high"])
    g = np.where(kind == 0, c[rows] * (-dJ + cfg["kl_beta"] * dk3), -cfg["sgt_lambda"] * c_sgt[rows])
    dH_o, _, _ = orc.head_backward(Hs, W, ys, g)
    dH_g = util.to_f64(out["dH"][ridx])
    # tokens whose ratio sits on a clip edge may legitimately take either branch in fp32
    near = (kind == 0) & ((np.abs(np.log(w) - np.log1p(-cfg["clip_eps_low"])) < KINK_MARGIN) |
                          (np.abs(np.log(w) - np.log1p(cfg["clip_eps_high"])) < KINK_MARGIN))
    assert near.sum() <= max(2, N_SAMPLES // 10)
    ok = ~near
    assert util.rel_fro(dH_g[ok], dH_o[ok]) <= util.REL_TOL
    per_row = np.linalg.norm(dH_g[ok] - dH_o[ok], axis=1) / np.maximum(np.linalg.norm(dH_o[ok], axis=1), 1e-30)
    assert np.max(per_row[np.linalg.norm(dH_o[ok], axis=1) > 0]) <= 3 * util.REL_TOL
    return mflat


def _check_epilogue_all_rows(sp, b, seq_adv, out, st):
    """Eq. (1) / Eq. (2) terms and statistics for every row: the oracle's O(N) part evaluated in
    fp64 on the log-probs the GPU produced."""
    B, T, G = b["B"], b["T"], b["G"]
    cfg = util.cfg_dict(sp)
    want = orc.loss_from_logp(out["logp"].cpu().numpy().astype(np.float64), b["mask"].cpu().numpy().reshape(B, T),
                              util.to_f64(b["behav"]), util.to_f64(b["ref"]), seq_adv.cpu().numpy().astype(np.float64),
                              b["seq_group"].cpu().numpy(), b["seq_kind"].cpu().numpy(), B, T, G, cfg)
    util.check_loss_terms(st, want, sp.kl_beta, sp.sgt_lambda)
    n = max(want["n_scored_tokens"], 1)
    # fp32 and fp64 may disagree on tokens whose ratio sits within rounding of a clip edge
    assert abs(st["n_clipped_tokens"] - want["n_clipped_tokens"]) <= max(2, int(2e-5 * n))
    assert abs(st["n_zero_grad_tokens"] - want["n_zero_grad_tokens"]) <= max(2, int(2e-5 * n))
    assert abs(st["mean_ratio"] - want["mean_ratio"]) <= 1e-5 * want["mean_ratio"]
    assert abs(st["max_ratio"] - want["max_ratio"]) <= 1e-5 * want["max_ratio"]
    assert abs(st["mean_k3"] - want["mean_k3"]) <= 1e-4 * want["mean_k3"]
    return want


def _check_dw_sampled_vocab_rows(sp, b, out, g_all, n_rows=16, chunk=32768):
    """dW[v, :] = sum_n g_n (1[y_n = v] - exp(z[n, v] - lse_n)) H[n, :] for sampled vocabulary ids
    v, over all scored rows n, in fp64 on the host, chunk by chunk.  lse_n = <H_n, W_{y_n}> (fp64)
    minus the GPU's log-prob of the row; g_n is the oracle's dL/dl evaluated on those log-probs.
    The sample always holds the last id of the vocabulary (ragged last tile when V % 256 != 0), id 0,
    ids that are targets of some scored row, and ids that are nobody's target."""
    V, d = b["V"], b["d"]
    m = b["mask"].reshape(-1).bool()
    rows = torch.nonzero(m)[:, 0]
    y_all = b["targets"][rows].long()
    rng = np.random.default_rng(4321 + sp.index)
    hit = torch.unique(y_all).cpu().numpy()
    vs = np.unique(np.concatenate([[0, V - 1, V - 2, V // 256 * 256 - 1, min(V - 1, V // 256 * 256)],
                                   rng.choice(hit, size=n_rows // 2, replace=False),
                                   rng.integers(0, V, size=n_rows // 2)]))
    Wv = util.to_f64(b["W"][torch.tensor(vs, device="cuda")])          # [n_v, d]
    logp_g = out["logp"]
    ref = np.zeros((vs.size, d))
    for r0 in range(0, rows.numel(), chunk):
        rr = rows[r0:r0 + chunk]
        Hc = util.to_f64(b["H"][rr])
        yc = b["targets"][rr].long()
        Wy = util.to_f64(b["W"][yc])
        zt = np.einsum("nk,nk->n", Hc, Wy)
        lse = zt - logp_g[rr].cpu().numpy().astype(np.float64)
        z = Hc @ Wv.T                                                   # [rows, n_v]
        dz = -g_all[rr.cpu().numpy()][:, None] * np.exp(z - lse[:, None])
        yc_np = yc.cpu().numpy()
        for j, v in enumerate(vs):
            sel = yc_np == v
            dz[sel, j] += g_all[rr.cpu().numpy()][sel]
        ref += dz.T @ Hc
    got = util.to_f64(out["dW"][torch.tensor(vs, device="cuda")])
    util.check_gradient(f"dW[{vs.size} sampled vocabulary rows]", got, ref)


def _check_properties(sp, b, out, st, n_scored, mflat):
    N, V, d = b["N"], b["V"], b["d"]
    assert st["n_scored_tokens"] == n_scored and st["n_unprocessed_rows"] == 0 and st["n_bad_targets"] == 0
    total = st["loss_pg"] + sp.kl_beta * st["loss_kl"] + sp.sgt_lambda * st["loss_sgt"]
    # beta and lambda are fp32 in the library's configuration block
    assert abs(st["loss_total"] - total) <= 1e-6 * (abs(st["loss_pg"]) + abs(st["loss_kl"]) + abs(st["loss_sgt"]))
    assert st["loss_kl"] >= 0 and 0 <= st["n_clipped_tokens"] <= n_scored
    m = torch.tensor(mflat, device="cuda")
    assert torch.all(out["logp"][~m] == 0)
    assert not torch.isnan(out["logp"]).any()
    # unscored dH rows are zero (checked on a strided subset to bound the time)
    um = torch.nonzero(~m)[:, 0]
    if um.numel():
        assert torch.all(out["dH"][um[:: max(1, um.numel() // 4096)]] == 0)
    # trace identity and zero column sums, accumulated in fp64 chunk by chunk on the device
    lhs = 0.0
    for r0 in range(0, N, 1 << 16):
        r1 = min(N, r0 + (1 << 16))
        lhs += float((out["dH"][r0:r1].double() * b["H"][r0:r1].double()).sum())
    rhs = 0.0
    colsum = torch.zeros(d, dtype=torch.float64, device="cuda")
    absum = 0.0
    for v0 in range(0, V, 1 << 14):
        v1 = min(V, v0 + (1 << 14))
        blk = out["dW"][v0:v1].double()
        rhs += float((blk * b["W"][v0:v1].double()).sum())
        colsum += blk.sum(dim=0)
        absum += float(blk.abs().sum())
    scale = float(out["dW"].double().norm() * b["W"].double().norm())
    assert abs(lhs - rhs) <= 1e-2 * max(abs(rhs), 1e-3 * scale), (lhs, rhs)
    assert float(colsum.abs().sum()) <= 1e-2 * absum


def test_config2_full_size_sampled():
    mrl, sp, b, seq_adv, out, st, n_scored = _run_full(2)
    mflat = _check_sampled(sp, b, seq_adv, out, st, n_scored)
    want = _check_epilogue_all_rows(sp, b, seq_adv, out, st)
    _check_dw_sampled_vocab_rows(sp, b, out, want["g"])
    _check_properties(sp, b, out, st, n_scored, mflat)


def test_config3_prp_pool_full_size_sampled():
    # PRP pooled batch (own + peer rollouts in one group, heavy-tailed peer ratios), all 32 prompts
    mrl, sp, b, seq_adv, out, st, n_scored = _run_full(3)
    assert st["n_clipped_tokens"] > 0.2 * n_scored          # peer ratios mostly leave the clip band
    mflat = _check_sampled(sp, b, seq_adv, out, st, n_scored)
    _check_epilogue_all_rows(sp, b, seq_adv, out, st)
    _check_properties(sp, b, out, st, n_scored, mflat)


def test_config4_xgrpo_sgt_full_size_sampled():
    # XGRPO pooled baseline and SGT auxiliary rows, all 64 prompts
    mrl, sp, b, seq_adv, out, st, n_scored = _run_full(4)
    assert b["n_aux"] > 0 and st["loss_sgt"] > 0
    mflat = _check_sampled(sp, b, seq_adv, out, st, n_scored)
    _check_epilogue_all_rows(sp, b, seq_adv, out, st)
    _check_properties(sp, b, out, st, n_scored, mflat)


def test_config5_full_size_sampled():
    mrl, sp, b, seq_adv, out, st, n_scored = _run_full(5)
    mflat = _check_sampled(sp, b, seq_adv, out, st, n_scored)
    want = _check_epilogue_all_rows(sp, b, seq_adv, out, st)
    _check_dw_sampled_vocab_rows(sp, b, out, want["g"])
    _check_properties(sp, b, out, st, n_scored, mflat)


def test_config5_scoring_pass_full_size_sampled():
    """Forward-only scoring pass (log-prob, lse, entropy) on configuration 5 as bench.py runs it:
    sampled scored rows against the oracle, and size-independent properties for all rows."""
    import paper_2605_07244_amd as mrl
    from workloads import synth
    sp = synth.spec(5)
    b = synth.make(sp, "cuda")
    mask = b["mask"].reshape(-1)
    lp, lse, ent = mrl.token_scores(b["H"], b["W"], b["targets"], mask)
    torch.cuda.synchronize()
    m = mask.bool()
    assert torch.all(lp[~m] == 0) and torch.all(lse[~m] == 0) and torch.all(ent[~m] == 0)
    assert not torch.isnan(lp).any() and not torch.isnan(ent).any()
    # 0 <= H <= log V and log p <= 0 on every scored row
    assert float(ent[m].min()) >= 0.0 and float(ent[m].max()) <= np.log(sp.V) + 1e-3
    assert float(lp[m].max()) <= 0.0
    rng = np.random.default_rng(77)
    scored_idx = torch.nonzero(m)[:, 0].cpu().numpy()
    rows = np.unique(np.concatenate([rng.choice(scored_idx, size=N_SAMPLES, replace=False),
                                     scored_idx[[0, -1]]]))
    ridx = torch.tensor(rows, device="cuda")
    Hs, W = util.to_f64(b["H"][ridx]), util.to_f64(b["W"])
    want_lp, want_lse = orc.token_logprobs(Hs, W, b["targets"][ridx].cpu().numpy())
    want_ent = orc.token_entropy(Hs, W)
    assert np.max(np.abs(lp[ridx].cpu().numpy() - want_lp)) <= util.LOGP_TOL
    assert np.max(np.abs(lse[ridx].cpu().numpy() - want_lse)) <= util.LOGP_TOL
    assert np.max(np.abs(ent[ridx].cpu().numpy() - want_ent)) <= util.LOGP_TOL
