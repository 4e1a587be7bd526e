"""Parity in the launch configuration the benchmark times, with every output compared
element by element.

The default chunking (passes of 65536 scored rows, forward launches of 16384 rows, fp32
read-modify-write of dW from the second pass on) is run over three passes with a ragged last
pass and a ragged last vocabulary tile, at a size the fp64 oracle computes in full: the oracle
functions are called on row chunks here in the test (its logits matrix for all rows at once would
need several GB), the O(N) loss part on the whole batch.
"""
import numpy as np
import pytest
import torch

from oracle import mrl_oracle as orc
from tests import util

pytestmark = pytest.mark.gpu

ORACLE_ROWS = 4096


def _oracle_chunked(b, seq_adv, cfg, eps):
    """Full oracle result (log-probs, loss terms, dH, dW) with the N x V work done ORACLE_ROWS
    scored rows at a time.  Also returns the behaviour trace moved off the clip kinks."""
    B, T, G, N, V, d = (b[k] for k in ("B", "T", "G", "N", "V", "d"))
    H, W = util.to_f64(b["H"]), util.to_f64(b["W"])
    y = b["targets"].cpu().numpy().astype(np.int64)
    m = b["mask"].cpu().numpy().astype(bool).reshape(-1)
    rows = np.nonzero(m)[0]
    logp = np.zeros(N)
    for r0 in range(0, rows.size, ORACLE_ROWS):
        rr = rows[r0:r0 + ORACLE_ROWS]
        logp[rr], _ = orc.token_logprobs(H[rr], W, y[rr])
    b["behav"] = util.move_off_kinks(b, logp, eps)
    res = orc.loss_from_logp(logp, m, util.to_f64(b["behav"]), util.to_f64(b["ref"]), seq_adv,
                             b["seq_group"].cpu().numpy(), b["seq_kind"].cpu().numpy(), B, T, G, cfg)
    dH = np.zeros((N, d))
    dW = np.zeros((V, d))
    for r0 in range(0, rows.size, ORACLE_ROWS):
        rr = rows[r0:r0 + ORACLE_ROWS]
        dH[rr], dW_part, _ = orc.head_backward(H[rr], W, y[rr], res["g"][rr])
        dW += dW_part
    res.update(logp=logp, dH=dH, dW=dW)
    return res, m


@pytest.fixture(scope="module")
def case():
    import paper_2605_07244_amd as mrl
    from workloads import synth
    # 28 prompts x 8 rollouts x 1024 slots, lengths uniform in [256, 1024]: about 143 k scored rows =
    # two full passes of 65536 and a ragged third; V = 32 full 256-wide tiles and a ragged one of 141
    sp = synth.spec(2, n_prompts=28, T=1024, V=8333, d=384)
    b = synth.make(sp, "cuda")
    n_scored = int(b["mask"].sum())
    assert 2 * 65536 < n_scored < 3 * 65536 and n_scored % 256 != 0 and b["V"] % 256 != 0
    adv, _, _, _ = mrl.group_advantages(b["rewards_all"], b["group_all"], b["G"], b["in_stats"], b["scored"], b["is_own"])
    adv_o, *_ = util.oracle_advantages(b)
    assert np.allclose(adv.cpu().numpy(), adv_o, rtol=2e-6, atol=1e-7)
    seq_adv = synth.seq_adv_from(adv, b)
    want, m = _oracle_chunked(b, seq_adv.cpu().numpy().astype(np.float64), util.cfg_dict(sp), sp.clip_eps)
    return mrl, sp, b, seq_adv, n_scored, want, m


@pytest.mark.parametrize("accumulate", [0, 1])
def test_default_chunking_three_passes_every_element(case, accumulate):
    mrl, sp, b, seq_adv, n_scored, want, m = case
    B, T, G, N, V, d = (b[k] for k in ("B", "T", "G", "N", "V", "d"))

    lc = mrl.LossConfig(clip_eps_low=sp.clip_eps, clip_eps_high=sp.clip_eps, kl_beta=sp.kl_beta,
                        sgt_lambda=sp.sgt_lambda, scored_rows_hint=n_scored, accumulate_dw=accumulate)   # chunk_rows = 0: default
    dW0 = None
    out_dW = None
    if accumulate:
        g = torch.Generator("cuda").manual_seed(5)
        dW0 = 1e-5 * torch.randn((V, d), device="cuda", generator=g)
        out_dW = dW0.clone()
    got = mrl.grpo_loss_fwd_bwd(b["H"], b["W"], b["targets"], b["mask"].reshape(-1), b["behav"], b["ref"], seq_adv,
                                b["seq_group"], b["seq_kind"], B, T, G, lc, out_dW=out_dW)
    torch.cuda.synchronize()
    st = mrl.read_stats(got["stats"])
    assert st["n_scored_tokens"] == n_scored and st["n_unprocessed_rows"] == 0 and st["n_bad_targets"] == 0

    logp = got["logp"].cpu().numpy().astype(np.float64)
    assert np.all(logp[~m] == 0.0)
    err = np.abs(logp[m] - want["logp"][m])
    print(f"logp: max err {err.max():.2e} over {m.sum()} rows")
    assert err.max() <= util.LOGP_TOL
    util.check_loss_terms(st, want, sp.kl_beta, sp.sgt_lambda)
    assert st["n_clipped_tokens"] == want["n_clipped_tokens"]
    assert st["n_zero_grad_tokens"] == want["n_zero_grad_tokens"]
    assert abs(st["mean_ratio"] - want["mean_ratio"]) <= 1e-4 * want["mean_ratio"]
    assert abs(st["max_ratio"] - want["max_ratio"]) <= 1e-4 * want["max_ratio"]
    assert abs(st["mean_k3"] - want["mean_k3"]) <= 1e-3 * want["mean_k3"]

    dH = util.to_f64(got["dH"])
    assert np.all(dH[~m] == 0.0)
    util.check_gradient("dH", dH, want["dH"])
    dW = util.to_f64(got["dW"])
    if accumulate:
        dW = dW - util.to_f64(dW0)
    util.check_gradient("dW", dW, want["dW"])
    # the ragged last vocabulary tile and the rows of the ragged last pass on their own
    util.check_gradient("dW[last tile]", dW[V // 256 * 256:], want["dW"][V // 256 * 256:])
    last_pass = np.nonzero(m)[0][2 * 65536:]
    util.check_gradient("dH[last pass]", dH[last_pass], want["dH"][last_pass])
