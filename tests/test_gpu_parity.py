"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import mrl_oracle as orc
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mrl():
    import paper_2605_07244_amd as m
    m.lib()
    return m


@pytest.fixture(scope="module")
def synth():
    from workloads import synth as s
    return s


def _gpu_adv(mrl, batch, mode=1, **kw):
    return mrl.group_advantages(batch["rewards_all"], batch["group_all"], batch["G"], batch["in_stats"],
                                batch["scored"], batch["is_own"], mode=mode, **kw)


def _run_both(mrl, synth, sp, chunk_rows=256, dh_dtype=None, logp_tol=util.LOGP_TOL, rel_tol=util.REL_TOL,
              adv_mode=1, h_scale=None, loss_agg=0, ratio_level=0, behav_jitter=None):
    batch = synth.make(sp, "cuda")
    if h_scale is not None:
        batch["H"] = (batch["H"].float() * h_scale).to(batch["H"].dtype)
        centre = synth.logp_proxy(batch["H"], batch["W"], batch["targets"])
        g = torch.Generator("cuda").manual_seed(1)
        batch["behav"] = centre + 0.1 * torch.randn(batch["N"], device="cuda", generator=g)
        batch["ref"] = centre + 0.1 * torch.randn(batch["N"], device="cuda", generator=g)
    cfg = util.cfg_dict(sp, loss_agg=loss_agg, ratio_level=ratio_level)
    if behav_jitter is not None:
        centre = synth.logp_proxy(batch["H"], batch["W"], batch["targets"])
        g = torch.Generator("cuda").manual_seed(2)
        batch["behav"] = centre + behav_jitter * torch.randn(batch["N"], device="cuda", generator=g)

    # advantages: HIP vs oracle
    adv_g, mean_g, std_g, flags_g = _gpu_adv(mrl, batch, mode=adv_mode)
    adv_o, mean_o, std_o, flags_o = util.oracle_advantages(batch, mode=adv_mode)
    assert np.array_equal(flags_g.cpu().numpy(), flags_o)
    assert np.allclose(adv_g.cpu().numpy(), adv_o, rtol=2e-6, atol=1e-7)
    assert np.allclose(mean_g.cpu().numpy(), mean_o, rtol=1e-6, atol=1e-7)
    assert np.allclose(std_g.cpu().numpy(), std_o, rtol=1e-6, atol=1e-7)
    seq_adv = synth.seq_adv_from(adv_g, batch)
    seq_adv_o = seq_adv.cpu().numpy().astype(np.float64)   # identical inputs to both loss paths

    # keep tokens off the clip kinks (decided from the oracle's log-probs)
    first = util.oracle_loss(batch, seq_adv_o, cfg, need_grads=False)
    if ratio_level == 0:
        batch["behav"] = util.move_off_kinks(batch, first["logp"], sp.clip_eps)
    else:
        batch["behav"] = util.move_off_kinks_seq(batch, first["logp"], sp.clip_eps, ratio_level)
    want = util.oracle_loss(batch, seq_adv_o, cfg)

    lc = mrl.LossConfig(clip_eps_low=sp.clip_eps, clip_eps_high=sp.clip_eps, kl_beta=sp.kl_beta,
                        sgt_lambda=sp.sgt_lambda, loss_agg=loss_agg, chunk_rows=chunk_rows, ratio_level=ratio_level,
                        dh_dtype=(mrl.F32 if sp.dtype == torch.float32 else mrl.BF16) if dh_dtype is None else dh_dtype)
    got = mrl.grpo_loss_fwd_bwd(batch["H"], batch["W"], batch["targets"], batch["mask"].reshape(-1),
                                batch["behav"], batch["ref"], seq_adv, batch["seq_group"], batch["seq_kind"],
                                batch["B"], batch["T"], batch["G"], lc)
    torch.cuda.synchronize()
    st = mrl.read_stats(got["stats"])

    m = batch["mask"].reshape(-1).cpu().numpy().astype(bool)
    logp = got["logp"].cpu().numpy().astype(np.float64)
    assert np.all(logp[~m] == 0.0)
    assert np.max(np.abs(logp[m] - want["logp"][m])) <= logp_tol if m.any() else True
    util.check_loss_terms(st, want, sp.kl_beta, sp.sgt_lambda, rel_tol)
    assert st["n_scored_tokens"] == want["n_scored_tokens"]
    assert st["n_clipped_tokens"] == want["n_clipped_tokens"]
    assert st["n_zero_grad_tokens"] == want["n_zero_grad_tokens"]
    assert st["n_bad_targets"] == 0
    assert abs(st["mean_ratio"] - want["mean_ratio"]) <= 1e-2 * max(want["mean_ratio"], 1e-12)
    assert abs(st["max_ratio"] - want["max_ratio"]) <= 1e-2 * max(want["max_ratio"], 1e-12)
    assert abs(st["mean_k3"] - want["mean_k3"]) <= 1e-2 * max(want["mean_k3"], 1e-9)

    dH = util.to_f64(got["dH"])
    assert np.all(dH[~m] == 0.0)
    util.check_gradient("dH", dH, want["dH"], rel_tol)
    util.check_gradient("dW", util.to_f64(got["dW"]), want["dW"], rel_tol)
    return batch, got, want, st


def test_config1_tiny_fp32_exhaustive(mrl, synth):
    sp = synth.spec(1)
    _run_both(mrl, synth, sp, chunk_rows=0, logp_tol=util.F32_LOGP_TOL, rel_tol=util.F32_REL_TOL)


def test_fp32_path_multichunk_ragged(mrl, synth):
    sp = synth.spec(1, n_prompts=5, T=150, V=777, d=72)      # 6000 slots, ragged everything
    _run_both(mrl, synth, sp, chunk_rows=2048, logp_tol=util.F32_LOGP_TOL, rel_tol=util.F32_REL_TOL)


@pytest.mark.parametrize("idx,over", [
    (2, dict(n_prompts=2, T=40, V=2500)),
    (3, dict(n_prompts=2, T=24, V=3001)),
    (4, dict(n_prompts=5, T=16, V=1000)),
    (5, dict(n_prompts=2, T=48, V=4100, d=512)),
])
def test_mini_configs_bf16(mrl, synth, idx, over):
    sp = synth.spec(idx, **over)
    _run_both(mrl, synth, sp, chunk_rows=256)


def test_mini_config5_full_vocab_and_width(mrl, synth):
    # full V = 151936 (593.5 tiles: ragged last tile) and d = 4096, a few hundred rows
    sp = synth.spec(5, n_prompts=1, T=56)
    _run_both(mrl, synth, sp, chunk_rows=256)


def test_single_chunk_default_and_fp32_dh(mrl, synth):
    sp = synth.spec(2, n_prompts=2, T=40, V=2500)
    _run_both(mrl, synth, sp, chunk_rows=0, dh_dtype=0)


def test_peaked_softmax(mrl, synth):
    # hidden states scaled x8: logits of std ~ 6, exercises the max-subtraction and fp16 stash
    sp = synth.spec(2, n_prompts=2, T=24, V=3000, d=256)
    _run_both(mrl, synth, sp, chunk_rows=256, h_scale=8.0)


def test_global_token_mean_and_batch_zn(mrl, synth):
    sp = synth.spec(2, n_prompts=3, T=20, V=1500, d=128)
    _run_both(mrl, synth, sp, chunk_rows=256, adv_mode=2, loss_agg=1)


@pytest.mark.parametrize("level,idx,over,jitter", [
    (1, 2, dict(n_prompts=3, T=40, V=2500), 0.03),     # summed log-ratio: small token jitter keeps responses near the band
    (2, 2, dict(n_prompts=3, T=40, V=2500), 0.8),      # per-token mean: large jitter to reach the band edges
    (1, 4, dict(n_prompts=5, T=16, V=1000), 0.05),     # with SGT auxiliary rows
    (2, 1, dict(), 2.0),                               # fp32 sanity path
])
def test_response_level_ratio(mrl, synth, level, idx, over, jitter):
    """Eq. (1) with the response-level ratio of App. I.1; responses span several 256-row passes."""
    sp = synth.spec(idx, **over)
    f32 = sp.dtype == torch.float32
    batch, got, want, st = _run_both(mrl, synth, sp, chunk_rows=0 if f32 else 256, ratio_level=level,
                                     behav_jitter=jitter, logp_tol=util.F32_LOGP_TOL if f32 else util.LOGP_TOL,
                                     rel_tol=util.F32_REL_TOL if f32 else util.REL_TOL)
    # the clip is exercised on both sides of the band or at least on one
    assert 0 < st["n_clipped_tokens"] < st["n_scored_tokens"]
