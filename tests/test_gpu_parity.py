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
              adv_mode=1, h_scale=None, loss_agg=0, ratio_level=0, behav_jitter=None, w_shift=None):
    batch = synth.make(sp, "cuda")
    if h_scale is not None:
        batch["H"] = (batch["H"].float() * h_scale).to(batch["H"].dtype)
    if h_scale is not None or w_shift is not None:
        centre = synth.logp_proxy(batch["H"], batch["W"], batch["targets"])
        g = torch.Generator("cuda").manual_seed(1)
        batch["behav"] = centre + 0.1 * torch.randn(batch["N"], device="cuda", generator=g)
        batch["ref"] = centre + 0.1 * torch.randn(batch["N"], device="cuda", generator=g)
    if w_shift is not None:
        # the same vector added to every row of W moves all logits of a token row by <h, shift>:
        # the softmax does not change (up to the rounding of W), the magnitude of the logits does;
        # the traces above stay centred on the unshifted head
        g = torch.Generator("cuda").manual_seed(3)
        c = w_shift / (sp.d ** 0.5) * torch.randn(sp.d, device="cuda", generator=g)
        batch["W"] = (batch["W"].float() + c[None, :]).to(batch["W"].dtype)
        batch["w_common"] = c.cpu().numpy().astype(np.float64)
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
    if w_shift is None:
        util.check_gradient("dH", dH, want["dH"], rel_tol)
    else:
        # dH = dz W.  With a common vector c in every row of W, dH = dz W0 + (sum_v dz) c, and the
        # exact sum_v dz = 0 is met by bf16 operands only up to their rounding: the component of
        # dH along c is ill-conditioned for ANY implementation whose dz operand is bf16.  Checked:
        # the part orthogonal to c to the usual tolerance, the part along c against the bound that
        # rounding implies, |sum_v delta(dz_v)| |c| <= 2^-9 sum_v |dz_v| |c| <= 2^-8 |g| |c|.
        c = batch["w_common"]
        chat = c / np.linalg.norm(c)
        perp = lambda x: x - np.outer(x @ chat, chat)
        util.check_gradient("dH orthogonal to the common vector", perp(dH), perp(want["dH"]), rel_tol)
        along = np.abs((dH - want["dH"]) @ chat)
        bound = 2.0 ** -8 * np.abs(want["g"]) * np.linalg.norm(c) + 2.0 ** -8 * np.linalg.norm(want["dH"], axis=1)
        assert np.all(along <= bound + 1e-30), float(np.max(along / np.maximum(bound, 1e-300)))
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
    (2, dict(n_prompts=2, T=40, V=2500, d=200)),     # width not a multiple of the 128-wide panel pairs: zero-padded operands
    (3, dict(n_prompts=2, T=24, V=3001, d=328)),     # one and a bit 256-wide tiles of d, ragged everything
])
def test_mini_configs_bf16(mrl, synth, idx, over):
    sp = synth.spec(idx, **over)
    _run_both(mrl, synth, sp, chunk_rows=256)


def test_mini_config5_full_vocab_and_width(mrl, synth):
    # full V = 151936 (593.5 tiles: ragged last tile) and d = 4096, a few hundred rows
    sp = synth.spec(5, n_prompts=1, T=56)
    _run_both(mrl, synth, sp, chunk_rows=256)


def test_mini_config2_full_vocab_uneven_dw_tail(mrl, synth):
    # full V = 151936 at d = 1536: the last two rows of dW tiles (12 tiles) are cut into K slices that
    # the launch plan deals to the XCDs unevenly (those that finish their whole tiles early take them)
    sp = synth.spec(2, n_prompts=1, T=40)
    _run_both(mrl, synth, sp, chunk_rows=256)


@pytest.mark.parametrize("V,d", [(8627, 2048), (20224, 2304), (7424, 2304), (11008, 1536), (16819, 640),
                                 (13312, 2304), (17587, 1024)])
def test_dw_tail_plans(mrl, synth, V, d):
    """Head shapes whose dW launch cuts its ragged last rows of tiles into K slices, with 1 to 7 such rows,
    2 to 8 slices, item counts that differ from XCD to XCD, and widths of a whole and of a ragged number of
    256-wide tiles; two passes, so that the second adds the slices into the first's result."""
    plan = mrl.dw_tail_plan(V, d)
    assert plan["split"] >= 2
    sp = synth.spec(2, n_prompts=2, T=40, V=V, d=d)
    _run_both(mrl, synth, sp, chunk_rows=256)


def test_single_chunk_default_and_fp32_dh(mrl, synth):
    sp = synth.spec(2, n_prompts=2, T=40, V=2500)
    _run_both(mrl, synth, sp, chunk_rows=0, dh_dtype=0)


def test_peaked_softmax(mrl, synth):
    # hidden states scaled x8: logits of std ~ 6, exercises the range of the stashed exponentials
    sp = synth.spec(2, n_prompts=2, T=24, V=3000, d=256)
    _run_both(mrl, synth, sp, chunk_rows=256, h_scale=8.0)


def test_large_logit_offsets(mrl, synth):
    """Logits of magnitude 30-100 with an ordinary softmax (a common vector added to every row of
    W shifts each token row's logits by about N(0, 40)): exponentials are taken relative to the
    row's target logit, so neither the log-probs nor the backward operands lose accuracy with the
    size of the logits."""
    sp = synth.spec(2, n_prompts=2, T=24, V=3000, d=256)
    batch, got, want, st = _run_both(mrl, synth, sp, chunk_rows=256, w_shift=40.0)
    z = util.to_f64(batch["H"]) @ util.to_f64(batch["W"]).T
    assert np.abs(z).max() > 60 and np.median(np.abs(z).max(axis=1)) > 20
    assert st["n_saturated_rows"] == 0


def test_rows_outside_the_representable_range_are_counted_and_dropped(mrl, synth):
    """A few token rows whose sampled token is (numerically) impossible under the learner: target
    log-prob far below -97.  They are counted, report a saturated finite log-prob, and drop out of
    the loss and the gradients; every other row and the totals minus those rows' terms match the
    oracle."""
    sp = synth.spec(2, n_prompts=2, T=24, V=3000, d=256)
    batch = synth.make(sp, "cuda")
    B, T, G = batch["B"], batch["T"], batch["G"]
    m = batch["mask"].reshape(-1).bool()
    scored = torch.nonzero(m)[:, 0]
    wild = scored[[5, 77, 200]]
    wild_np = wild.cpu().numpy()
    batch["H"][wild] = (batch["H"][wild].float() * 120.0).to(torch.bfloat16)     # logits of std ~ 40
    z = util.to_f64(batch["H"][wild]) @ util.to_f64(batch["W"]).T
    batch["targets"][wild] = torch.tensor(np.argmin(z, axis=1), dtype=torch.int32, device="cuda")   # the least likely id
    adv, *_ = util.oracle_advantages(batch)
    seq_adv = torch.tensor(adv[:B], dtype=torch.float32, device="cuda")
    cfg = util.cfg_dict(sp)
    first = util.oracle_loss(batch, adv[:B], cfg, need_grads=False)
    assert np.all(first["logp"][wild_np] < -150)
    # keep the oracle's own terms of those rows finite: on-policy and on-reference there
    batch["behav"] = util.move_off_kinks(batch, first["logp"], sp.clip_eps)
    batch["behav"][wild] = torch.tensor(first["logp"][wild_np], dtype=torch.float32, device="cuda")
    batch["ref"][wild] = batch["behav"][wild]
    want = util.oracle_loss(batch, adv[:B], cfg)
    lc = mrl.LossConfig(kl_beta=sp.kl_beta, sgt_lambda=sp.sgt_lambda, chunk_rows=256, dh_dtype=mrl.BF16)
    got = mrl.grpo_loss_fwd_bwd(batch["H"], batch["W"], batch["targets"], batch["mask"].reshape(-1), batch["behav"],
                                batch["ref"], seq_adv, batch["seq_group"], batch["seq_kind"], B, T, G, lc)
    torch.cuda.synchronize()
    st = mrl.read_stats(got["stats"])
    assert st["n_saturated_rows"] == 3 and st["n_scored_tokens"] == int(m.sum())
    assert torch.isfinite(got["logp"]).all() and torch.isfinite(got["dH"].float()).all() and torch.isfinite(got["dW"]).all()
    assert torch.all(got["logp"][wild] < -97) and torch.all(got["dH"][wild] == 0)
    ok = m.clone()
    ok[wild] = False
    okn = ok.cpu().numpy()
    assert np.max(np.abs(got["logp"].cpu().numpy()[okn] - want["logp"][okn])) <= util.LOGP_TOL
    dH_want = want["dH"].copy()
    dH_want[wild_np] = 0.0
    util.check_gradient("dH", util.to_f64(got["dH"]), dH_want)
    _, dW_wild, _ = orc.head_backward(util.to_f64(batch["H"][wild]), util.to_f64(batch["W"]),
                                      batch["targets"][wild].cpu().numpy(), want["g"][wild_np])
    util.check_gradient("dW", util.to_f64(got["dW"]), want["dW"] - dW_wild)
    # loss: the oracle's total minus the dropped rows' terms (J = A at ratio 1, k3 = 0 there)
    J = np.minimum(want["s1"], want["s2"])
    pg = want["loss_pg"] + float(np.sum(want["c"][wild_np] * J[wild_np]))
    assert abs(st["loss_pg"] - pg) <= 1e-4 * float(np.sum(want["c"] * np.abs(J)))
    assert abs(st["loss_kl"] - want["loss_kl"]) <= 1e-2 * want["loss_kl"]


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
