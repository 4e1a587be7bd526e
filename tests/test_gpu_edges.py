"""GPU edge cases of the C-ABI entry points, each checked against the CPU oracle."""
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


def _small(synth, **over):
    kw = dict(n_prompts=2, T=24, V=1200, d=128)
    kw.update(over)
    sp = synth.spec(2, **kw)
    b = synth.make(sp, "cuda")
    adv, *_ = util.oracle_advantages(b)
    b["seq_adv"] = torch.tensor(adv[:b["B"]], dtype=torch.float32, device="cuda")
    return sp, b


def _gpu_loss(mrl, sp, b, mask=None, targets=None, **kw):
    cfgkw = dict(kl_beta=sp.kl_beta, sgt_lambda=sp.sgt_lambda, chunk_rows=256)
    cfgkw.update(kw.pop("cfg", {}))
    lc = mrl.LossConfig(**cfgkw)
    mask = b["mask"].reshape(-1) if mask is None else mask
    targets = b["targets"] if targets is None else targets
    out = mrl.grpo_loss_fwd_bwd(b["H"], b["W"], targets, mask, b["behav"], b["ref"], b["seq_adv"],
                                b["seq_group"], b["seq_kind"], b["B"], b["T"], b["G"], lc, **kw)
    torch.cuda.synchronize()
    out["st"] = mrl.read_stats(out["stats"])
    return out


def _oracle_loss(sp, b, mask=None):
    bb = dict(b)
    if mask is not None:
        bb["mask"] = mask
    return util.oracle_loss(bb, b["seq_adv"].cpu().numpy().astype(np.float64), util.cfg_dict(sp))


def test_all_masked_input(mrl, synth):
    sp, b = _small(synth)
    mask = torch.zeros_like(b["mask"]).reshape(-1)
    dW = torch.full((b["V"], b["d"]), 7.0, dtype=torch.float32, device="cuda")
    out = _gpu_loss(mrl, sp, b, mask=mask, out_dW=dW)
    assert out["st"]["n_scored_tokens"] == 0 and out["st"]["loss_total"] == 0.0
    assert torch.all(out["logp"] == 0) and torch.all(out["dH"] == 0)
    assert torch.all(out["dW"] == 0)            # overwrite mode clears dW even without rows


def test_single_scored_token(mrl, synth):
    sp, b = _small(synth)
    mask = torch.zeros_like(b["mask"])
    mask[1, 3] = 1
    out = _gpu_loss(mrl, sp, b, mask=mask.reshape(-1))
    want = _oracle_loss(sp, b, mask=mask)
    n = 1 * b["T"] + 3
    assert abs(out["logp"][n].item() - want["logp"][n]) <= util.LOGP_TOL
    assert out["st"]["n_scored_tokens"] == 1
    assert util.rel_fro(util.to_f64(out["dH"]), want["dH"]) <= util.REL_TOL
    assert util.rel_fro(util.to_f64(out["dW"]), want["dW"]) <= util.REL_TOL


def test_bad_targets_are_treated_as_masked(mrl, synth):
    sp, b = _small(synth)
    targets = b["targets"].clone()
    m = b["mask"].reshape(-1).bool()
    idx = torch.nonzero(m)[:, 0][[2, 17, 40]]
    targets[idx[0]] = -1
    targets[idx[1]] = b["V"]
    targets[idx[2]] = 2 ** 30
    out = _gpu_loss(mrl, sp, b, targets=targets)
    mask2 = b["mask"].clone().reshape(-1)
    mask2[idx] = 0
    bb = dict(b)
    bb["targets"] = torch.where(mask2.bool(), targets, torch.zeros_like(targets))
    want = util.oracle_loss(dict(bb, mask=mask2.reshape(b["B"], b["T"])), b["seq_adv"].cpu().numpy().astype(np.float64),
                            util.cfg_dict(sp))
    assert out["st"]["n_bad_targets"] == 3
    assert out["st"]["n_scored_tokens"] == int(mask2.sum())
    assert torch.all(out["logp"][idx] == 0) and torch.all(out["dH"][idx] == 0)
    mm = mask2.cpu().numpy().astype(bool)
    assert np.max(np.abs(out["logp"].cpu().numpy()[mm] - want["logp"][mm])) <= util.LOGP_TOL
    assert util.rel_fro(util.to_f64(out["dW"]), want["dW"]) <= util.REL_TOL


def test_debug_sync_turns_range_counters_into_error_codes(mrl, synth):
    """The synchronous debugging mode of the loss call: a scored slot with a target id outside
    [0, V) returns MRL_ERR_TARGET_RANGE (-4), a sequence with a group id outside [0, G)
    MRL_ERR_GROUP_RANGE (-5), clean inputs run as usual and give the same bits as the asynchronous
    mode."""
    sp, b = _small(synth)
    clean = _gpu_loss(mrl, sp, b, cfg=dict(debug_sync=1))
    ref = _gpu_loss(mrl, sp, b)
    assert torch.equal(clean["logp"], ref["logp"]) and torch.equal(clean["dW"], ref["dW"])
    targets = b["targets"].clone()
    first = torch.nonzero(b["mask"].reshape(-1))[0, 0]
    targets[first] = b["V"] + 5
    with pytest.raises(mrl.MrlError) as e:
        _gpu_loss(mrl, sp, b, targets=targets, cfg=dict(debug_sync=1))
    assert e.value.status == -4
    bb = dict(b)
    bb["seq_group"] = b["seq_group"].clone()
    bb["seq_group"][3] = b["G"]
    with pytest.raises(mrl.MrlError) as e:
        _gpu_loss(mrl, sp, bb, cfg=dict(debug_sync=1))
    assert e.value.status == -5
    # the asynchronous mode skips the offenders instead
    out = _gpu_loss(mrl, sp, b, targets=targets)
    assert out["st"]["n_bad_targets"] == 1


def test_accumulate_dw_and_optional_gradients(mrl, synth):
    sp, b = _small(synth)
    base = _gpu_loss(mrl, sp, b)
    start = torch.randn((b["V"], b["d"]), dtype=torch.float32, device="cuda") * 1e-4
    acc = _gpu_loss(mrl, sp, b, out_dW=start.clone(), cfg=dict(accumulate_dw=1))
    assert torch.allclose(acc["dW"], start + base["dW"], rtol=1e-5, atol=1e-9)
    only_h = _gpu_loss(mrl, sp, b, want_dW=False)
    only_w = _gpu_loss(mrl, sp, b, want_dH=False)
    fwd = _gpu_loss(mrl, sp, b, want_dH=False, want_dW=False)
    assert only_h["dW"] is None and torch.equal(only_h["dH"], base["dH"])
    assert only_w["dH"] is None and torch.equal(only_w["dW"], base["dW"])
    assert fwd["dH"] is None and fwd["dW"] is None
    for o in (only_h, only_w, fwd):
        assert o["st"]["loss_total"] == base["st"]["loss_total"]
        assert torch.equal(o["logp"], base["logp"])


def test_runs_are_bit_reproducible(mrl, synth):
    sp, b = _small(synth, n_prompts=3, T=40)
    a = _gpu_loss(mrl, sp, b)
    c = _gpu_loss(mrl, sp, b)
    assert torch.equal(a["logp"], c["logp"]) and torch.equal(a["dH"], c["dH"]) and torch.equal(a["dW"], c["dW"])
    assert a["st"] == c["st"]


def test_dw_with_k_split_tail_is_bit_reproducible_and_accumulates(mrl, synth):
    # V = 151936, d = 1536: the ragged last rows of dW tiles are cut into K slices whose partial tiles a
    # second kernel adds in slice order; two passes, so that the second adds into the first's result
    sp, b = _small(synth, n_prompts=2, T=48, V=151936, d=1536)
    a = _gpu_loss(mrl, sp, b)
    c = _gpu_loss(mrl, sp, b)
    assert int(b["mask"].sum()) > 256 and torch.equal(a["dW"], c["dW"]) and torch.equal(a["dH"], c["dH"])
    one = _gpu_loss(mrl, sp, b, cfg=dict(chunk_rows=512))          # one pass
    scale = float(one["dW"].abs().max())
    assert float((a["dW"] - one["dW"]).abs().max()) <= 1e-5 * scale   # fp32 sums in a different order
    tail = a["dW"][151936 // 256 // 8 * 8 * 256:]                     # the rows of the split tiles
    assert float(tail.abs().max()) > 0


def test_kl_off_without_reference(mrl, synth):
    sp, b = _small(synth)
    lc = mrl.LossConfig(kl_beta=0.0, chunk_rows=256)
    out = mrl.grpo_loss_fwd_bwd(b["H"], b["W"], b["targets"], b["mask"].reshape(-1), b["behav"], None, b["seq_adv"],
                                b["seq_group"], b["seq_kind"], b["B"], b["T"], b["G"], lc)
    torch.cuda.synchronize()
    st = mrl.read_stats(out["stats"])
    want = util.oracle_loss(b, b["seq_adv"].cpu().numpy().astype(np.float64), util.cfg_dict(sp, kl_beta=0.0))
    assert st["loss_kl"] == 0.0
    assert util.rel_fro(util.to_f64(out["dW"]), want["dW"]) <= util.REL_TOL
    with pytest.raises(mrl.MrlError):
        mrl.grpo_loss_fwd_bwd(b["H"], b["W"], b["targets"], b["mask"].reshape(-1), b["behav"], None, b["seq_adv"],
                              b["seq_group"], b["seq_kind"], b["B"], b["T"], b["G"], mrl.LossConfig(kl_beta=0.1))


def test_too_small_hint_is_reported_not_silent(mrl, synth):
    sp, b = _small(synth, n_prompts=4, T=40)
    n_scored = int(b["mask"].sum())
    assert n_scored > 256
    out = _gpu_loss(mrl, sp, b, cfg=dict(scored_rows_hint=200))     # one pass of 256 rows only
    assert out["st"]["n_unprocessed_rows"] == n_scored - 256
    lp = out["logp"].cpu().numpy()
    assert int(np.isnan(lp).sum()) == n_scored - 256
    ok = _gpu_loss(mrl, sp, b, cfg=dict(scored_rows_hint=n_scored))
    assert ok["st"]["n_unprocessed_rows"] == 0 and not torch.isnan(ok["logp"]).any()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_token_logprobs_entry_point(mrl, synth, dtype):
    sp = synth.spec(2, n_prompts=2, T=40, V=2700, d=384, dtype=dtype)
    b = synth.make(sp, "cuda")
    H, W, y = util.to_f64(b["H"]), util.to_f64(b["W"]), b["targets"].cpu().numpy()
    want_lp, want_lse = orc.token_logprobs(H, W, y)
    tol = util.LOGP_TOL if dtype == torch.bfloat16 else util.F32_LOGP_TOL
    lp, lse = mrl.token_logprobs(b["H"], b["W"], b["targets"])                 # mask = NULL: every row
    torch.cuda.synchronize()
    assert np.max(np.abs(lp.cpu().numpy() - want_lp)) <= tol
    assert np.max(np.abs(lse.cpu().numpy() - want_lse)) <= tol
    mask = b["mask"].reshape(-1)
    lp2, lse2 = mrl.token_logprobs(b["H"], b["W"], b["targets"], mask)
    lp3, none = mrl.token_logprobs(b["H"], b["W"], b["targets"], mask, want_lse=False)
    torch.cuda.synchronize()
    m = mask.bool()
    assert none is None and torch.equal(lp2, lp3)
    assert torch.all(lp2[~m] == 0) and torch.all(lse2[~m] == 0)
    assert torch.equal(lp2[m], lp[m]) and torch.equal(lse2[m], lse[m])
    empty = mrl.token_logprobs(b["H"][:0], b["W"], b["targets"][:0])            # N = 0 is a no-op
    assert empty[0].numel() == 0


def test_softmax_normalisation_via_lse(mrl, synth):
    # sum_v exp(z - lse) = 1: check on the device result against fp64 logits of a few rows
    sp = synth.spec(2, n_prompts=1, T=16, V=5000, d=256)
    b = synth.make(sp, "cuda")
    _, lse = mrl.token_logprobs(b["H"], b["W"], b["targets"])
    z = orc.logits(util.to_f64(b["H"][:32]), util.to_f64(b["W"]))
    s = np.exp(z - lse[:32].cpu().numpy().astype(np.float64)[:, None]).sum(axis=1)
    assert np.max(np.abs(s - 1.0)) < 2e-3


ADV_CASES = [
    dict(mode=0), dict(mode=1), dict(mode=2), dict(mode=1, ddof=1), dict(mode=2, ddof=1),
    dict(mode=1, mix_alpha=0.0), dict(mode=0, mix_alpha=0.0), dict(mode=1, eps_norm=1e-3),
    dict(mode=1, mix_alpha=0.2), dict(mode=0, mix_alpha=0.2), dict(mode=2, mix_alpha=0.5),
    dict(mode=1, shift=True), dict(mode=0, mix_alpha=0.2, shift=True), dict(mode=2, shift=True, eps_norm=1e-3),
]


@pytest.mark.parametrize("kw", ADV_CASES)
def test_group_advantages_modes(mrl, kw):
    rng = np.random.default_rng(5)
    G, B = 37, 700
    gid = rng.integers(0, G, B).astype(np.int32)        # interleaved groups of uneven size, some empty/singletons
    gid[:5] = 36                                        # make sure one group exists with known members
    r = (rng.random(B) < 0.3).astype(np.float32)
    st = (rng.random(B) < 0.8).astype(np.uint8)
    sc = (rng.random(B) < 0.7).astype(np.uint8)
    own = (rng.random(B) < 0.5).astype(np.uint8)
    t = lambda a: torch.tensor(a, device="cuda")
    kw, okw = dict(kw), dict(kw)
    if kw.pop("shift", False):      # perturbed per-prompt baseline; the values are an input to both sides
        del okw["shift"]
        shift = (rng.normal(size=G) * 0.3).astype(np.float32)
        kw["baseline_shift"], okw["baseline_shift"] = t(shift), shift.astype(np.float64)
    adv, mean, std, flags = mrl.group_advantages(t(r), t(gid), G, t(st), t(sc), t(own), **kw)
    a_o, m_o, s_o, f_o = orc.group_advantages(r.astype(np.float64), gid, G, st, sc, own, **okw)
    assert np.array_equal(flags.cpu().numpy(), f_o)
    assert np.allclose(mean.cpu().numpy(), m_o, rtol=1e-6, atol=1e-7)
    assert np.allclose(std.cpu().numpy(), s_o, rtol=1e-6, atol=1e-7)
    assert np.allclose(adv.cpu().numpy(), a_o, rtol=3e-6, atol=1e-6)
    assert np.all(adv.cpu().numpy()[sc == 0] == 0)


def test_group_advantages_defaults_and_orphans(mrl):
    # NULL masks = all ones; K = 1 groups give 0; out-of-range group ids get 0 and enter no statistic
    r = torch.tensor([1, 0, 0, 1, 1, 0, 1], dtype=torch.float32, device="cuda")
    gid = torch.tensor([0, 0, 0, 0, 1, 9, -3], dtype=torch.int32, device="cuda")
    adv, mean, std, flags = mrl.group_advantages(r, gid, 3)
    a_o, m_o, s_o, f_o = orc.group_advantages(r.cpu().numpy()[:5].astype(np.float64), gid.cpu().numpy()[:5], 3)
    got = adv.cpu().numpy()
    assert np.allclose(got[:5], a_o, atol=1e-6) and got[4] == 0 and np.all(got[5:] == 0)
    assert np.allclose(mean.cpu().numpy(), m_o) and np.array_equal(flags.cpu().numpy(), f_o)
    # XGRPO mix strictly between 0 and 1 with orphans present
    own = torch.tensor([1, 1, 0, 0, 1, 1, 1], dtype=torch.uint8, device="cuda")
    adv2, *_ = mrl.group_advantages(r, gid, 3, None, own, own, mix_alpha=0.2)
    a2, *_ = orc.group_advantages(r.cpu().numpy()[:5].astype(np.float64), gid.cpu().numpy()[:5], 3, None,
                                  own.cpu().numpy()[:5], own.cpu().numpy()[:5], mix_alpha=0.2)
    assert np.allclose(adv2.cpu().numpy()[:5], a2, atol=1e-6)


def test_mfma_rate_probe(mrl):
    """The diagnostic runs and reports a plausible rate; random operands never beat constant ones by much."""
    const = mrl.probe_mfma_rate(False, 0.05)
    rnd = mrl.probe_mfma_rate(True, 0.05)
    assert 300.0 < const < 2600.0, const
    assert 300.0 < rnd < 2600.0, rnd
    assert rnd < 1.05 * const


@pytest.mark.parametrize("dtype,scale", [(torch.bfloat16, 1.0), (torch.bfloat16, 8.0), (torch.float32, 1.0)])
def test_token_scores_entropy(mrl, synth, dtype, scale):
    """Forward-only scoring pass with the entropy output against the oracle: several vocabulary
    tiles with a ragged last one, masked rows, and a peaked softmax (hidden states scaled by 8)."""
    sp = synth.spec(2, n_prompts=2, T=40, V=2700, d=384, dtype=dtype)
    b = synth.make(sp, "cuda")
    Hs = (b["H"].float() * scale).to(dtype)
    H, W, y = util.to_f64(Hs), util.to_f64(b["W"]), b["targets"].cpu().numpy()
    mask = b["mask"].reshape(-1)
    m = mask.cpu().numpy().astype(bool)
    want_lp, want_lse = orc.token_logprobs(H, W, y, m)
    want_ent = orc.token_entropy(H, W, m)
    tol = util.LOGP_TOL if dtype == torch.bfloat16 else util.F32_LOGP_TOL
    lp, lse, ent = mrl.token_scores(Hs, b["W"], b["targets"], mask)
    torch.cuda.synchronize()
    assert np.max(np.abs(lp.cpu().numpy() - want_lp)) <= tol
    assert np.max(np.abs(lse.cpu().numpy() - want_lse)) <= tol
    assert np.max(np.abs(ent.cpu().numpy() - want_ent)) <= tol
    assert torch.all(ent[~mask.bool()] == 0)
    assert float(ent.max()) <= np.log(sp.V) + 1e-3 and float(ent.min()) >= -1e-3
    # the log-probs are those of the plain entry point, bit for bit
    lp0, lse0 = mrl.token_logprobs(Hs, b["W"], b["targets"], mask)
    lp1, none_lse, none_ent = mrl.token_scores(Hs, b["W"], b["targets"], mask, want_lse=False, want_entropy=False)
    torch.cuda.synchronize()
    assert torch.equal(lp0, lp) and torch.equal(lse0, lse) and torch.equal(lp1, lp)
    assert none_lse is None and none_ent is None
