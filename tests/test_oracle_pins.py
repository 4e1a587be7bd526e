"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each pin is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign or index, transposed
operand, wrong normaliser) fails at least one of them.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import mrl_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CFG = orc.default_config()


def _tiny(seed, B=4, T=5, G=2, V=11, d=6, mask_tail=True, away_from_kinks=True):
    rng = np.random.default_rng(seed)
    N = B * T
    H = rng.normal(size=(N, d))
    W = rng.normal(size=(V, d)) * 0.4
    y = rng.integers(0, V, N)
    m = np.ones((B, T), dtype=bool)
    if mask_tail:
        for b in range(B):
            m[b, rng.integers(2, T + 1):] = False
    logp, _ = orc.token_logprobs(H, W, y)
    delta = rng.normal(size=N) * 0.15
    if away_from_kinks:
        for edge in (np.log(0.8), np.log(1.2)):
            near = np.abs(delta - edge) < 0.02
            delta[near] += 0.05
    behav = logp - delta
    ref = logp + rng.normal(size=N) * 0.1
    gid = np.repeat(np.arange(G), B // G)
    rewards = rng.integers(0, 2, B).astype(np.float64)
    adv, *_ = orc.group_advantages(rewards, gid, G)
    adv = adv + 0.1 * rng.normal(size=B)   # generic non-zero advantages
    return dict(H=H, W=W, y=y, m=m, behav=behav, ref=ref, adv=adv, gid=gid, B=B, T=T, G=G,
                V=V, d=d, logp=logp)


def _run(t, cfg=CFG, seq_kind=None, **over):
    a = dict(t)
    a.update(over)
    return orc.grpo_loss_fwd_bwd(a["H"], a["W"], a["y"], a["m"], a["behav"], a["ref"], a["adv"],
                                 a["gid"], seq_kind, a["B"], a["T"], a["G"], cfg)


# ---------------------------------------------------------------- P1 / P9 (forward)
def test_softmax_normalised_and_matches_library():
    rng = np.random.default_rng(1)
    z = rng.normal(size=(7, 33)) * 5.0
    logp, lse = orc.log_softmax(z)
    assert np.allclose(np.exp(logp).sum(axis=1), 1.0, atol=1e-12)
    assert np.all(logp <= 0)
    assert np.allclose(lse, scipy.special.logsumexp(z, axis=1), rtol=0, atol=1e-12)
    assert np.allclose(logp, scipy.special.log_softmax(z, axis=1), atol=1e-12)


def test_lse_is_shift_invariant_and_stable_for_large_logits():
    z = np.array([[1000.0, 999.0, 998.0], [-1000.0, -1001.0, -1002.0]])
    logp, lse = orc.log_softmax(z)
    ref = np.log(np.sum(np.exp(np.array([0.0, -1.0, -2.0]))))
    assert np.allclose(lse, [1000.0 + ref, -1000.0 + ref], atol=1e-10)
    assert np.all(np.isfinite(logp))


def test_logits_orientation_by_explicit_loops():
    # W is [V, d]: z[n, v] = sum_k H[n, k] W[v, k]; a transposed operand fails here.
    rng = np.random.default_rng(2)
    H = rng.normal(size=(3, 4))
    W = rng.normal(size=(5, 4))
    z = orc.logits(H, W)
    for n in range(3):
        for v in range(5):
            assert abs(z[n, v] - sum(H[n, k] * W[v, k] for k in range(4))) < 1e-13


def test_token_logprobs_gathers_target_and_masks():
    rng = np.random.default_rng(3)
    H = rng.normal(size=(6, 4))
    W = rng.normal(size=(9, 4))
    y = np.array([0, 8, 3, 3, 1, 7])
    mask = np.array([1, 1, 0, 1, 1, 0], dtype=np.uint8)
    logp, lse = orc.token_logprobs(H, W, y, mask)
    full = scipy.special.log_softmax(H @ W.T, axis=1)
    for n in range(6):
        if mask[n]:
            assert abs(logp[n] - full[n, y[n]]) < 1e-12
        else:
            assert logp[n] == 0.0 and lse[n] == 0.0


def test_uniform_logits_give_minus_log_V():
    H = np.zeros((2, 3))
    W = np.ones((17, 3))
    logp, lse = orc.token_logprobs(H, W, [4, 9])
    assert np.allclose(logp, -np.log(17.0))
    assert np.allclose(lse, np.log(17.0))


# ---------------------------------------------------------------- P2 advantages
def _read_worked():
    rows = []
    for line in open(os.path.join(GOLDEN, "worked_advantages.txt")):
        if line.startswith("#") or not line.strip():
            continue
        r, c, z = [np.array(part.split(), dtype=np.float64) for part in line.split("|")]
        rows.append((r, c, z))
    return rows


def test_worked_advantage_examples():
    for r, centred, zn in _read_worked():
        gid = np.zeros(r.size, dtype=np.int64)
        a, mean, std, _ = orc.group_advantages(r, gid, 1, mode=orc.ADV_CENTER)
        assert np.allclose(a, centred, atol=1e-15)
        a, mean, std, _ = orc.group_advantages(r, gid, 1, mode=orc.ADV_GROUP_ZN, eps_norm=0.0)
        assert np.allclose(a, zn, atol=1e-14)
        assert abs(mean[0] - r.mean()) < 1e-15


@pytest.mark.parametrize("mode", [orc.ADV_CENTER, orc.ADV_GROUP_ZN, orc.ADV_BATCH_ZN])
@pytest.mark.parametrize("ddof", [0, 1])
def test_advantages_zero_mean_per_group(mode, ddof):
    rng = np.random.default_rng(4)
    G, K = 6, 8
    r = (rng.random(G * K) < 0.3).astype(np.float64)
    gid = rng.permutation(np.repeat(np.arange(G), K))   # interleaved groups
    a, mean, std, _ = orc.group_advantages(r, gid, G, mode=mode, ddof=ddof)
    for g in range(G):
        assert abs(a[gid == g].sum()) < 1e-12
        assert abs(mean[g] - r[gid == g].mean()) < 1e-15
        assert abs(std[g] - np.std(r[gid == g], ddof=ddof)) < 1e-14


def test_group_zn_second_moment_closed_form():
    rng = np.random.default_rng(5)
    K, eps = 8, 1e-3
    r = rng.random(K)
    a, _, std, _ = orc.group_advantages(r, np.zeros(K, dtype=int), 1, eps_norm=eps)
    sigma = np.std(r)
    assert abs(np.sum(a ** 2) - K * sigma ** 2 / (sigma + eps) ** 2) < 1e-12


def test_all_equal_group_gives_exact_zero():
    for val in (0.0, 1.0):
        a, _, std, _ = orc.group_advantages(np.full(8, val), np.zeros(8, dtype=int), 1)
        assert np.all(a == 0.0) and std[0] == 0.0


def test_batch_zn_rescales_centred_advantages_to_unit_batch_variance():
    rng = np.random.default_rng(6)
    G, K = 5, 5
    r = (rng.random(G * K) < 0.4).astype(np.float64)
    gid = np.repeat(np.arange(G), K)
    c, *_ = orc.group_advantages(r, gid, G, mode=orc.ADV_CENTER)
    b, *_ = orc.group_advantages(r, gid, G, mode=orc.ADV_BATCH_ZN, eps_norm=0.0)
    assert abs(np.std(b) - 1.0) < 1e-12
    assert np.allclose(b * np.std(c), c, atol=1e-12)


def test_unscored_members_enter_stats_but_get_zero_advantage():
    # XGRPO (App. I.1): the peers' rewards only shift the baseline.
    r = np.array([0, 0, 1, 0, 1, 1, 1, 0], dtype=np.float64)
    gid = np.zeros(8, dtype=int)
    own = np.array([1, 1, 1, 1, 0, 0, 0, 0], dtype=np.uint8)
    a, mean, std, _ = orc.group_advantages(r, gid, 1, in_stats=np.ones(8, np.uint8), scored=own,
                                           is_own=own, eps_norm=0.0)
    assert mean[0] == 0.5 and std[0] == 0.5
    assert np.allclose(a, [-1, -1, 1, -1, 0, 0, 0, 0])
    a0, *_ = orc.group_advantages(r, gid, 1, in_stats=np.ones(8, np.uint8), scored=own,
                                  is_own=own, eps_norm=0.0, mix_alpha=0.0)
    own_ref, *_ = orc.group_advantages(r[:4], gid[:4], 1, eps_norm=0.0)
    assert np.allclose(a0[:4], own_ref)


# ---------------------------------------------------------------- mixing rule and perturbed baseline
def _mixed_groups(seed, G=5, K=4, peers=6):
    rng = np.random.default_rng(seed)
    r, gid, own = [], [], []
    for g in range(G):
        r += list(rng.random(K + peers))
        gid += [g] * (K + peers)
        own += [1] * K + [0] * peers
    perm = rng.permutation(len(r))
    return (np.array(r)[perm], np.array(gid)[perm], np.array(own, dtype=np.uint8)[perm], G)


@pytest.mark.parametrize("mode", [orc.ADV_CENTER, orc.ADV_GROUP_ZN])
def test_mix_alpha_is_the_linear_blend_of_local_and_pooled_advantages(mode):
    # Sec. 5.2: the local group-relative advantage is combined with its pool-aggregated
    # counterpart; App. A gives the cross-model factor.  Endpoints against scipy's z-score
    # on the own / pooled rewards, linearity in alpha in between, and the centred closed
    # form r - ((1 - alpha) mean_own + alpha mean_pool).
    import scipy.stats
    r, gid, own, G = _mixed_groups(21)
    ones = np.ones(r.size, np.uint8)
    kw = dict(in_stats=ones, scored=own, is_own=own, mode=mode, eps_norm=0.0)
    a0, *_ = orc.group_advantages(r, gid, G, mix_alpha=0.0, **kw)
    a1, *_ = orc.group_advantages(r, gid, G, mix_alpha=1.0, **kw)
    for g in range(G):
        o = (gid == g) & (own == 1)
        allm = gid == g
        if mode == orc.ADV_GROUP_ZN:
            assert np.allclose(a0[o], scipy.stats.zscore(r[o]), atol=1e-12)
            assert np.allclose(a1[allm], np.where(own[allm] == 1, scipy.stats.zscore(r[allm]), 0.0), atol=1e-12)
        else:
            assert np.allclose(a0[o], r[o] - r[o].mean(), atol=1e-14)
            assert np.allclose(a1[o], r[o] - r[allm].mean(), atol=1e-14)
    for alpha in (0.2, 0.5, 0.85):
        a, *_ = orc.group_advantages(r, gid, G, mix_alpha=alpha, **kw)
        assert np.allclose(a - a0, alpha * (a1 - a0), atol=1e-13)
        assert np.all(a[own == 0] == 0.0)
        if mode == orc.ADV_CENTER:
            for g in range(G):
                o = (gid == g) & (own == 1)
                base = (1 - alpha) * r[o].mean() + alpha * r[gid == g].mean()
                assert np.allclose(a[o], r[o] - base, atol=1e-14)
    # own advantages under the blend no longer sum to zero once the pool mean differs
    a, *_ = orc.group_advantages(r, gid, G, mix_alpha=0.2, **kw)
    assert max(abs(a[(gid == g) & (own == 1)].sum()) for g in range(G)) > 1e-3


def test_baseline_shift_closed_form():
    # App. C.4 control: a perturbation d_g of the per-prompt baseline moves every scored
    # advantage of the group by -d_g (centred) or -d_g / (std_g + eps) (z-normalised); the
    # reported statistics and the gate flags do not move.
    r, gid, own, G = _mixed_groups(22)
    ones = np.ones(r.size, np.uint8)
    shift = np.array([0.3, -0.2, 0.0, 1.5, -0.05])
    for alpha in (1.0, 0.2):
        for mode, eps in ((orc.ADV_CENTER, 1e-6), (orc.ADV_GROUP_ZN, 1e-3)):
            kw = dict(in_stats=ones, scored=own, is_own=own, mode=mode, eps_norm=eps, mix_alpha=alpha)
            a, mean, std, fl = orc.group_advantages(r, gid, G, **kw)
            b, mean2, std2, fl2 = orc.group_advantages(r, gid, G, baseline_shift=shift, **kw)
            assert np.array_equal(mean, mean2) and np.array_equal(std, std2) and np.array_equal(fl, fl2)
            for g in range(G):
                o = (gid == g) & (own == 1)
                if mode == orc.ADV_CENTER:
                    want = -shift[g]
                else:
                    sd_o = np.std(r[o])
                    want = -shift[g] * ((1 - alpha) / (sd_o + eps) + alpha / (std[g] + eps))
                assert np.allclose(b[o] - a[o], want, atol=1e-12)
            assert np.all(b[own == 0] == 0.0)
    z, *_ = orc.group_advantages(r, gid, G, baseline_shift=np.zeros(G))
    z0, *_ = orc.group_advantages(r, gid, G)
    assert np.array_equal(z, z0)


def test_prompt_level_baseline_leaves_expected_score_gradient_unchanged():
    # Lemma "Prompt-level pooled baselines are unbiased" (App. I): for a softmax bandit
    # with K = 2 rollouts per prompt, enumerate all arm pairs; the expectation of
    # (1/K) sum_i A_i grad log pi(y_i), with centred advantages computed around a baseline
    # moved by any constant, equals the one without the move (exact rationals would give
    # equality; here to rounding).  grad log pi(a) = e_a - pi for softmax logits.
    pi = np.array([0.5, 0.3, 0.2])
    reward = np.array([1.0, 0.0, 0.0])
    peers = np.array([1.0, 1.0, 0.0])           # fixed peer rewards entering the pooled mean

    def expected_grad(shift):
        g = np.zeros(3)
        for y0, y1 in itertools.product(range(3), repeat=2):
            r = np.concatenate([reward[[y0, y1]], peers])
            own = np.array([1, 1, 0, 0, 0], np.uint8)
            # the lemma needs a baseline that does not depend on the sampled responses:
            # pooled statistics over the peers only (in_stats = not own)
            a, *_ = orc.group_advantages(r, np.zeros(5, dtype=int), 1, in_stats=1 - own, scored=own,
                                         is_own=own, mode=orc.ADV_CENTER,
                                         baseline_shift=None if shift is None else np.array([shift]))
            for yi, ai in ((y0, a[0]), (y1, a[1])):
                score = -pi.copy()
                score[yi] += 1.0
                g += pi[y0] * pi[y1] * 0.5 * ai * score
        return g

    g0 = expected_grad(None)
    assert np.linalg.norm(g0) > 0.1
    # without any baseline the expectation is sum_y pi(y) r(y) (e_y - pi)
    plain = sum(pi[y] * reward[y] * (np.eye(3)[y] - pi) for y in range(3))
    assert np.allclose(g0, plain, atol=1e-14)
    for shift in (0.7, -2.0):
        assert np.allclose(expected_grad(shift), g0, atol=1e-14)


def test_pooled_baseline_variance_identity():
    # Thm. "When pooled XGRPO normalization reduces variance" (App. I): for baselines that do not
    # depend on the scored rollout, Var((r - b_pool) s) - Var((r - b_n) s) = H (Delta^2 - 2 D Delta)
    # with H = E|s|^2, b* = E[r |s|^2] / H, D = b_n - b*, Delta = b_n - b_pool.  The advantages come
    # from the oracle (one own rollout per group, the baseline formed by fixed other entries); the
    # expectation over the own rollout is an exact enumeration of a softmax bandit.
    pi = np.array([0.55, 0.25, 0.15, 0.05])
    reward = np.array([1.0, 0.0, 1.0, 0.0])
    score = np.eye(4) - pi                                  # grad log pi(a) = e_a - pi
    sq = np.sum(score ** 2, axis=1)
    H = float(pi @ sq)
    b_star = float(pi @ (reward * sq)) / H
    local = np.array([1.0, 0.0, 0.0, 1.0, 0.0])              # the learner's other rollouts: b_n = 0.4
    peers = np.array([1.0, 1.0, 1.0, 0.0, 1.0, 1.0, 0.0])    # the other policies' rollouts

    def variance(stat_rewards):
        # own rollout y (scored, not in the statistics) + the fixed entries that form the baseline
        first = np.zeros(4)
        second = 0.0
        for y in range(4):
            r = np.concatenate([[reward[y]], stat_rewards])
            scored = np.zeros(r.size, np.uint8); scored[0] = 1
            a, mean, _, _ = orc.group_advantages(r, np.zeros(r.size, dtype=int), 1, in_stats=1 - scored,
                                                 scored=scored, mode=orc.ADV_CENTER)
            assert abs(mean[0] - stat_rewards.mean()) < 1e-15
            first += pi[y] * a[0] * score[y]
            second += pi[y] * a[0] ** 2 * sq[y]
        return second - float(first @ first), first

    var_n, g_n = variance(local)
    var_pool, g_pool = variance(np.concatenate([local, peers]))
    assert np.allclose(g_n, g_pool, atol=1e-15)               # same expected direction (the lemma)
    b_n, b_pool = local.mean(), np.concatenate([local, peers]).mean()
    D, Delta = b_n - b_star, b_n - b_pool
    assert abs(Delta) > 0.1
    assert abs((var_pool - var_n) - H * (Delta ** 2 - 2 * D * Delta)) < 1e-14
    # and the completed square: Var(b) = Var(b*) + H (b - b*)^2
    var_star, _ = variance(np.array([b_star]))
    assert abs(var_n - (var_star + H * D ** 2)) < 1e-14


# ---------------------------------------------------------------- P7 zero-support boundary
def test_zero_support_boundary_sign():
    # Prop. "Zero-support success boundary": learner all-fail, pool holds a
    # success and a failure => pooled z-normalised own advantages are negative;
    # with own-only statistics they vanish.
    K = 5
    r = np.concatenate([np.zeros(K), np.array([1, 0, 0, 0, 0.0])])
    gid = np.zeros(2 * K, dtype=int)
    own = np.concatenate([np.ones(K), np.zeros(K)]).astype(np.uint8)
    a, mean, std, flags = orc.group_advantages(r, gid, 1, in_stats=np.ones(2 * K, np.uint8),
                                               scored=own, is_own=own)
    assert mean[0] > 0
    assert np.all(a[:K] < 0) and np.all(a[K:] == 0)
    expected = (0 - 0.1) / (0.3 + 1e-6)    # mu_pool = 1/10, sigma_pool = sqrt(.1*.9) = .3
    assert np.allclose(a[:K], expected, atol=1e-12)
    a_own, *_ = orc.group_advantages(r, gid, 1, in_stats=own, scored=own, is_own=own)
    assert np.all(a_own == 0)
    assert flags[0] == (orc.FLAG_ALL_FAIL | orc.FLAG_PEER_SUCCESS | orc.FLAG_RESCUE)


# ---------------------------------------------------------------- P8 gate
def test_gate_truth_table_brute_force():
    for K_own, K_peer in [(1, 1), (2, 2), (3, 2), (2, 3)]:
        own = np.array([1] * K_own + [0] * K_peer, dtype=np.uint8)
        gid = np.zeros(K_own + K_peer, dtype=int)
        for bits in itertools.product([0.0, 1.0], repeat=K_own + K_peer):
            r = np.array(bits)
            *_, flags = orc.group_advantages(r, gid, 1, is_own=own)
            all_fail = all(b == 0 for b in bits[:K_own])
            peer = any(b == 1 for b in bits[K_own:])
            want = (1 if all_fail else 0) | (2 if peer else 0) | (4 if (all_fail and peer) else 0)
            assert flags[0] == want


def test_gate_thresholds_are_strict():
    own = np.array([1, 1, 0], dtype=np.uint8)
    gid = np.zeros(3, dtype=int)
    *_, f = orc.group_advantages(np.array([0.2, 0.0, 1.0]), gid, 1, is_own=own)
    assert f[0] == orc.FLAG_PEER_SUCCESS           # 0.2 is not "below 0.2"
    *_, f = orc.group_advantages(np.array([0.1, 0.0, 0.8]), gid, 1, is_own=own)
    assert f[0] == orc.FLAG_ALL_FAIL               # 0.8 is not "above 0.8"


def test_gate_frequency_matches_rescue_probability():
    # Def. "Rescue gate probability": G_n = (1-p_n)^K [1 - prod_m (1-p_m)^K].
    rng = np.random.default_rng(7)
    K, p_n, p_m, trials = 3, 0.3, 0.2, 20000
    r = np.concatenate([(rng.random((trials, K)) < p_n), (rng.random((trials, K)) < p_m)],
                       axis=1).astype(np.float64)
    gid = np.repeat(np.arange(trials), 2 * K)
    own = np.tile(np.array([1] * K + [0] * K, dtype=np.uint8), trials)
    *_, flags = orc.group_advantages(r.reshape(-1), gid, trials, is_own=own)
    freq = np.mean((flags & orc.FLAG_RESCUE) != 0)
    prob = (1 - p_n) ** K * (1 - (1 - p_m) ** K)
    assert abs(freq - prob) < 4 * np.sqrt(prob * (1 - prob) / trials)


# ---------------------------------------------------------------- Eq. 1 aggregation by brute force
def _loss_by_nested_loops(t, res, cfg, kind=None):
    """Eq. (1) / Eq. (2) written as literal nested loops over prompts, rollouts, tokens."""
    B, T, G = t["B"], t["T"], t["G"]
    kind = np.zeros(B, dtype=int) if kind is None else kind
    logp = res["logp"].reshape(B, T)
    beh, ref = t["behav"].reshape(B, T), t["ref"].reshape(B, T)
    groups = [g for g in range(G) if any(t["gid"][b] == g and kind[b] == 0 for b in range(B))]
    total_pg = total_kl = 0.0
    for g in groups:
        rows = [b for b in range(B) if t["gid"][b] == g and kind[b] == 0]
        acc_pg = acc_kl = 0.0
        for b in rows:
            toks = [s for s in range(T) if t["m"][b, s]]
            if not toks:
                continue
            tok_pg = tok_kl = 0.0
            for s in toks:
                w = np.exp(logp[b, s] - beh[b, s])
                A = t["adv"][b]
                clipped = min(max(w, 1 - cfg["clip_eps_low"]), 1 + cfg["clip_eps_high"])
                tok_pg += min(w * A, clipped * A)
                rho = ref[b, s] - logp[b, s]
                tok_kl += np.exp(rho) - rho - 1
            acc_pg += tok_pg / len(toks)
            acc_kl += tok_kl / len(toks)
        total_pg += acc_pg / len(rows)
        total_kl += acc_kl / len(rows)
    pg = -total_pg / len(groups)
    kl = total_kl / len(groups)
    aux = [b for b in range(B) if kind[b] == 1 and t["m"][b].any()]
    sgt = 0.0
    for b in aux:
        toks = [s for s in range(T) if t["m"][b, s]]
        sgt += -sum(logp[b, s] for s in toks) / len(toks)
    sgt = sgt / len(aux) if aux else 0.0
    return pg, kl, sgt


@pytest.mark.parametrize("seed", [10, 11, 12])
def test_loss_matches_nested_loop_form_of_eq1(seed):
    t = _tiny(seed, B=6, T=5, G=3)
    res = _run(t)
    pg, kl, sgt = _loss_by_nested_loops(t, res, CFG)
    assert abs(res["loss_pg"] - pg) < 1e-13
    assert abs(res["loss_kl"] - kl) < 1e-13
    assert abs(res["loss_total"] - (pg + CFG["kl_beta"] * kl)) < 1e-13


def test_sgt_rows_and_eq2_total():
    t = _tiny(13, B=6, T=5, G=3)
    kind = np.array([0, 0, 0, 1, 0, 1])
    res = _run(t, seq_kind=kind)
    pg, kl, sgt = _loss_by_nested_loops(t, res, CFG, kind)
    assert abs(res["loss_sgt"] - sgt) < 1e-13
    assert abs(res["loss_total"] - (pg + CFG["kl_beta"] * kl + CFG["sgt_lambda"] * sgt)) < 1e-13
    # no auxiliary row => pure GRPO (App. A: "the update is pure GRPO")
    assert _run(t)["loss_sgt"] == 0.0


def test_zero_length_row_counts_in_K_but_adds_nothing():
    t = _tiny(14, B=4, T=5, G=2)
    t["m"][1, :] = False
    res = _run(t)
    pg, kl, _ = _loss_by_nested_loops(t, res, CFG)
    assert abs(res["loss_pg"] - pg) < 1e-13
    assert np.all(res["dH"][5:10] == 0)


def test_global_token_mean_aggregation():
    t = _tiny(15)
    cfg = dict(CFG, loss_agg=1)
    res = _run(t, cfg=cfg)
    m = t["m"].reshape(-1)
    w = np.exp(res["logp"] - t["behav"])
    A = np.repeat(t["adv"], t["T"])
    J = np.minimum(w * A, np.clip(w, 0.8, 1.2) * A)
    assert abs(res["loss_pg"] + np.sum(J[m]) / m.sum()) < 1e-13


# ---------------------------------------------------------------- P3 / P4 special cases
def test_on_policy_ratio_one_clip_inactive():
    t = _tiny(20)
    res = _run(t, behav=t["logp"].copy())
    m = t["m"].reshape(-1)
    assert np.allclose(res["ratio"][m], 1.0, atol=1e-15)
    assert res["n_clipped_tokens"] == 0 and res["n_zero_grad_tokens"] == 0
    c = res["c"]
    A = np.repeat(t["adv"], t["T"])
    assert abs(res["loss_pg"] + np.sum(c * A)) < 1e-14
    beta0 = _run(t, cfg=dict(CFG, kl_beta=0.0), behav=t["logp"].copy())
    assert np.allclose(beta0["g"], -c * A, atol=1e-15)
    # with K equal-length rows and centred advantages the surrogate value is 0
    t2 = _tiny(21, mask_tail=False)
    r = np.array([1, 0, 0, 1.0])
    adv, *_ = orc.group_advantages(r, t2["gid"], t2["G"])
    res2 = _run(t2, behav=t2["logp"].copy(), adv=adv)
    assert abs(res2["loss_pg"]) < 1e-14


def test_k3_zero_at_reference_and_quadratic_nearby():
    t = _tiny(22)
    res = _run(t, ref=t["logp"].copy())
    assert abs(res["loss_kl"]) < 1e-15
    g0 = _run(t, ref=t["logp"].copy(), cfg=dict(CFG, kl_beta=0.0))["g"]
    assert np.allclose(res["g"], g0, atol=1e-16)      # no KL gradient at rho = 0
    *_, k3, dk3 = orc.token_terms(np.array([-2.0]), np.array([-2.0]), np.array([-2.0 + 1e-4]),
                                  np.array([1.0]), 0.2, 0.2)
    assert abs(k3[0] - 0.5e-8) < 1e-12 and k3[0] >= 0
    rng = np.random.default_rng(0)
    *_, k3, _ = orc.token_terms(rng.normal(size=100), rng.normal(size=100), rng.normal(size=100),
                                np.ones(100), 0.2, 0.2)
    assert np.all(k3 >= 0)


def test_clip_semantics_by_cases():
    # A > 0: gain is capped at (1+eps) A;  A < 0: loss is floored at (1-eps) A.
    l = np.zeros(4)
    beh = -np.log(np.array([1.5, 0.5, 1.5, 0.5]))     # w = 1.5, 0.5, 1.5, 0.5
    A = np.array([1.0, 1.0, -1.0, -1.0])
    w, s1, s2, J, dJ, _, _ = orc.token_terms(l, beh, None, A, 0.2, 0.2)
    assert np.allclose(w, [1.5, 0.5, 1.5, 0.5])
    assert np.allclose(J, [1.2, 0.5, -1.5, -0.8])
    assert np.allclose(dJ, [0.0, 0.5, -1.5, 0.0])
    assert np.all(np.abs(np.clip(w, 0.8, 1.2)) <= 1.2)   # Thm 3's bound on clipped weights
    # asymmetric band
    _, _, _, J, _, _, _ = orc.token_terms(l, beh, None, A, 0.1, 0.3)
    assert np.allclose(J, [1.3, 0.5, -1.5, -0.9])


def test_clip_statistics_definitions():
    t = _tiny(23, away_from_kinks=True)
    res = _run(t)
    m = t["m"].reshape(-1)
    w = res["ratio"]
    assert res["n_clipped_tokens"] == int(np.sum(m & ((w < 0.8) | (w > 1.2))))
    A = np.repeat(t["adv"], t["T"])
    dead = m & (((w > 1.2) & (A > 0)) | ((w < 0.8) & (A < 0)))
    assert res["n_zero_grad_tokens"] == int(dead.sum())
    assert abs(res["max_ratio"] - w[m].max()) < 1e-15
    assert res["n_scored_tokens"] == int(m.sum())


def test_ratio_and_k3_means_run_over_grpo_tokens_only():
    """mean_ratio, max_ratio, mean_k3 and the clip counts are statistics of the scored tokens of
    GRPO rows (App. E.3, token-ratio table: mean / p99 / clip rate of the importance ratio over the
    response tokens that enter Eq. 1).  Written out as a literal loop with an auxiliary SGT row and
    an empty row in the batch: dividing by all scored tokens, by all slots, or letting the SGT
    row's tokens in would each give a different number."""
    t = _tiny(24, B=6, T=5, G=3)
    kind = np.array([0, 1, 0, 0, 1, 0])
    t["m"][3, :] = False                                   # an empty GRPO row
    t["behav"] = t["behav"] + np.where(np.repeat(kind, t["T"]) == 1, 1.7, 0.0)   # SGT rows would move every statistic
    res = _run(t, seq_kind=kind)
    logp = res["logp"].reshape(t["B"], t["T"])
    beh, ref = t["behav"].reshape(t["B"], t["T"]), t["ref"].reshape(t["B"], t["T"])
    n = 0
    sum_w = sum_k3 = 0.0
    max_w = 0.0
    n_clip = 0
    for b in range(t["B"]):
        if kind[b] != 0:
            continue
        for s in range(t["T"]):
            if not t["m"][b, s]:
                continue
            w = float(np.exp(logp[b, s] - beh[b, s]))
            rho = float(ref[b, s] - logp[b, s])
            n += 1
            sum_w += w
            sum_k3 += np.exp(rho) - rho - 1.0
            max_w = max(max_w, w)
            n_clip += int(w < 0.8 or w > 1.2)
    n_all = int(t["m"].sum())
    assert 0 < n < n_all                                   # the SGT rows hold scored tokens too
    assert abs(res["mean_ratio"] - sum_w / n) < 1e-14
    assert abs(res["mean_k3"] - sum_k3 / n) < 1e-14
    assert abs(res["max_ratio"] - max_w) < 1e-15
    assert res["n_clipped_tokens"] == n_clip
    assert res["n_scored_tokens"] == n_all
    # the wrong denominators are far outside the tolerance above
    assert abs(res["mean_ratio"] - sum_w / n_all) > 1e-3
    assert abs(res["mean_k3"] - sum_k3 / n_all) > 1e-6


# ---------------------------------------------------------------- P5 finite differences
@pytest.mark.parametrize("seed,kind", [(30, None), (31, np.array([0, 0, 0, 1]))])
def test_gradients_by_central_differences(seed, kind):
    t = _tiny(seed, B=4, T=3, G=2, V=7, d=4)
    res = _run(t, seq_kind=kind)
    h = 1e-6

    def loss(H, W):
        return orc.grpo_loss_fwd_bwd(H, W, t["y"], t["m"], t["behav"], t["ref"], t["adv"], t["gid"],
                                     kind, t["B"], t["T"], t["G"], CFG, need_grads=False)["loss_total"]

    for name, X, grad in (("H", t["H"], res["dH"]), ("W", t["W"], res["dW"])):
        num = np.zeros_like(X)
        for idx in np.ndindex(*X.shape):
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += h
            Xm[idx] -= h
            num[idx] = ((loss(Xp, t["W"]) - loss(Xm, t["W"])) if name == "H"
                        else (loss(t["H"], Xp) - loss(t["H"], Xm))) / (2 * h)
        denom = np.linalg.norm(num)
        assert denom > 0
        assert np.linalg.norm(num - grad) / denom < 1e-6, name
        assert np.max(np.abs(num - grad)) < 1e-8, name


# ---------------------------------------------------------------- P9 autograd (independent backward)
def test_gradients_match_autograd():
    t = _tiny(40, B=6, T=4, G=3, V=13, d=5)
    kind = np.array([0, 0, 0, 0, 1, 0])
    res = _run(t, seq_kind=kind)
    H = torch.tensor(t["H"], dtype=torch.float64, requires_grad=True)
    W = torch.tensor(t["W"], dtype=torch.float64, requires_grad=True)
    lp = torch.log_softmax(H @ W.T, dim=1).gather(1, torch.tensor(t["y"])[:, None])[:, 0]
    c = torch.tensor(res["c"])
    cs = torch.tensor(res["c_sgt"])
    A = torch.tensor(np.repeat(t["adv"], t["T"]))
    w = torch.exp(lp - torch.tensor(t["behav"]))
    J = torch.minimum(w * A, torch.clamp(w, 0.8, 1.2) * A)
    rho = torch.tensor(t["ref"]) - lp
    k3 = torch.exp(rho) - rho - 1
    L = -(c * J).sum() + CFG["kl_beta"] * (c * k3).sum() - CFG["sgt_lambda"] * (cs * lp).sum()
    L.backward()
    assert abs(L.item() - res["loss_total"]) < 1e-13
    assert np.allclose(H.grad.numpy(), res["dH"], atol=1e-13)
    assert np.allclose(W.grad.numpy(), res["dW"], atol=1e-13)


# ---------------------------------------------------------------- P6 Prop. 4 bandit
def _read_prop4():
    poly, etas = None, None
    for line in open(os.path.join(GOLDEN, "prop4_bandit.txt")):
        parts = line.split()
        if parts and parts[0] == "inner_product_poly":
            poly = [Fraction(x) for x in parts[1:]]
        if parts and parts[0] == "eta":
            etas = [Fraction(x) for x in parts[1:]]
    return poly, etas


def _bandit_gradient(pi, sampling, A):
    """-dW of the oracle for three length-1 sequences in one group with w = 1,
    beta = 0; seq_adv folds in the sampling weight (c = 1/3 per sequence)."""
    pi = np.array([float(x) for x in pi])
    H = np.ones((3, 1))
    W = np.log(pi)[:, None]
    y = np.arange(3)
    logp, _ = orc.token_logprobs(H, W, y)
    assert np.allclose(np.exp(logp), pi, atol=1e-15)
    adv = 3.0 * np.array([float(s) * float(a) for s, a in zip(sampling, A)])
    cfg = dict(CFG, kl_beta=0.0)
    res = orc.grpo_loss_fwd_bwd(H, W, y, np.ones((3, 1), bool), logp, None, adv,
                                np.zeros(3, dtype=int), None, 3, 1, 1, cfg)
    return -res["dW"][:, 0]


def test_prop4_bandit_gradients_and_inner_product():
    poly, etas = _read_prop4()
    A = [Fraction(2, 3), Fraction(-1, 3), Fraction(-1, 3)]
    for eta in etas:
        pi = [Fraction(1, 3), Fraction(2, 3) - eta, eta]
        mu = [eta, eta, 1 - 2 * eta]
        g_on = _bandit_gradient(pi, pi, A)
        g_naive = _bandit_gradient(pi, mu, A)
        # vectors printed in the proof
        want_on = [Fraction(2, 9), -Fraction(1, 3) * (Fraction(2, 3) - eta), -eta / 3]
        e_mu_A = eta - Fraction(1, 3)
        want_naive = [Fraction(2, 3) * eta - pi[0] * e_mu_A, -eta / 3 - pi[1] * e_mu_A,
                      -(1 - 2 * eta) / 3 - pi[2] * e_mu_A]
        assert np.allclose(g_on, [float(x) for x in want_on], atol=1e-15)
        assert np.allclose(g_naive, [float(x) for x in want_naive], atol=1e-15)
        inner = sum(c * eta ** k for c, k in zip(poly, (3, 2, 1, 0)))
        assert inner < 0
        assert abs(float(np.dot(g_on, g_naive)) - float(inner)) < 1e-15


# ---------------------------------------------------------------- P10 structural invariants
def test_structural_invariants():
    t = _tiny(50, B=6, T=5, G=3)
    res = _run(t)
    assert np.allclose(res["dW"].sum(axis=0), 0.0, atol=1e-15)   # sum_v dz[n, v] = 0
    m = t["m"].reshape(-1)
    assert np.all(res["dH"][~m] == 0) and np.all(res["g"][~m] == 0)
    # masked rows' contents do not matter
    H2 = t["H"].copy()
    H2[~m] = 123.0
    res2 = _run(t, H=H2)
    assert np.allclose(res2["dW"], res["dW"], atol=1e-15) and res2["loss_total"] == res["loss_total"]
    # permuting sequences permutes dH and leaves loss, dW unchanged
    perm = np.array([3, 0, 5, 1, 4, 2])
    T = t["T"]
    rows = (perm[:, None] * T + np.arange(T)[None, :]).reshape(-1)
    res3 = orc.grpo_loss_fwd_bwd(t["H"][rows], t["W"], t["y"][rows], t["m"][perm], t["behav"][rows],
                                 t["ref"][rows], t["adv"][perm], t["gid"][perm], None,
                                 t["B"], T, t["G"], CFG)
    assert abs(res3["loss_total"] - res["loss_total"]) < 1e-14
    assert np.allclose(res3["dW"], res["dW"], atol=1e-14)
    assert np.allclose(res3["dH"], res["dH"][rows], atol=1e-14)


def test_loss_from_logp_agrees_with_full_path():
    t = _tiny(51)
    res = _run(t)
    tail = orc.loss_from_logp(res["logp"], t["m"], t["behav"], t["ref"], t["adv"], t["gid"], None,
                              t["B"], t["T"], t["G"], CFG)
    assert tail["loss_total"] == res["loss_total"]
    dH, dW, dz = orc.head_backward(t["H"], t["W"], t["y"], tail["g"])
    assert np.allclose(dz.sum(axis=1), 0, atol=1e-15)
    assert np.array_equal(dH, res["dH"])


def test_bf16_decode_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x3DCD, 0x7F7F], dtype=np.uint16)
    want = [1.0, -1.0, 3.140625, 0.0, 0.10009765625, 3.3895313892515355e38]
    assert np.array_equal(orc.decode_bf16(bits), np.array(want))
    x = torch.randn(1000, dtype=torch.float32).to(torch.bfloat16)
    assert np.array_equal(orc.decode_bf16(x.view(torch.int16).numpy().view(np.uint16)),
                          x.to(torch.float64).numpy())


# ---------------------------------------------------------------- token entropy
def test_entropy_closed_forms_and_library():
    import scipy.stats
    rng = np.random.default_rng(11)
    # uniform distribution: log V, whatever the common logit is
    H = np.ones((3, 4))
    W = np.tile(rng.normal(size=(1, 4)), (9, 1))
    assert np.allclose(orc.token_entropy(H, W), np.log(9.0), atol=1e-12)
    # two-point distribution with log-odds a: H = log(1 + e^a) - a * sigma(a)
    a = 1.7
    ent = orc.token_entropy(np.array([[1.0]]), np.array([[a], [0.0]]))[0]
    assert abs(ent - (np.log1p(np.exp(a)) - a / (1.0 + np.exp(-a)))) < 1e-12
    # library routine on random rows, and the identity H = lse - E_p[z]
    H = rng.normal(size=(6, 5))
    W = rng.normal(size=(13, 5))
    z = orc.logits(H, W)
    logp, lse = orc.log_softmax(z)
    ent = orc.token_entropy(H, W)
    assert np.allclose(ent, scipy.stats.entropy(np.exp(logp), axis=1), atol=1e-12)
    assert np.allclose(ent, lse - np.sum(np.exp(logp) * z, axis=1), atol=1e-12)
    # a sharply peaked row has entropy near 0, a masked row exactly 0
    W2 = W.copy()
    W2[4] *= 200.0
    ent2 = orc.token_entropy(H, W2, token_mask=[1, 1, 1, 0, 1, 1])
    assert ent2[3] == 0.0 and np.all(ent2 >= 0.0) and ent2.min() < 1e-6
    assert np.all(ent <= np.log(13.0) + 1e-12)


# ---------------------------------------------------------------- response-level ratio (App. I.1)
def _seq_tiny(seed, jitter=0.12):
    """Like _tiny, with jitters such that response-level ratios straddle the clip band."""
    t = _tiny(seed, B=6, T=4, G=3, V=9, d=4)
    rng = np.random.default_rng(seed + 1000)
    t["behav"] = t["logp"] - rng.normal(size=t["logp"].shape) * jitter
    return t


@pytest.mark.parametrize("level", [1, 2])
def test_response_ratio_by_hand_and_autograd(level):
    t = _seq_tiny(50, 0.12 if level == 1 else 0.4)
    cfg = dict(CFG, ratio_level=level)
    kind = np.array([0, 0, 0, 0, 0, 1])
    res = _run(t, cfg=cfg, seq_kind=kind)
    B, T = t["B"], t["T"]
    m = t["m"]
    # literal nested loops: rho_b from the response's summed log-ratio, J_b once per response
    lp = res["logp"].reshape(B, T)
    beh = t["behav"].reshape(B, T)
    K = np.zeros(t["G"])
    for b in range(B):
        if kind[b] == 0:
            K[t["gid"][b]] += 1
    P = np.sum(K > 0)
    total, ratios = 0.0, []
    for b in range(B):
        L = m[b].sum()
        if kind[b] != 0 or L == 0:
            continue
        delta = sum(lp[b, j] - beh[b, j] for j in range(T) if m[b, j])
        rho = np.exp(delta if level == 1 else delta / L)
        ratios.append(rho)
        A = t["adv"][b]
        total += -min(rho * A, min(max(rho, 0.8), 1.2) * A) / (P * K[t["gid"][b]])
    assert abs(res["loss_pg"] - total) < 1e-13
    assert min(ratios) < 0.8 or max(ratios) > 1.2          # the clip is exercised
    # independent backward
    H = torch.tensor(t["H"], dtype=torch.float64, requires_grad=True)
    W = torch.tensor(t["W"], dtype=torch.float64, requires_grad=True)
    lpt = torch.log_softmax(H @ W.T, dim=1).gather(1, torch.tensor(t["y"])[:, None])[:, 0].reshape(B, T)
    mt = torch.tensor(m)
    d = torch.where(mt, lpt - torch.tensor(beh), torch.zeros_like(lpt)).sum(dim=1)
    Lb = mt.sum(dim=1).clamp(min=1).double()
    rho = torch.exp(d if level == 1 else d / Lb)
    A = torch.tensor(t["adv"])
    J = torch.minimum(rho * A, torch.clamp(rho, 0.8, 1.2) * A)
    wseq = torch.tensor([(1.0 / (P * K[t["gid"][b]])) if (kind[b] == 0 and m[b].sum() > 0) else 0.0 for b in range(B)])
    c = torch.tensor(res["c"]).reshape(B, T)
    cs = torch.tensor(res["c_sgt"]).reshape(B, T)
    r = torch.tensor(t["ref"]).reshape(B, T) - lpt
    loss = -(wseq * J).sum() + CFG["kl_beta"] * (c * (torch.exp(r) - r - 1)).sum() - CFG["sgt_lambda"] * (cs * lpt).sum()
    loss.backward()
    assert abs(loss.item() - res["loss_total"]) < 1e-13
    assert np.allclose(H.grad.numpy(), res["dH"], atol=1e-13)
    assert np.allclose(W.grad.numpy(), res["dW"], atol=1e-13)


def test_response_ratio_special_cases():
    t = _seq_tiny(51)
    base = _run(t)
    # one-token responses: the response ratio is the token ratio, all three levels coincide
    one = dict(t)
    one["m"] = np.zeros_like(t["m"])
    one["m"][:, 0] = True
    r0 = _run(one)
    for level in (1, 2):
        r = _run(one, cfg=dict(CFG, ratio_level=level))
        assert abs(r["loss_total"] - r0["loss_total"]) < 1e-15
        assert np.allclose(r["dW"], r0["dW"], atol=1e-15)
    # behaviour trace = current trace: rho = 1, J = A, clip inactive, gradient -A / (P K) per token
    # at level 1 and -A / (P K L) at level 2
    for level in (1, 2):
        r = _run(t, cfg=dict(CFG, ratio_level=level, kl_beta=0.0), behav=base["logp"])
        m = t["m"]
        Kg = np.bincount(t["gid"], minlength=t["G"])
        wseq = 1.0 / (t["G"] * Kg[t["gid"]])
        assert abs(r["loss_pg"] + np.sum(wseq * t["adv"] * (m.sum(axis=1) > 0))) < 1e-14
        assert r["n_clipped_tokens"] == 0
        expect = -(wseq * t["adv"])[:, None] * m / (1.0 if level == 1 else np.maximum(m.sum(axis=1), 1)[:, None])
        assert np.allclose(r["g"].reshape(m.shape), expect, atol=1e-15)
    # the clipped weight never exceeds 1 + eps in magnitude (App. I, proof of the PRP theorem)
    r = _run(t, cfg=dict(CFG, ratio_level=1))
    A = np.repeat(t["adv"], t["T"])
    live = t["m"].reshape(-1) & (np.abs(A) > 0)
    assert np.all(np.abs(r["s2"][live] / A[live]) <= 1.2 + 1e-15)
    with pytest.raises(ValueError):
        _run(t, cfg=dict(CFG, ratio_level=1, loss_agg=1))
