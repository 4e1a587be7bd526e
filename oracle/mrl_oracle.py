"""CPU oracle for the GRPO scoring hot path (TEST INFRASTRUCTURE, not the product).

A plain, slow, fp64 NumPy implementation of what the hot path computes, written
from the paper's definitions.  Everything is materialised (the full N x V logit
and softmax matrices), nothing is blocked, fused or reordered, so each function
can be checked against the equation it cites by eye.

Only tests, the smoke check and the bench's `cpu_baseline` leg may import this
module.  It shares no code with the HIP path and imports nothing from the
package.

Citations are to the paper's sections / equations:
  * Sec. 3 "Preliminaries", GRPO paragraph: token log-probs, importance weights
    w = exp(l_theta - l_old), group-relative advantages, Eq. (1) (the clipped
    surrogate plus beta * R(theta)).
  * Sec. 5.1 (PRP): pool-wide advantage normalisation, behaviour denominator.
  * App. I.1 (XGRPO paragraph): pooled mean / std baseline.
  * Sec. 5.3, Eq. (2), App. B (SGT): gate, auxiliary NLL, lambda weighting.
  * App. I, proof of Prop. 4: grad log pi(a_i) = e_i - pi for a softmax.

Readings of points the paper leaves open (each is listed in the design notes):
  * R(theta) is the k3 estimator exp(rho) - rho - 1, rho = l_ref - l_theta,
    aggregated with the same token weights as the surrogate.
  * std is the population std (ddof = 0) unless ddof = 1 is asked for.
  * E_x (1/K) sum_i E_tok[.] is taken literally: token mean per sequence, then
    mean over the K_g GRPO rows of a group, then mean over the P groups that
    have a GRPO row.
  * gradient indicator at the clip kink is 1[s1 <= s2].

Parity status: every function here is pinned by tests/test_oracle_pins.py
except the XGRPO alpha-mix with alpha strictly between 0 and 1, whose rule the
paper does not print; the blend as read is pinned, the reading is not.
"""
from __future__ import annotations

import numpy as np

ADV_CENTER = 0
ADV_GROUP_ZN = 1
ADV_BATCH_ZN = 2

FLAG_ALL_FAIL = 1
FLAG_PEER_SUCCESS = 2
FLAG_RESCUE = 4


def decode_bf16(bits):
    """Exact fp64 value of bfloat16 bit patterns (uint16 array)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    as_f32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return as_f32.astype(np.float64)


# --------------------------------------------------------------------------
# Sec. 3: token log-probabilities  l_theta[n] = log pi_theta(y_n | context)
# --------------------------------------------------------------------------
def logits(H, W):
    """z[n, v] = sum_k H[n, k] * W[v, k]; no bias, temperature 1."""
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    return np.matmul(H, W.T)


def log_softmax(z):
    """Returns (log p, lse) with lse[n] = log sum_v exp z[n, v], max-subtracted."""
    z = np.asarray(z, dtype=np.float64)
    M = np.max(z, axis=1, keepdims=True)
    lse = M + np.log(np.sum(np.exp(z - M), axis=1, keepdims=True))
    return z - lse, lse[:, 0]


def token_logprobs(H, W, target_ids, token_mask=None):
    """Per-token log-prob of the target id and the row's log-sum-exp.

    Masked rows report 0 for both outputs.
    """
    z = logits(H, W)
    logp_all, lse = log_softmax(z)
    n = np.arange(z.shape[0])
    logp = logp_all[n, np.asarray(target_ids, dtype=np.int64)]
    if token_mask is not None:
        m = np.asarray(token_mask).astype(bool)
        logp = np.where(m, logp, 0.0)
        lse = np.where(m, lse, 0.0)
    return logp, lse


def token_entropy(H, W, token_mask=None):
    """Shannon entropy of the next-token distribution of every row, - sum_v p[n, v] log p[n, v]
    (the per-token quantity behind the entropy traces of Sec. 5, "Optimization Diagnostics").
    Masked rows report 0."""
    logp_all, _ = log_softmax(logits(H, W))
    p = np.exp(logp_all)
    ent = -np.sum(np.where(p > 0.0, p * logp_all, 0.0), axis=1)
    if token_mask is not None:
        ent = np.where(np.asarray(token_mask).astype(bool), ent, 0.0)
    return ent


# --------------------------------------------------------------------------
# Sec. 3 advantages; Sec. 5.1 pool-wide; App. I.1 pooled baseline; SGT gate
# --------------------------------------------------------------------------
def _mean_std(r, ddof):
    k = r.size
    if k == 0:
        return 0.0, 0.0
    mu = float(np.sum(r) / k)
    denom = k - ddof
    if denom <= 0:
        return mu, 0.0
    return mu, float(np.sqrt(np.sum((r - mu) ** 2) / denom))


def group_advantages(rewards, group_id, G, in_stats=None, scored=None, is_own=None,
                     mode=ADV_GROUP_ZN, eps_norm=1e-6, ddof=0, mix_alpha=1.0,
                     neg_thresh=0.2, pos_thresh=0.8, baseline_shift=None):
    """Group-relative advantages and SGT gate flags.

    Stat members of group g are the entries with in_stats = 1; their rewards
    form rbar and std (Sec. 3).  PRP puts own and peer rollouts in the same
    group with in_stats = scored = 1 (Sec. 5.1); XGRPO adds the peers' rewards
    with in_stats = 1, scored = 0, which makes rbar, std the pooled statistics
    of App. I.1.  Entries with scored = 0 get advantage 0.

    mix_alpha blends own-only statistics (stat members that are also is_own)
    with the pooled ones: A = (1 - alpha) * A_own + alpha * A_pool.  alpha = 1
    is the pooled rule of App. I.1, alpha = 0 plain per-policy GRPO.

    baseline_shift[g] (optional) is added to the per-prompt baseline of group g
    (its pooled and its own-only mean alike) before the rewards are centred; the
    standard deviations stay those of the unshifted rewards.  This is the
    perturbed-baseline control of App. C.4 ("Ablation: shared normalization for
    XGRPO"); the perturbation values are an input.

    Flags per group (Sec. 5.3 gate, thresholds from App. A):
      bit0 all_fail    : every is_own entry has reward < neg_thresh (and one exists)
      bit1 peer_success: some non-own entry has reward > pos_thresh
      bit2 rescue      : bit0 and bit1
    Returns (adv[B], mean[G], std[G], flags[G] uint8); mean/std are the pooled ones.
    """
    r = np.asarray(rewards, dtype=np.float64)
    gid = np.asarray(group_id, dtype=np.int64)
    B = r.size
    ones = np.ones(B, dtype=bool)
    st = ones if in_stats is None else np.asarray(in_stats).astype(bool)
    sc = ones if scored is None else np.asarray(scored).astype(bool)
    own = ones if is_own is None else np.asarray(is_own).astype(bool)
    if np.any(gid < 0) or np.any(gid >= G):
        raise ValueError("group id out of range")

    adv = np.zeros(B)
    mean = np.zeros(G)
    std = np.zeros(G)
    flags = np.zeros(G, dtype=np.uint8)
    shift = np.zeros(G) if baseline_shift is None else np.asarray(baseline_shift, dtype=np.float64)

    def normalise(x, mu, sd):
        if mode == ADV_GROUP_ZN:
            return (x - mu) / (sd + eps_norm)
        return x - mu

    for g in range(G):
        members = np.nonzero(gid == g)[0]
        pool = members[st[members]]
        mu_p, sd_p = _mean_std(r[pool], ddof)
        mean[g], std[g] = mu_p, sd_p
        own_pool = pool[own[pool]]
        mu_o, sd_o = _mean_std(r[own_pool], ddof)
        for b in members:
            if not sc[b]:
                continue
            a_pool = normalise(r[b], mu_p + shift[g], sd_p) if pool.size else 0.0
            if mix_alpha == 1.0:
                adv[b] = a_pool
            else:
                a_own = normalise(r[b], mu_o + shift[g], sd_o) if own_pool.size else 0.0
                adv[b] = (1.0 - mix_alpha) * a_own + mix_alpha * a_pool
        own_m = members[own[members]]
        peer_m = members[~own[members]]
        all_fail = own_m.size > 0 and bool(np.all(r[own_m] < neg_thresh))
        peer_succ = bool(np.any(r[peer_m] > pos_thresh))
        flags[g] = (FLAG_ALL_FAIL * all_fail) | (FLAG_PEER_SUCCESS * peer_succ) | \
                   (FLAG_RESCUE * (all_fail and peer_succ))

    if mode == ADV_BATCH_ZN:
        # App. A: subtract the group mean, then unit variance across the batch.
        vals = adv[sc]
        _, sd_b = _mean_std(vals, ddof)
        adv = np.where(sc, adv / (sd_b + eps_norm), 0.0)
    return adv, mean, std, flags


# --------------------------------------------------------------------------
# Eq. (1) aggregation weights:  E_x (1/K) sum_i E_tok[.]
# --------------------------------------------------------------------------
def sequence_weights(token_mask, group_id, seq_kind, G, loss_agg=0):
    """Per-token weights c (GRPO rows) and c_sgt (auxiliary rows), shape [B, T].

    GRPO rows (seq_kind 0): c[b, t] = m[b, t] / (P * K_g * L_b) with L_b the
    number of scored tokens of the row, K_g the number of GRPO rows of its
    group and P the number of groups that have a GRPO row.  A row with L_b = 0
    contributes nothing but still counts in K_g.  loss_agg = 1 replaces this by
    one mean over all scored GRPO tokens.
    SGT rows (seq_kind 1): c_sgt[b, t] = m[b, t] / (S_aux * L_b), S_aux the
    number of auxiliary rows with L_b > 0 (token mean per example, then mean
    over gated examples; App. B).
    """
    m = np.asarray(token_mask).astype(np.float64)
    B, T = m.shape
    gid = np.asarray(group_id, dtype=np.int64)
    kind = np.zeros(B, dtype=np.int64) if seq_kind is None else np.asarray(seq_kind, dtype=np.int64)
    L = m.sum(axis=1)
    is_grpo = kind == 0
    K = np.zeros(G)
    for b in range(B):
        if is_grpo[b]:
            K[gid[b]] += 1
    P = float(np.sum(K > 0))
    c = np.zeros((B, T))
    c_sgt = np.zeros((B, T))
    n_grpo_tokens = float(np.sum(L[is_grpo]))
    S_aux = float(np.sum((~is_grpo) & (L > 0)))
    for b in range(B):
        if L[b] == 0:
            continue
        if is_grpo[b]:
            if loss_agg == 1:
                c[b] = m[b] / n_grpo_tokens
            else:
                c[b] = m[b] / (P * K[gid[b]] * L[b])
        else:
            c_sgt[b] = m[b] / (S_aux * L[b])
    return c, c_sgt


# --------------------------------------------------------------------------
# Eq. (1) token terms and their derivative with respect to l_theta
# --------------------------------------------------------------------------
def token_terms(logp, behav_logp, ref_logp, adv_tok, eps_lo, eps_hi):
    """Importance ratio, clipped surrogate J, k3 KL and dJ/dl, dk3/dl per token.

    w = exp(l - l_beh); s1 = w A; s2 = clip(w, 1 - eps_lo, 1 + eps_hi) A;
    J = min(s1, s2)  (Eq. 1).  k3 = exp(rho) - rho - 1 with rho = l_ref - l.
    The behaviour trace, the reference trace and A are constants (Sec. 3: the
    behaviour policy is not differentiated).
    """
    l = np.asarray(logp, dtype=np.float64)
    w = np.exp(l - np.asarray(behav_logp, dtype=np.float64))
    A = np.asarray(adv_tok, dtype=np.float64)
    s1 = w * A
    s2 = np.minimum(np.maximum(w, 1.0 - eps_lo), 1.0 + eps_hi) * A
    J = np.minimum(s1, s2)
    dJ = np.where(s1 <= s2, w * A, 0.0)
    if ref_logp is None:
        k3 = np.zeros_like(l)
        dk3 = np.zeros_like(l)
    else:
        rho = np.asarray(ref_logp, dtype=np.float64) - l
        k3 = np.exp(rho) - rho - 1.0
        dk3 = 1.0 - np.exp(rho)
    return w, s1, s2, J, dJ, k3, dk3


def default_config():
    return dict(clip_eps_low=0.2, clip_eps_high=0.2, kl_beta=0.04, sgt_lambda=0.1, loss_agg=0)


def loss_from_logp(logp, token_mask, behav_logp, ref_logp, seq_adv, group_id, seq_kind,
                   B, T, G, cfg):
    """The O(N) part of the step for given token log-probs l (shape [B*T]).

    L = L_pg + beta * L_kl + lambda * L_sgt  (Eq. 1 and Eq. 2) with
      L_pg  = - sum c * J,  L_kl = sum c * k3,  L_sgt = - sum c_sgt * l.
    g = dL/dl = c * (-dJ + beta * dk3) on GRPO rows, -lambda * c_sgt on SGT rows.
    Statistics: a token is "clipped" when its ratio lies outside
    [1 - eps_lo, 1 + eps_hi] (App. E.3, token-ratio table caption); it has zero
    surrogate gradient when s2 < s1.  Means run over scored GRPO tokens.

    cfg["ratio_level"] (default 0 = the token ratio of Eq. 1) selects the response-level ratio
    of App. I.1 instead: 1 = exp of the summed log-ratio, 2 = exp of its per-token mean (the
    magnitudes of App. E.3's sequence-ratio table, medians 0.75-0.91 over whole responses, are
    those of a per-token mean).  The KL term stays per token.  Statistics then use the
    response's ratio for each of its tokens.
    """
    N = B * T
    m = np.asarray(token_mask).astype(bool).reshape(B, T)
    kind = np.zeros(B, dtype=np.int64) if seq_kind is None else np.asarray(seq_kind, dtype=np.int64)
    c, c_sgt = sequence_weights(m, group_id, kind, G, cfg.get("loss_agg", 0))
    c, c_sgt = c.reshape(N), c_sgt.reshape(N)
    mflat = m.reshape(N)
    adv_tok = np.repeat(np.asarray(seq_adv, dtype=np.float64), T)
    l = np.where(mflat, np.asarray(logp, dtype=np.float64).reshape(N), 0.0)
    beh = np.where(mflat, np.asarray(behav_logp, dtype=np.float64).reshape(N), 0.0)
    ref = None if ref_logp is None else \
        np.where(mflat, np.asarray(ref_logp, dtype=np.float64).reshape(N), 0.0)
    w, s1, s2, J, dJ, k3, dk3 = token_terms(l, beh, ref, adv_tok,
                                            cfg["clip_eps_low"], cfg["clip_eps_high"])
    level = int(cfg.get("ratio_level", 0))
    if level != 0:
        # Response-level ratio of App. I.1: rho_b = exp{L_theta - L_behavior} with the sums over the
        # response's scored tokens (level 1), or their per-token mean (level 2); it takes the place
        # of the token ratio in Eq. (1).  Every token of a response then carries the response's J,
        # so E_tok[J] = J_b, and d rho_b / d l_t = rho_b (level 1) or rho_b / L_b (level 2).
        if cfg.get("loss_agg", 0) != 0:
            raise ValueError("the response-level ratio is defined for the Eq. (1) aggregation only")
        L_b = m.sum(axis=1).astype(np.float64)
        delta = np.where(mflat, l - beh, 0.0).reshape(B, T).sum(axis=1)
        expo = delta if level == 1 else np.where(L_b > 0, delta / np.maximum(L_b, 1.0), 0.0)
        rho_tok = np.repeat(np.exp(expo), T)
        A = adv_tok
        w = rho_tok
        s1 = w * A
        s2 = np.minimum(np.maximum(w, 1.0 - cfg["clip_eps_low"]), 1.0 + cfg["clip_eps_high"]) * A
        J = np.minimum(s1, s2)
        scale = np.repeat(L_b, T) if level == 1 else 1.0
        dJ = np.where(s1 <= s2, w * A, 0.0) * scale
    beta, lam = float(cfg["kl_beta"]), float(cfg["sgt_lambda"])
    loss_pg = -float(np.sum(c * J))
    loss_kl = float(np.sum(c * k3))
    loss_sgt = -float(np.sum(c_sgt * l))
    g = c * (-dJ + beta * dk3) - lam * c_sgt

    grpo_tok = mflat & np.repeat(kind == 0, T)
    n_grpo = int(np.sum(grpo_tok))
    lo, hi = 1.0 - cfg["clip_eps_low"], 1.0 + cfg["clip_eps_high"]
    return dict(
        loss_total=loss_pg + beta * loss_kl + lam * loss_sgt,
        loss_pg=loss_pg, loss_kl=loss_kl, loss_sgt=loss_sgt,
        n_scored_tokens=int(np.sum(mflat)),
        n_clipped_tokens=int(np.sum(grpo_tok & ((w < lo) | (w > hi)))),
        n_zero_grad_tokens=int(np.sum(grpo_tok & (s2 < s1))),
        mean_ratio=float(np.sum(w[grpo_tok]) / n_grpo) if n_grpo else 0.0,
        max_ratio=float(np.max(w[grpo_tok])) if n_grpo else 0.0,
        mean_k3=float(np.sum(k3[grpo_tok]) / n_grpo) if n_grpo else 0.0,
        g=g, ratio=w, s1=s1, s2=s2, c=c, c_sgt=c_sgt, grpo_tok=grpo_tok)


def head_backward(H, W, target_ids, g):
    """Back-propagation of g = dL/dl through log-softmax and the LM head.

    dz[n, v] = g[n] * (1[v = y_n] - p[n, v])  (score of a softmax: e_i - pi,
    proof of Prop. 4);  dH = dz W;  dW = dz^T H.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    y = np.asarray(target_ids, dtype=np.int64)
    g = np.asarray(g, dtype=np.float64)
    logp_all, _ = log_softmax(logits(H, W))
    dz = -g[:, None] * np.exp(logp_all)
    dz[np.arange(H.shape[0]), y] += g
    return np.matmul(dz, W), np.matmul(dz.T, H), dz


def grpo_loss_fwd_bwd(H, W, target_ids, token_mask, behav_logp, ref_logp, seq_adv,
                      group_id, seq_kind, B, T, G, cfg, need_grads=True):
    """Forward and backward of the whole scoring step: token_logprobs, then
    loss_from_logp, then head_backward.  Returns the union of their results."""
    N = B * T
    y = np.asarray(target_ids, dtype=np.int64).reshape(N)
    mflat = np.asarray(token_mask).astype(bool).reshape(N)
    logp, lse = token_logprobs(H, W, y, mflat)
    out = loss_from_logp(logp, mflat, behav_logp, ref_logp, seq_adv, group_id, seq_kind,
                         B, T, G, cfg)
    out["logp"], out["lse"] = logp, lse
    if need_grads:
        out["dH"], out["dW"], _ = head_backward(H, W, y, out["g"])
    return out
