"""Seeded synthetic workloads with the shapes and value distributions of the
benchmark configurations (stand-ins for rollouts on the paper's MATH / QA
prompts, which are not available here).

This module only draws inputs.  It contains none of the scoring arithmetic and
imports neither the HIP binding nor the CPU oracle; both sides receive the same
tensors.  The behaviour / reference traces are centred on a closed-form proxy
of the current log-prob (see `logp_proxy`) plus Gaussian jitter, so that the
importance ratios have the spread each configuration asks for without running
either implementation to produce inputs.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch

SEED_BASE = 20260507 * 10
W_STD = 0.02


@dataclass
class Spec:
    name: str
    V: int
    d: int
    n_prompts: int
    k_own: int
    T: int
    dtype: torch.dtype = torch.bfloat16
    k_peer: int = 0                 # pooled peer rollouts per prompt (PRP, scored)
    k_peer_rewards: int = 0         # peer reward-only entries per prompt (XGRPO pool, unscored)
    len_dist: str = "uniform"       # "uniform" in [T/4, T] | "loguniform" in [T/16, T] | "tail" | "full"
    reward_p: float = 0.25
    old_jitter: float = 0.1
    peer_jitter: float = 0.5
    ref_jitter: float = 0.1
    frac_all_fail: float = 0.0      # SGT: share of prompts forced to all-zero own reward
    clip_eps: float = 0.2
    kl_beta: float = 0.04
    sgt_lambda: float = 0.1
    index: int = 0
    extra: dict = field(default_factory=dict)


def spec(index: int, **over) -> Spec:
    """The five benchmark configurations (index 1..5); keyword overrides shrink them."""
    base = {
        1: Spec("tiny-fp32", 512, 64, 2, 4, 32, dtype=torch.float32, len_dist="tail", reward_p=0.3,
                old_jitter=0.05, ref_jitter=0.1),
        2: Spec("qwen-like", 151936, 1536, 32, 8, 1024, len_dist="uniform", reward_p=0.25),
        3: Spec("llama-like-prp", 128256, 2048, 32, 8, 1536, k_peer=8, len_dist="prp", reward_p=0.3),
        4: Spec("xgrpo-sgt", 151936, 3584, 64, 8, 2048, k_peer_rewards=8, len_dist="uniform", reward_p=0.3,
                frac_all_fail=0.2),
        5: Spec("large-vocab-stress", 151936, 4096, 128, 8, 2048, len_dist="loguniform", reward_p=0.2),
    }[index]
    base.index = index
    for k, v in over.items():
        setattr(base, k, v)
    return base


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn_into(out: torch.Tensor, std: float, g, rows_per_chunk: int = 1 << 15):
    """Fills `out` ([rows, cols], any float dtype) with N(0, std) drawn in fp32 and rounded."""
    for r0 in range(0, out.shape[0], rows_per_chunk):
        r1 = min(out.shape[0], r0 + rows_per_chunk)
        blk = torch.randn((r1 - r0, out.shape[1]), dtype=torch.float32, device=out.device, generator=g)
        out[r0:r1] = (blk * std).to(out.dtype)


def logp_proxy(H: torch.Tensor, W: torch.Tensor, targets: torch.Tensor, rows_per_chunk: int = 1 << 15):
    """Closed-form stand-in for the current log-prob of each row, used only to centre
    the synthetic behaviour / reference traces: the target's logit <h, w_y> minus the
    log-partition of V i.i.d. Gaussian logits of variance |h|^2 * W_STD^2, i.e.
    log V + |h|^2 W_STD^2 / 2.  Accurate to a few 1e-3..1e-2 for these random inputs."""
    N = H.shape[0]
    V = W.shape[0]
    out = torch.empty(N, dtype=torch.float32, device=H.device)
    for r0 in range(0, N, rows_per_chunk):
        r1 = min(N, r0 + rows_per_chunk)
        h = H[r0:r1].float()
        wy = W[targets[r0:r1].long()].float()
        zt = (h * wy).sum(dim=1)
        var = (h * h).sum(dim=1) * (W_STD * W_STD)
        out[r0:r1] = zt - (math.log(V) + 0.5 * var)
    return out


def _lengths(sp: Spec, n: int, g, device, kind="own"):
    T = sp.T
    u = torch.rand(n, device=device, generator=g)
    if sp.len_dist == "full":
        return torch.full((n,), T, dtype=torch.int64, device=device)
    if sp.len_dist == "tail":                       # about 10 % of the tail masked
        lo = max(1, int(round(T * 0.8125)))         # 26 of 32
        return (lo + torch.floor(u * (T - lo + 1))).long().clamp(max=T)
    if sp.len_dist == "loguniform":
        lo = max(1.0, T / 16.0)
        return torch.round(torch.exp(math.log(lo) + u * (math.log(T) - math.log(lo)))).long().clamp(1, T)
    if sp.len_dist == "prp" and kind == "peer":
        # source length, then a retokenisation factor in [1.0, 1.3]
        lo, hi = max(1, T // 6), max(1, int(T / 1.3))
        src = lo + torch.floor(u * (hi - lo + 1))
        f = 1.0 + 0.3 * torch.rand(n, device=device, generator=g)
        return torch.round(src * f).long().clamp(1, T)
    lo = max(1, T // 6 if sp.len_dist == "prp" else T // 4)
    return (lo + torch.floor(u * (T - lo + 1))).long().clamp(max=T)


def make(sp: Spec, device="cuda") -> dict:
    """Draws one batch.  Returns a dict of tensors on `device` plus Python metadata.

    Rollout rows are ordered prompt-major: for prompt p the own rollouts, then the
    pooled peer rollouts (PRP); SGT auxiliary rows follow all rollout rows.
    Advantage-call entries are the rollout rows followed by the peer reward-only
    entries (XGRPO pool).
    """
    g = _gen(device, SEED_BASE + sp.index)
    P, T, V, d = sp.n_prompts, sp.T, sp.V, sp.d
    k_seq = sp.k_own + sp.k_peer
    B_roll = P * k_seq

    prompt_of = torch.arange(P, device=device).repeat_interleave(k_seq)
    is_own_roll = (torch.arange(k_seq, device=device) < sp.k_own).repeat(P)
    rewards_roll = (torch.rand(B_roll, device=device, generator=g) < sp.reward_p).float()
    peer_rewards = (torch.rand(P * sp.k_peer_rewards, device=device, generator=g) < sp.reward_p).float()
    peer_prompt = torch.arange(P, device=device).repeat_interleave(sp.k_peer_rewards)

    # SGT: force some prompts to all-fail, give them 1-2 peer successes and 1-2 auxiliary rows
    aux_prompt = []
    if sp.frac_all_fail > 0:
        n_fail = max(1, int(round(P * sp.frac_all_fail)))
        fail_prompts = torch.randperm(P, device=device, generator=g)[:n_fail]
        n_inject = 1 + (torch.rand(n_fail, device=device, generator=g) < 0.5).long()
        for fp, ni in zip(fail_prompts.tolist(), n_inject.tolist()):
            rewards_roll[(prompt_of == fp) & is_own_roll] = 0.0
            if sp.k_peer_rewards > 0:
                sel = torch.nonzero(peer_prompt == fp)[:, 0]
                peer_rewards[sel[:ni]] = 1.0
            aux_prompt += [fp] * ni
    n_aux = len(aux_prompt)
    B = B_roll + n_aux
    N = B * T

    seq_group = torch.cat([prompt_of, torch.tensor(aux_prompt, dtype=torch.int64, device=device)]).int()
    seq_kind = torch.cat([torch.zeros(B_roll, dtype=torch.uint8, device=device),
                          torch.ones(n_aux, dtype=torch.uint8, device=device)])
    is_own_seq = torch.cat([is_own_roll, torch.zeros(n_aux, dtype=torch.bool, device=device)])

    # lengths and masks
    L = torch.empty(B, dtype=torch.int64, device=device)
    L[:B_roll] = torch.where(is_own_roll, _lengths(sp, B_roll, g, device, "own"),
                             _lengths(sp, B_roll, g, device, "peer"))
    if n_aux:
        L[B_roll:] = _lengths(sp, n_aux, g, device, "own")
    mask = (torch.arange(T, device=device)[None, :] < L[:, None])
    if sp.k_peer > 0:   # a few peer tokens carry no aligned behaviour trace and stay unscored
        drop = (torch.rand((B, T), device=device, generator=g) < 0.02) & (~is_own_seq)[:, None]
        mask = mask & ~drop
    mask = mask.to(torch.uint8).contiguous()

    H = torch.empty((N, d), dtype=sp.dtype, device=device)
    W = torch.empty((V, d), dtype=sp.dtype, device=device)
    _randn_into(W, W_STD, g)
    _randn_into(H, 1.0, g)
    targets = torch.randint(0, V, (N,), device=device, generator=g, dtype=torch.int64).int()

    centre = logp_proxy(H, W, targets)
    jit = torch.where(is_own_seq, torch.tensor(sp.old_jitter, device=device),
                      torch.tensor(sp.peer_jitter, device=device)).repeat_interleave(T)
    behav = centre + jit * torch.randn(N, device=device, generator=g)
    ref = centre + sp.ref_jitter * torch.randn(N, device=device, generator=g)

    # advantage-call entries
    rewards_all = torch.cat([rewards_roll, peer_rewards])
    group_all = torch.cat([prompt_of, peer_prompt]).int()
    in_stats = torch.ones(rewards_all.numel(), dtype=torch.uint8, device=device)
    scored = torch.cat([torch.ones(B_roll, dtype=torch.uint8, device=device),
                        torch.zeros(peer_rewards.numel(), dtype=torch.uint8, device=device)])
    is_own = torch.cat([is_own_roll.to(torch.uint8),
                        torch.zeros(peer_rewards.numel(), dtype=torch.uint8, device=device)])

    return dict(spec=sp, B=B, T=T, G=P, N=N, V=V, d=d, B_roll=B_roll, n_aux=n_aux,
                H=H, W=W, targets=targets, mask=mask, behav=behav.contiguous(), ref=ref.contiguous(),
                seq_group=seq_group.contiguous(), seq_kind=seq_kind.contiguous(), lengths=L,
                rewards_all=rewards_all.contiguous(), group_all=group_all.contiguous(),
                in_stats=in_stats, scored=scored, is_own=is_own)


def seq_adv_from(adv_all: torch.Tensor, batch: dict) -> torch.Tensor:
    """Per-sequence advantages for the loss call: rollout rows take their entry of the
    advantage call, auxiliary rows get 0 (they do not use an advantage)."""
    out = torch.zeros(batch["B"], dtype=torch.float32, device=adv_all.device)
    out[:batch["B_roll"]] = adv_all[:batch["B_roll"]]
    return out


def make_thl(B: int, S_src: int, S_tgt: int, seed: int = SEED_BASE + 7, device="cuda",
             p_none: float = 0.02, p_drop_word: float = 0.01, p_drift: float = 0.05,
             prompt_max: int = 64) -> dict:
    """Seeded inputs for the word-level trace alignment with the structure of retokenized peer
    rollouts: a prompt prefix outside the response mask, then a response of whitespace words,
    each split into 1-4 tokens independently on the source and on the target grid (target
    1.0-1.3 x the source length on average, as in configuration 3), a few delimiter tokens
    without a word, a few words missing on one side, and for a few sequences a map that is
    shorter or longer than the response (incremental vs full tokenization drift).  Log-probs
    are -Gamma(1, 1).  Built on the CPU with NumPy (integer bookkeeping), then moved to `device`.
    """
    import numpy as np
    rng = np.random.default_rng(seed)
    src_m = np.zeros((B, S_src), dtype=np.uint8)
    tgt_m = np.zeros((B, S_tgt), dtype=np.uint8)
    src_map = np.full((B, S_src), -1, dtype=np.int32)
    tgt_map = np.full((B, S_tgt), -1, dtype=np.int32)
    src_len = np.zeros(B, dtype=np.int32)
    tgt_len = np.zeros(B, dtype=np.int32)
    max_word = 0
    for i in range(B):
        pre_s, pre_t = (int(rng.integers(0, min(prompt_max, S // 4) + 1)) for S in (S_src, S_tgt))
        budget = int(rng.integers(max(1, (S_src - pre_s) // 6), S_src - pre_s + 1))   # source response tokens
        n_words = max(1, int(budget / 1.5))
        split_s = rng.choice([1, 2, 3, 4], size=n_words, p=[0.62, 0.28, 0.08, 0.02])
        ratio = rng.uniform(1.0, 1.3)
        split_t = np.maximum(1, np.rint(split_s * ratio + rng.uniform(-0.5, 0.5, n_words))).astype(np.int64)
        sides = []
        for split, S, pre in ((split_s, S_src, pre_s), (split_t, S_tgt, pre_t)):
            keep = rng.random(n_words) >= p_drop_word
            words = np.repeat(np.arange(n_words)[keep], split[keep])
            lead = int(rng.integers(0, 2))
            words = np.concatenate([np.full(lead, -1, dtype=np.int64), words])
            words = np.where(rng.random(words.size) < p_none, -1, words)[: S - pre]
            n_resp = words.size
            if rng.random() < p_drift and n_resp > 4:
                n_resp = int(np.clip(n_resp + rng.integers(-3, 4), 0, S - pre))
            sides.append((words, n_resp, pre))
        (ws, ns, ps), (wt, nt, pt) = sides
        src_m[i, ps:ps + ns] = 1
        tgt_m[i, pt:pt + nt] = 1
        src_map[i, :ws.size] = ws
        tgt_map[i, :wt.size] = wt
        src_len[i], tgt_len[i] = ws.size, wt.size
        max_word = max(max_word, int(ws.max(initial=0)), int(wt.max(initial=0)))
    src_lp = -rng.gamma(1.0, 1.0, size=(B, S_src)).astype(np.float32)
    t = lambda a: torch.from_numpy(a).to(device)
    return dict(src_logp=t(src_lp), src_mask=t(src_m), src_word_map=t(src_map), src_map_len=t(src_len),
                tgt_mask=t(tgt_m), tgt_word_map=t(tgt_map), tgt_map_len=t(tgt_len),
                max_words=max_word + 1, B=B, S_src=S_src, S_tgt=S_tgt)
