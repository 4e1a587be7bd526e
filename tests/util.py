"""Helpers shared by the GPU parity tests: batch -> oracle inputs, comparisons."""
import numpy as np
import torch

from oracle import mrl_oracle as orc

LOGP_TOL = 2e-3      # |delta logp| per token (bf16 inputs, fp32 accumulation)
REL_TOL = 1e-2       # relative Frobenius error on dH, dW; relative error on the loss
F32_LOGP_TOL = 2e-5  # fp32 sanity path
F32_REL_TOL = 2e-4


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact fp64 copy of a float32 / bfloat16 tensor."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).numpy().view(np.uint16)
        return orc.decode_bf16(bits).reshape(t.shape)
    return t.numpy().astype(np.float64)


def cfg_dict(sp, **over):
    c = dict(clip_eps_low=sp.clip_eps, clip_eps_high=sp.clip_eps, kl_beta=sp.kl_beta,
             sgt_lambda=sp.sgt_lambda, loss_agg=0)
    c.update(over)
    return c


def oracle_advantages(batch, mode=orc.ADV_GROUP_ZN, **kw):
    return orc.group_advantages(to_f64(batch["rewards_all"]), batch["group_all"].cpu().numpy(), batch["G"],
                                batch["in_stats"].cpu().numpy(), batch["scored"].cpu().numpy(),
                                batch["is_own"].cpu().numpy(), mode=mode, **kw)


def oracle_loss(batch, seq_adv, cfg, behav=None, ref=None, need_grads=True):
    behav = batch["behav"] if behav is None else behav
    ref = batch["ref"] if ref is None else ref
    return orc.grpo_loss_fwd_bwd(
        to_f64(batch["H"]), to_f64(batch["W"]), batch["targets"].cpu().numpy(),
        batch["mask"].cpu().numpy().reshape(batch["B"], batch["T"]), to_f64(behav),
        None if ref is None else to_f64(ref), np.asarray(seq_adv, dtype=np.float64),
        batch["seq_group"].cpu().numpy(), batch["seq_kind"].cpu().numpy(),
        batch["B"], batch["T"], batch["G"], cfg, need_grads=need_grads)


def move_off_kinks(batch, oracle_logp, eps, margin=4e-3, shift=0.03):
    """Shifts the behaviour trace of tokens whose ratio sits within `margin` (in log
    space) of a clip edge, so that fp32 and fp64 take the same clip decision.  Uses
    the oracle's log-probs only.  Returns the new behaviour tensor (fp32, on device)."""
    behav = batch["behav"].detach().cpu().numpy().astype(np.float64)
    delta = oracle_logp - behav
    for edge in (np.log1p(-eps), np.log1p(eps), 0.0):   # 0.0: w = 1 exactly is harmless, kept for symmetry
        if edge == 0.0:
            continue
        near = np.abs(delta - edge) < margin
        behav = np.where(near, behav - shift, behav)
    return torch.tensor(behav, dtype=torch.float32, device=batch["behav"].device)


def move_off_kinks_seq(batch, oracle_logp, eps, level, margin=2e-2, shift=0.08):
    """Response-level ratios (App. I.1): shifts the behaviour log-prob of the first scored token
    of every response whose ratio sits within `margin` (in log space) of a clip edge, so that fp32
    and fp64 take the same clip decision.  Uses the oracle's log-probs only."""
    B, T = batch["B"], batch["T"]
    behav = batch["behav"].detach().cpu().numpy().astype(np.float64).reshape(B, T)
    m = batch["mask"].cpu().numpy().astype(bool).reshape(B, T)
    lp = np.asarray(oracle_logp).reshape(B, T)
    for b in range(B):
        L = int(m[b].sum())
        if L == 0:
            continue
        expo = float(np.sum((lp[b] - behav[b])[m[b]])) / (L if level == 2 else 1)
        for edge in (np.log1p(-eps), np.log1p(eps)):
            if abs(expo - edge) < margin:
                first = int(np.nonzero(m[b])[0][0])
                behav[b, first] -= shift * (L if level == 2 else 1)
    return torch.tensor(behav.reshape(-1), dtype=torch.float32, device=batch["behav"].device)


def rel_fro(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / den) if den > 0 else float(np.linalg.norm(x))


def rel_err(x, ref):
    return abs(x - ref) / max(abs(ref), 1e-12)
