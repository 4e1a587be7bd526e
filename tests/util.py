"""Helpers shared by the GPU parity tests: batch -> oracle inputs, comparisons."""
import numpy as np
import torch

from oracle import mrl_oracle as orc

LOGP_TOL = 2e-3      # |delta logp| per token (bf16 inputs, fp32 accumulation)
REL_TOL = 1e-2       # relative Frobenius error on dH, dW; relative error on the loss
F32_LOGP_TOL = 2e-5  # fp32 sanity path
F32_REL_TOL = 2e-4
ROW_REL_FACTOR = 2.0     # per-row relative error bound on dH / dW rows = ROW_REL_FACTOR * the Frobenius tolerance
ROW_NORM_FLOOR = 1e-4    # ... for rows whose reference norm is at least this share of the largest row norm
CANCEL_SHARE = 1e-4      # a loss value below this share of the sum of its absolute token terms is cancellation-dominated
ABS_TERM_TOL = 1e-4      # error bound relative to the sum of absolute token terms (fp32 token terms: ~1e-6 in practice)


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


def check_gradient(name, got, ref, rel_tol=REL_TOL):
    """dH / dW against the oracle, three ways: relative Frobenius error of the whole tensor,
    largest elementwise error against the largest reference element, and the relative error of
    every row whose reference norm is above a floor (a defect confined to a few rows - a ragged
    last tile, a pass boundary - is invisible in the whole-tensor norm).  Returns the three
    figures."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), name
    fro = rel_fro(got, ref)
    diff = got - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    ref_max = float(np.max(np.abs(ref))) if ref.size else 0.0
    row_ref = np.linalg.norm(ref, axis=1)
    row_err = np.linalg.norm(diff, axis=1)
    floor = ROW_NORM_FLOOR * (row_ref.max() if row_ref.size else 0.0)
    big = row_ref > max(floor, 0.0)
    worst_row = float(np.max(row_err[big] / row_ref[big])) if big.any() else 0.0
    # rows below the floor (incl. exact zeros of the reference) are bounded absolutely
    small_err = float(np.max(row_err[~big])) if (~big).any() else 0.0
    print(f"{name}: rel fro {fro:.2e}, max|err| {max_abs:.2e} (max|ref| {ref_max:.2e}), "
          f"worst row rel {worst_row:.2e} over {int(big.sum())} rows, small-row err {small_err:.2e}")
    assert fro <= rel_tol, (name, "fro", fro)
    assert max_abs <= rel_tol * ref_max, (name, "max-abs", max_abs, ref_max)
    assert worst_row <= ROW_REL_FACTOR * rel_tol, (name, "row", worst_row)
    assert small_err <= ROW_REL_FACTOR * rel_tol * max(floor, 1e-300) or small_err == 0.0, (name, "small rows", small_err, floor)
    return fro, max_abs, worst_row


def check_loss_terms(st, want, beta, lam, rel_tol=REL_TOL):
    """Loss values against the oracle.  The plain relative error |got - ref| / |ref| must meet
    `rel_tol` for every term that is not cancellation-dominated.  The surrogate sums
    advantage-signed token terms that can cancel to (almost) nothing under centred advantages;
    then |ref| is no scale for the error, and the error is bounded against the sum of the
    absolute token terms instead (tightly: fp32 token terms leave about 1e-6 of it).  That second
    bound is asserted always."""
    pg_abs = float(np.sum(want["c"] * np.abs(np.minimum(want["s1"], want["s2"]))))
    scales = dict(loss_pg=pg_abs, loss_kl=abs(want["loss_kl"]), loss_sgt=abs(want["loss_sgt"]))
    scales["loss_total"] = pg_abs + beta * scales["loss_kl"] + lam * scales["loss_sgt"]
    for key in ("loss_total", "loss_pg", "loss_kl", "loss_sgt"):
        err = abs(st[key] - want[key])
        sc = scales[key]
        plain = err / abs(want[key]) if want[key] != 0 else (0.0 if err == 0 else np.inf)
        print(f"{key}: got {st[key]:.9e} want {want[key]:.9e} plain rel {plain:.2e} vs abs-term sum {err / max(sc, 1e-300):.2e}")
        assert err <= ABS_TERM_TOL * max(sc, 1e-12), (key, st[key], want[key], sc)
        if abs(want[key]) >= CANCEL_SHARE * sc and sc > 0:
            assert plain <= rel_tol, (key, st[key], want[key], plain)
