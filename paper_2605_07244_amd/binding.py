"""ctypes binding of include/mrl.h.  Argument marshalling only.

Every function takes torch tensors that already live on the GPU (the library
only accepts device pointers), checks dtype / contiguity / device on the host,
and forwards raw pointers plus the current torch stream.  There is no CPU or
PyTorch fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from dataclasses import dataclass

import torch

F32, BF16 = 0, 1
ADV_CENTER, ADV_GROUP_ZN, ADV_BATCH_ZN = 0, 1, 2
PROF_CLASSES = ("prep", "adv", "gemm_fwd", "row_epilogue", "operand_prep", "gemm_dh", "gemm_dw", "final")

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class MrlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: mrl status {status} ({status_string(status)})")


def library_path() -> str:
    return os.path.join(_HERE, "libmrl.so")


class _LossConfig(ctypes.Structure):
    _fields_ = [("clip_eps_low", c_float), ("clip_eps_high", c_float), ("kl_beta", c_float),
                ("sgt_lambda", c_float), ("loss_agg", c_int32), ("accumulate_dw", c_int32),
                ("dh_dtype", c_int32), ("chunk_rows", c_int32), ("scored_rows_hint", c_int64),
                ("ratio_level", c_int32), ("debug_sync", c_int32)]


@dataclass
class LossConfig:
    clip_eps_low: float = 0.2
    clip_eps_high: float = 0.2
    kl_beta: float = 0.04
    sgt_lambda: float = 0.1
    loss_agg: int = 0
    accumulate_dw: int = 0
    dh_dtype: int = BF16
    chunk_rows: int = 0
    scored_rows_hint: int = 0
    ratio_level: int = 0
    debug_sync: int = 0

    def to_c(self) -> _LossConfig:
        return _LossConfig(self.clip_eps_low, self.clip_eps_high, self.kl_beta, self.sgt_lambda,
                           self.loss_agg, self.accumulate_dw, self.dh_dtype, self.chunk_rows,
                           self.scored_rows_hint, self.ratio_level, self.debug_sync)


STATS_FIELDS = ("loss_total", "loss_pg", "loss_kl", "loss_sgt", "mean_ratio", "max_ratio", "mean_k3",
                "n_scored_tokens", "n_clipped_tokens", "n_zero_grad_tokens", "n_bad_targets",
                "n_unprocessed_rows", "n_saturated_rows")
STATS_BYTES = 7 * 8 + 6 * 8


def lib() -> ctypes.CDLL:
    """Loads libmrl.so (once).  Raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2605_07244_amd.build` "
            "(there is no fallback implementation)")
    L = ctypes.CDLL(path)
    L.mrl_status_string.restype = c_char_p
    L.mrl_status_string.argtypes = [c_int]
    L.mrl_version.restype = c_int
    L.mrl_token_logprobs_workspace.restype = c_size_t
    L.mrl_token_logprobs_workspace.argtypes = [c_int64, c_int32, c_int32, c_int32]
    L.mrl_token_logprobs.restype = c_int
    L.mrl_token_logprobs.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32,
                                     c_int32, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    L.mrl_token_logprobs_static.restype = c_int
    L.mrl_token_logprobs_static.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32,
                                            c_int32, c_void_p, c_void_p, c_void_p]
    L.mrl_token_scores_workspace.restype = c_size_t
    L.mrl_token_scores_workspace.argtypes = [c_int64, c_int32, c_int32, c_int32]
    L.mrl_token_scores.restype = c_int
    L.mrl_token_scores.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32,
                                   c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    L.mrl_group_advantages.restype = c_int
    L.mrl_group_advantages.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32,
                                       c_int32, c_float, c_int32, c_float, c_float, c_float,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.mrl_grpo_loss_workspace.restype = c_size_t
    L.mrl_grpo_loss_workspace.argtypes = [c_int64, c_int32, c_int32, c_int32, c_int32, POINTER(_LossConfig)]
    L.mrl_grpo_loss_fwd_bwd.restype = c_int
    L.mrl_grpo_loss_fwd_bwd.argtypes = [c_void_p] * 9 + [c_int64, c_int32, c_int32, c_int32, c_int32, c_int32,
                                                         POINTER(_LossConfig), c_void_p, c_void_p, c_void_p,
                                                         c_void_p, c_void_p, c_size_t, c_void_p]
    L.mrl_profile_enable.restype = c_int
    L.mrl_profile_enable.argtypes = [c_int]
    L.mrl_profile_collect.restype = c_int
    L.mrl_profile_collect.argtypes = [POINTER(c_double), POINTER(c_int64)]
    L.mrl_thl_word_align.restype = c_int
    L.mrl_thl_word_align.argtypes = [c_void_p] * 7 + [c_int64, c_int32, c_int32, c_int32, c_float, c_void_p,
                                                      c_void_p, c_void_p]
    L.mrl_diag_dw_tail_plan.restype = c_int
    L.mrl_diag_dw_tail_plan.argtypes = [c_int32, c_int32, POINTER(c_int32)]
    L.mrl_probe_mfma_rate.restype = c_int
    L.mrl_probe_mfma_rate.argtypes = [c_int32, c_double, c_void_p, c_size_t, POINTER(c_double)]
    _LIB = L
    return L


def status_string(status: int) -> str:
    return lib().mrl_status_string(int(status)).decode()


def version() -> int:
    return lib().mrl_version()


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU torch tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return c_void_p(t.data_ptr())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"hidden / lm_head_w must be bfloat16 or float32, got {t.dtype}")


def _stream() -> c_void_p:
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise MrlError(rc, where)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def token_logprobs_workspace(N: int, d: int, V: int, dtype: int) -> int:
    return int(lib().mrl_token_logprobs_workspace(N, d, V, dtype))


def token_logprobs(hidden, lm_head_w, target_ids, token_mask=None, workspace=None, want_lse=True):
    """mrl_token_logprobs: returns (logp[N] f32, lse[N] f32 or None)."""
    N, d = hidden.shape
    V = lm_head_w.shape[0]
    dt = _dtype_code(hidden)
    if lm_head_w.dtype != hidden.dtype or lm_head_w.shape[1] != d:
        raise ValueError("lm_head_w must be [V, d] with the dtype of hidden")
    out_logp = torch.empty(N, dtype=torch.float32, device=hidden.device)
    out_lse = torch.empty(N, dtype=torch.float32, device=hidden.device) if want_lse else None
    if N == 0:            # empty tensors have no device pointer; the library treats N = 0 as a no-op too
        return out_logp, out_lse
    if workspace is None:
        workspace = _workspace(token_logprobs_workspace(N, d, V, dt), hidden.device)
    rc = lib().mrl_token_logprobs(_ptr(hidden, name="hidden"), _ptr(lm_head_w, name="lm_head_w"),
                                  _ptr(target_ids, torch.int32, "target_ids"),
                                  _ptr(token_mask, torch.uint8, "token_mask"), N, d, V, dt,
                                  _ptr(out_logp), _ptr(out_lse), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "mrl_token_logprobs")
    return out_logp, out_lse


STATIC_SCRATCH_BYTES = 32 << 20


def token_logprobs_static(hidden, lm_head_w, target_ids, token_mask, out_logp, out_lse=None):
    """mrl_token_logprobs_static: the log-prob call on the library's built-in scratch buffer.  The
    caller passes the output tensors; nothing is allocated here or in the library."""
    N, d = hidden.shape
    V = lm_head_w.shape[0]
    rc = lib().mrl_token_logprobs_static(_ptr(hidden, name="hidden"), _ptr(lm_head_w, name="lm_head_w"),
                                         _ptr(target_ids, torch.int32, "target_ids"),
                                         _ptr(token_mask, torch.uint8, "token_mask"), N, d, V, _dtype_code(hidden),
                                         _ptr(out_logp, torch.float32, "out_logp"),
                                         _ptr(out_lse, torch.float32, "out_lse"), _stream())
    _check(rc, "mrl_token_logprobs_static")


def token_scores(hidden, lm_head_w, target_ids, token_mask=None, workspace=None, want_lse=True,
                 want_entropy=True):
    """Forward-only scoring pass: (logp, lse | None, entropy | None), each [N] float32."""
    N, d = hidden.shape
    V = lm_head_w.shape[0]
    dt = _dtype_code(hidden)
    dev = hidden.device
    need = lib().mrl_token_scores_workspace(N, d, V, dt) if want_entropy else \
        lib().mrl_token_logprobs_workspace(N, d, V, dt)
    if workspace is None:
        workspace = _workspace(need, dev)
    out_logp = torch.empty(N, dtype=torch.float32, device=dev)
    out_lse = torch.empty(N, dtype=torch.float32, device=dev) if want_lse else None
    out_ent = torch.empty(N, dtype=torch.float32, device=dev) if want_entropy else None
    _check(lib().mrl_token_scores(_ptr(hidden), _ptr(lm_head_w), _ptr(target_ids, torch.int32, "target_ids"),
                                  _ptr(token_mask, torch.uint8, "token_mask"), N, d, V, dt, _ptr(out_logp),
                                  _ptr(out_lse), _ptr(out_ent), _ptr(workspace), workspace.numel(), _stream()),
           "mrl_token_scores")
    return out_logp, out_lse, out_ent


def group_advantages(rewards, group_id, G, in_stats=None, scored=None, is_own=None, mode=ADV_GROUP_ZN,
                     eps_norm=1e-6, ddof=0, mix_alpha=1.0, neg_thresh=0.2, pos_thresh=0.8, baseline_shift=None):
    """mrl_group_advantages: returns (adv[B], mean[G], std[G], flags[G] uint8)."""
    if baseline_shift is not None and baseline_shift.numel() != G:
        raise ValueError("baseline_shift must have G entries")
    B = rewards.numel()
    dev = rewards.device
    adv = torch.empty(B, dtype=torch.float32, device=dev)
    mean = torch.empty(G, dtype=torch.float32, device=dev)
    std = torch.empty(G, dtype=torch.float32, device=dev)
    flags = torch.empty(G, dtype=torch.uint8, device=dev)
    rc = lib().mrl_group_advantages(_ptr(rewards, torch.float32, "rewards"), _ptr(group_id, torch.int32, "group_id"),
                                    _ptr(in_stats, torch.uint8, "in_stats"), _ptr(scored, torch.uint8, "scored"),
                                    _ptr(is_own, torch.uint8, "is_own"),
                                    _ptr(baseline_shift, torch.float32, "baseline_shift"), B, G, mode, eps_norm, ddof, mix_alpha,
                                    neg_thresh, pos_thresh, _ptr(adv), _ptr(mean), _ptr(std), _ptr(flags), _stream())
    _check(rc, "mrl_group_advantages")
    return adv, mean, std, flags


def grpo_loss_workspace(B: int, T: int, d: int, V: int, dtype: int, cfg: LossConfig) -> int:
    c = cfg.to_c()
    return int(lib().mrl_grpo_loss_workspace(B, T, d, V, dtype, ctypes.byref(c)))


def grpo_loss_fwd_bwd(hidden, lm_head_w, target_ids, token_mask, behav_logp, ref_logp, seq_adv, group_id,
                      seq_kind, B, T, G, cfg: LossConfig, out_dH=None, out_dW=None, want_dH=True, want_dW=True,
                      workspace=None, out_logp=None, out_stats=None):
    """mrl_grpo_loss_fwd_bwd.  Returns dict(logp, dH, dW, stats_tensor); `read_stats`
    turns the device stats block into a Python dict (synchronises)."""
    N, d = hidden.shape
    if N != B * T:
        raise ValueError("hidden must be [B*T, d]")
    V = lm_head_w.shape[0]
    dt = _dtype_code(hidden)
    dev = hidden.device
    if out_logp is None:
        out_logp = torch.empty(N, dtype=torch.float32, device=dev)
    if out_dH is None and want_dH:
        out_dH = torch.empty((N, d), dtype=torch.bfloat16 if cfg.dh_dtype == BF16 else torch.float32, device=dev)
    if out_dW is None and want_dW:
        out_dW = torch.empty((V, d), dtype=torch.float32, device=dev)
    if out_stats is None:
        out_stats = torch.empty(STATS_BYTES, dtype=torch.uint8, device=dev)
    if workspace is None:
        workspace = _workspace(grpo_loss_workspace(B, T, d, V, dt, cfg), dev)
    c = cfg.to_c()
    rc = lib().mrl_grpo_loss_fwd_bwd(
        _ptr(hidden, name="hidden"), _ptr(lm_head_w, name="lm_head_w"), _ptr(target_ids, torch.int32, "target_ids"),
        _ptr(token_mask, torch.uint8, "token_mask"), _ptr(behav_logp, torch.float32, "behav_logp"),
        _ptr(ref_logp, torch.float32, "ref_logp"), _ptr(seq_adv, torch.float32, "seq_adv"),
        _ptr(group_id, torch.int32, "group_id"), _ptr(seq_kind, torch.uint8, "seq_kind"),
        B, T, G, d, V, dt, ctypes.byref(c), _ptr(out_logp), _ptr(out_dH), _ptr(out_dW, torch.float32, "out_dW"),
        _ptr(out_stats), _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "mrl_grpo_loss_fwd_bwd")
    return dict(logp=out_logp, dH=out_dH, dW=out_dW, stats=out_stats)


def read_stats(stats: torch.Tensor) -> dict:
    """Copies the device stats block to the host (synchronises) and decodes it."""
    raw = stats.cpu().numpy().tobytes()
    import struct
    vals = struct.unpack("<7d6q", raw)
    return dict(zip(STATS_FIELDS, vals))


def profile_enable(on: bool = True):
    _check(lib().mrl_profile_enable(1 if on else 0), "mrl_profile_enable")


def profile_collect() -> dict:
    """Returns {class: (milliseconds, launches)} since the last collect (synchronises)."""
    ms = (c_double * len(PROF_CLASSES))()
    n = (c_int64 * len(PROF_CLASSES))()
    _check(lib().mrl_profile_collect(ms, n), "mrl_profile_collect")
    return {name: (ms[i], n[i]) for i, name in enumerate(PROF_CLASSES)}


def dw_tail_plan(V: int, d: int) -> dict:
    """Launch plan of the dW GEMM's K-split tail for a [V, d] head (host code only)."""
    out = (c_int32 * 12)()
    _check(lib().mrl_diag_dw_tail_plan(int(V), int(d), out), "mrl_diag_dw_tail_plan")
    return dict(first_tile_row=out[0], tile_rows=out[1], split=out[2], items_before_xcd=list(out[3:12]))


def probe_mfma_rate(random_operands: bool, seconds: float = 0.5, device="cuda:0") -> float:
    """TFLOP/s the matrix cores sustain on the GEMM kernels' MFMA instruction, registers only."""
    scratch = torch.empty(512 * 1024, dtype=torch.uint8, device=device)
    out = c_double(0.0)
    torch.cuda.synchronize()
    _check(lib().mrl_probe_mfma_rate(1 if random_operands else 0, float(seconds), _ptr(scratch),
                                     scratch.numel(), ctypes.byref(out)), "mrl_probe_mfma_rate")
    return out.value


def thl_word_align(src_logp, src_mask, src_word_map, src_map_len, tgt_mask, tgt_word_map, tgt_map_len,
                   max_words: int, ignore_value: float = -100.0, want_bad_count: bool = True):
    """Word-level trace alignment (App. D, Alg. 2).  Returns (out [B, S_tgt] float32, bad-entry count tensor)."""
    B, S_src = src_logp.shape
    S_tgt = tgt_mask.shape[1]
    dev = src_logp.device
    out = torch.empty((B, S_tgt), dtype=torch.float32, device=dev)
    bad = torch.empty(1, dtype=torch.int64, device=dev) if want_bad_count else None
    _check(lib().mrl_thl_word_align(
        _ptr(src_logp, torch.float32, "src_logp"), _ptr(src_mask, torch.uint8, "src_mask"),
        _ptr(src_word_map, torch.int32, "src_word_map"), _ptr(src_map_len, torch.int32, "src_map_len"),
        _ptr(tgt_mask, torch.uint8, "tgt_mask"), _ptr(tgt_word_map, torch.int32, "tgt_word_map"),
        _ptr(tgt_map_len, torch.int32, "tgt_map_len"), B, S_src, S_tgt, int(max_words), float(ignore_value),
        _ptr(out), _ptr(bad) if bad is not None else None, _stream()), "mrl_thl_word_align")
    return out, bad
