"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol declared in include/*.h, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2605_07244_amd as m
from paper_2605_07244_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mrl_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = m.lib()
    names = _declared_symbols()
    assert {"mrl_token_logprobs", "mrl_group_advantages", "mrl_grpo_loss_fwd_bwd"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_version_and_status_strings():
    assert m.version() >= 100
    assert m.status_string(0) == "ok"
    for code in range(-9, 0):
        assert m.status_string(code) not in ("ok", "unknown status")
    assert m.status_string(-99) == "unknown status"


def test_stats_struct_size_matches_header():
    # 7 doubles + 6 int64 (see mrl_loss_stats)
    assert binding.STATS_BYTES == 104 and len(binding.STATS_FIELDS) == 13


P = ctypes.c_void_p
FAKE = P(0x1000)   # never dereferenced: validation fails first


def _cfg(**kw):
    return binding.LossConfig(**kw).to_c()


def test_token_logprobs_argument_errors():
    lib = m.lib()
    f = lib.mrl_token_logprobs
    assert f(None, FAKE, FAKE, None, 8, 128, 32, 1, FAKE, None, FAKE, 1 << 20, None) == -1
    assert f(FAKE, FAKE, FAKE, None, 8, 128, 32, 1, None, None, FAKE, 1 << 20, None) == -1
    assert f(FAKE, FAKE, FAKE, None, 8, 64, 32, 7, FAKE, None, FAKE, 1 << 20, None) == -3
    assert f(FAKE, FAKE, FAKE, None, -1, 128, 32, 1, FAKE, None, FAKE, 1 << 20, None) == -2
    assert f(FAKE, FAKE, FAKE, None, 8, 0, 32, 1, FAKE, None, FAKE, 1 << 20, None) == -2
    assert f(FAKE, FAKE, FAKE, None, 8, 64, 0, 1, FAKE, None, FAKE, 1 << 20, None) == -2
    assert f(FAKE, FAKE, FAKE, None, 8, 36, 32, 1, FAKE, None, FAKE, 1 << 20, None) == -2   # bf16: d % 8
    assert f(FAKE, FAKE, FAKE, None, 0, 128, 32, 1, FAKE, None, None, 0, None) == 0          # N = 0: no-op
    assert f(FAKE, FAKE, FAKE, None, 8, 128, 32, 1, FAKE, None, None, 0, None) == -6
    assert f(FAKE, FAKE, FAKE, None, 8, 128, 32, 1, FAKE, None, P(0x1001), 1 << 20, None) == -6  # misaligned
    assert f(FAKE, FAKE, FAKE, None, 8, 128, 32, 1, FAKE, None, FAKE, 16, None) == -6           # too small


def test_workspace_queries():
    assert m.token_logprobs_workspace(1024, 128, 1000, m.BF16) > 0
    assert m.token_logprobs_workspace(1024, 100, 1000, m.BF16) == 0      # invalid shape -> 0
    small = m.grpo_loss_workspace(4, 64, 128, 1000, m.BF16, m.LossConfig(chunk_rows=256))
    big = m.grpo_loss_workspace(4, 64, 128, 1000, m.BF16, m.LossConfig(chunk_rows=1024))
    assert 0 < small < big
    assert m.grpo_loss_workspace(4, 64, 128, 1000, m.BF16, m.LossConfig(chunk_rows=100)) == 0
    # the stress configuration fits comfortably into one GPU's HBM
    ws5 = m.grpo_loss_workspace(1024, 2048, 4096, 151936, m.BF16, m.LossConfig())
    assert 5e9 < ws5 < 40e9


def test_group_advantages_argument_errors():
    f = m.lib().mrl_group_advantages
    ok_tail = (FAKE, None, None, None, None)
    assert f(None, FAKE, None, None, None, None, 8, 2, 1, 1e-6, 0, 1.0, 0.2, 0.8, *ok_tail) == -1
    assert f(FAKE, FAKE, None, None, None, None, 8, 2, 1, 1e-6, 0, 1.0, 0.2, 0.8, None, None, None, None, None) == -1
    assert f(FAKE, FAKE, None, None, None, None, 8, 0, 1, 1e-6, 0, 1.0, 0.2, 0.8, *ok_tail) == -2
    assert f(FAKE, FAKE, None, None, None, None, -1, 2, 1, 1e-6, 0, 1.0, 0.2, 0.8, *ok_tail) == -2
    assert f(FAKE, FAKE, None, None, None, None, 8, 2, 5, 1e-6, 0, 1.0, 0.2, 0.8, *ok_tail) == -7
    assert f(FAKE, FAKE, None, None, None, None, 8, 2, 1, -1.0, 0, 1.0, 0.2, 0.8, *ok_tail) == -7
    assert f(FAKE, FAKE, None, None, None, None, 8, 2, 1, 1e-6, 2, 1.0, 0.2, 0.8, *ok_tail) == -7
    assert f(FAKE, FAKE, None, None, None, None, 8, 2, 1, 1e-6, 0, 1.5, 0.2, 0.8, *ok_tail) == -7
    assert f(FAKE, FAKE, None, None, None, None, 0, 2, 1, 1e-6, 0, 1.0, 0.2, 0.8, *ok_tail) == 0


def _loss(cfg, *, hidden=FAKE, ref=FAKE, B=4, T=8, G=2, d=128, V=100, dt=1, ws=FAKE, ws_bytes=1 << 30,
          stats=FAKE, seq_adv=FAKE):
    f = m.lib().mrl_grpo_loss_fwd_bwd
    return f(hidden, FAKE, FAKE, FAKE, FAKE, ref, seq_adv, FAKE, None, B, T, G, d, V, dt,
             ctypes.byref(cfg) if cfg is not None else None, FAKE, FAKE, FAKE, stats, ws, ws_bytes, None)


def test_loss_argument_errors():
    good = _cfg()
    assert _loss(good, hidden=None) == -1
    assert _loss(good, stats=None) == -1
    assert _loss(None) == -1
    assert _loss(good, ref=None) == -1                       # beta > 0 needs a reference trace
    assert _loss(good, B=0) == -2
    assert _loss(good, T=0) == -2
    assert _loss(good, G=0) == -2
    assert _loss(good, G=9) == -2                            # more groups than sequences
    assert _loss(good, d=65) == -2
    assert _loss(good, dt=3) == -3
    assert _loss(_cfg(clip_eps_low=-0.1)) == -7
    assert _loss(_cfg(kl_beta=-1.0)) == -7
    assert _loss(_cfg(loss_agg=2)) == -7
    assert _loss(_cfg(ratio_level=3)) == -7
    assert _loss(_cfg(ratio_level=1, loss_agg=1)) == -7
    assert _loss(_cfg(accumulate_dw=3)) == -7
    assert _loss(_cfg(dh_dtype=5)) == -7
    assert _loss(_cfg(chunk_rows=300)) == -7
    assert _loss(_cfg(scored_rows_hint=-5)) == -7
    assert _loss(_cfg(dh_dtype=1), dt=0) == -7               # fp32 path writes fp32 dH only
    assert _loss(good, ws=None) == -6
    assert _loss(good, ws_bytes=1024) == -6


def test_no_device_is_an_error_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    # all arguments valid: the call must stop at the device check, nothing is computed on the CPU
    rc = _loss(_cfg())
    assert rc in (-8, -9)


def test_profile_calls_without_device():
    assert m.lib().mrl_profile_enable(0) == 0
    assert m.lib().mrl_profile_collect(None, None) == -1
    out = m.profile_collect()
    assert set(out) == set(m.PROF_CLASSES)


def test_probe_argument_errors():
    f = m.lib().mrl_probe_mfma_rate
    out = ctypes.c_double(0.0)
    assert f(0, 0.1, None, 1 << 20, ctypes.byref(out)) == -1
    assert f(0, 0.1, FAKE, 1 << 20, None) == -1
    assert f(0, 0.0, FAKE, 1 << 20, ctypes.byref(out)) == -7
    assert f(0, 60.0, FAKE, 1 << 20, ctypes.byref(out)) == -7


def test_dw_tail_plan_host_logic():
    """The plan of the dW launch's K-split tail: every item of every split tile is dealt to exactly one XCD,
    the partial-tile scratch (256 tiles) is never exceeded, whole super-tile rows are left alone."""
    f = m.lib().mrl_diag_dw_tail_plan
    out = (ctypes.c_int32 * 12)()
    assert f(1000, 64, None) == -1 and f(0, 64, out) == -2 and f(1000, 0, out) == -2
    seen_split = set()
    for V in (300, 2048, 2500, 3001, 8333, 32000, 50257, 128256, 151936, 262144):
        for d in (64, 384, 768, 1536, 2048, 3584, 4096, 5120, 8192):
            assert f(V, d, out) == 0
            m0, rows, split = out[0], out[1], out[2]
            pre = list(out[3:12])
            Mt, Nt = -(-V // 256), -(-d // 256)
            sup_m = 16 if Nt == 1 else 8
            assert m0 % sup_m == 0 and m0 + rows == Mt and 0 <= rows < sup_m
            assert split == 0 or 2 <= split <= 8
            if split:
                items = rows * Nt * split
                assert m0 > 0 and rows > 0 and items <= 256
                assert pre[0] == 0 and pre[8] == items and all(a <= b for a, b in zip(pre, pre[1:]))
            else:
                assert pre == [0] * 9
            seen_split.add(split)
    assert 0 in seen_split and 8 in seen_split and len(seen_split) >= 3
    # the benchmark shapes: V = 151936 leaves two ragged tile rows
    assert f(151936, 4096, out) == 0 and (out[0], out[1], out[2]) == (592, 2, 8) and list(out[3:12]) == list(range(0, 257, 32))
    assert f(151936, 1536, out) == 0 and out[2] >= 2 and out[11] == 12 * out[2]


def test_thl_word_align_argument_errors():
    f = m.lib().mrl_thl_word_align
    args = lambda **kw: [kw.get("p0", FAKE), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, kw.get("B", 4), kw.get("S", 16), 16,
                         kw.get("W", 32), ctypes.c_float(-100.0), kw.get("out", FAKE), None, None]
    assert f(*args(p0=None)) == -1
    assert f(*args(out=None)) == -1
    assert f(*args(S=0)) == -2
    assert f(*args(B=-1)) == -2
    assert f(*args(W=0)) == -2
    assert f(*args(W=8193)) == -2
    assert f(*args(B=0)) == 0          # empty batch: no-op


def test_token_scores_argument_errors():
    lib = m.lib()
    f = lib.mrl_token_scores
    assert f(None, FAKE, FAKE, None, 8, 128, 32, 1, FAKE, None, None, FAKE, 1 << 20, None) == -1
    assert f(FAKE, FAKE, FAKE, None, 8, 36, 32, 1, FAKE, None, FAKE, FAKE, 1 << 20, None) == -2
    assert f(FAKE, FAKE, FAKE, None, 8, 128, 32, 1, FAKE, None, FAKE, FAKE, 16, None) == -6    # workspace too small
    assert f(FAKE, FAKE, FAKE, None, 0, 128, 32, 1, FAKE, None, FAKE, None, 0, None) == 0
    # the entropy needs a third partial buffer: its workspace is the larger one
    assert lib.mrl_token_scores_workspace(4096, 256, 4000, 1) > lib.mrl_token_logprobs_workspace(4096, 256, 4000, 1)


def test_static_logprobs_argument_errors():
    """The allocation-free variant validates on the host before it touches a device: NULL
    pointers, shapes, and inputs beyond its built-in scratch buffer."""
    f = m.lib().mrl_token_logprobs_static
    one = 8  # any non-null address: rejected arguments are never dereferenced
    assert f(None, one, one, None, 16, 128, 512, 1, one, None, None) == -1
    assert f(one, one, one, None, 16, 100, 512, 1, one, None, None) == -2        # d % 8
    assert f(one, one, one, None, 16, 128, 512, 7, one, None, None) == -3
    assert f(one, one, one, None, 0, 128, 512, 1, one, None, None) == 0           # empty input: no-op
    assert f(one, one, one, None, 1 << 23, 128, 512, 1, one, None, None) == -10   # 8 B per row > 32 MiB
    assert f(one, one, one, None, 1024, 128, 1 << 22, 1, one, None, None) == -10  # partials of one pass > 32 MiB
    assert "scratch" in m.status_string(-10)
