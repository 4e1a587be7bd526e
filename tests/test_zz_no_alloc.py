"""The allocation-free log-prob entry point (mrl_token_logprobs_static) against the workspace
variant it shares its kernels with, through the C ABI: two calls in a row on the library's
built-in scratch buffer, the second on a smaller input, each compared with mrl_token_logprobs on
the same input (|delta logp| <= 2e-3 is the bar; the two are expected to agree bit for bit) and
with the CPU oracle on sampled rows."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import mrl_oracle as orc
from tests import util

pytestmark = pytest.mark.gpu


def _inputs(N, d, V, seed, dtype=torch.bfloat16):
    g = torch.Generator("cuda").manual_seed(seed)
    H = torch.randn((N, d), device="cuda", generator=g).to(dtype)
    W = (0.02 * torch.randn((V, d), device="cuda", generator=g)).to(dtype)
    y = torch.randint(0, V, (N,), device="cuda", generator=g, dtype=torch.int64).int()
    mask = (torch.rand(N, device="cuda", generator=g) < 0.8).to(torch.uint8)
    return H, W, y, mask


def _raw_static_call(mrl, H, W, y, mask, out_logp, out_lse):
    """Straight through ctypes: raw device pointers and sizes, nothing else."""
    L = mrl.lib()
    N, d = H.shape
    return L.mrl_token_logprobs_static(ctypes.c_void_p(H.data_ptr()), ctypes.c_void_p(W.data_ptr()),
                                       ctypes.c_void_p(y.data_ptr()), ctypes.c_void_p(mask.data_ptr()),
                                       N, d, W.shape[0], mrl.BF16 if H.dtype == torch.bfloat16 else mrl.F32,
                                       ctypes.c_void_p(out_logp.data_ptr()), ctypes.c_void_p(out_lse.data_ptr()),
                                       ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


def test_static_entry_point_matches_workspace_variant_twice_in_a_row():
    import paper_2605_07244_amd as mrl
    cases = [(5000, 256, 5003, 11),       # 20 passes' worth of rows in one 5120-row pass, ragged vocabulary tile
             (700, 128, 1200, 12)]        # smaller input afterwards: stale scratch contents beyond it must not matter
    for N, d, V, seed in cases:
        H, W, y, mask = _inputs(N, d, V, seed)
        want_lp, want_lse = mrl.token_logprobs(H, W, y, mask)
        got_lp = torch.full((N,), 7.0, dtype=torch.float32, device="cuda")
        got_lse = torch.full((N,), 7.0, dtype=torch.float32, device="cuda")
        rc = _raw_static_call(mrl, H, W, y, mask, got_lp, got_lse)
        assert rc == 0, mrl.status_string(rc)
        torch.cuda.synchronize()
        m = mask.bool()
        assert float((got_lp - want_lp).abs().max()) <= util.LOGP_TOL
        assert float((got_lse - want_lse).abs().max()) <= util.LOGP_TOL
        assert torch.equal(got_lp, want_lp) and torch.equal(got_lse, want_lse)
        assert torch.all(got_lp[~m] == 0) and torch.all(got_lse[~m] == 0)
        # and against the oracle on a sample of scored rows
        rows = torch.nonzero(m)[:, 0][:: max(1, int(m.sum()) // 64)]
        lp_o, lse_o = orc.token_logprobs(util.to_f64(H[rows]), util.to_f64(W), y[rows].cpu().numpy())
        assert np.max(np.abs(got_lp[rows].cpu().numpy() - lp_o)) <= util.LOGP_TOL
        assert np.max(np.abs(got_lse[rows].cpu().numpy() - lse_o)) <= util.LOGP_TOL


def test_static_entry_point_fp32_and_binding():
    import paper_2605_07244_amd as mrl
    H, W, y, mask = _inputs(300, 72, 777, 13, dtype=torch.float32)
    want_lp, want_lse = mrl.token_logprobs(H, W, y, mask)
    got_lp = torch.empty(300, dtype=torch.float32, device="cuda")
    got_lse = torch.empty(300, dtype=torch.float32, device="cuda")
    mrl.token_logprobs_static(H, W, y, mask, got_lp, got_lse)
    torch.cuda.synchronize()
    assert torch.equal(got_lp, want_lp) and torch.equal(got_lse, want_lse)


def test_static_entry_point_rejects_inputs_beyond_its_buffer():
    import paper_2605_07244_amd as mrl
    H, W, y, mask = _inputs(256, 128, 1024, 14)
    out = torch.empty(256, dtype=torch.float32, device="cuda")
    L = mrl.lib()
    # 8 bytes per row alone exceed the 32 MiB buffer: refused on the host, nothing launched
    rc = L.mrl_token_logprobs_static(ctypes.c_void_p(H.data_ptr()), ctypes.c_void_p(W.data_ptr()),
                                     ctypes.c_void_p(y.data_ptr()), None, 1 << 23, 128, 1024, mrl.BF16,
                                     ctypes.c_void_p(out.data_ptr()), None, None)
    assert rc == -10 and "scratch" in mrl.status_string(rc)
