"""Pins of the THL alignment oracle (Sec. 4.3 formula; App. D) against what the paper and the
mathematics fix.  None of these tests touches the HIP path."""
import os

import numpy as np
import pytest

from oracle import thl_oracle as thl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
IGN = -100.0


def _random_case(seed, B=5, S_src=40, S_tgt=48, p_none=0.1, drop_words=True, truncate=True):
    """Random word maps with the structure the method meets: a prompt prefix outside the
    response mask, words split into 1..3 tokens on either side, some None entries, some words
    missing on one side, maps shorter than the mask (tokenization drift) or longer."""
    rng = np.random.default_rng(seed)
    src_lp = -rng.gamma(1.0, 1.0, size=(B, S_src))
    src_m = np.zeros((B, S_src), dtype=np.int64)
    tgt_m = np.zeros((B, S_tgt), dtype=np.int64)
    src_map = np.full((B, S_src), thl.NONE, dtype=np.int64)
    tgt_map = np.full((B, S_tgt), thl.NONE, dtype=np.int64)
    src_len = np.zeros(B, dtype=np.int64)
    tgt_len = np.zeros(B, dtype=np.int64)
    for i in range(B):
        n_words = int(rng.integers(0, 12))
        for (m, mp, ln, S) in ((src_m, src_map, src_len, S_src), (tgt_m, tgt_map, tgt_len, S_tgt)):
            words = []
            for w in range(n_words):
                if drop_words and rng.random() < 0.1:
                    continue
                words += [w] * int(rng.integers(1, 4))
            words = [thl.NONE] * int(rng.integers(0, 2)) + words
            words = [thl.NONE if rng.random() < p_none else w for w in words]
            pre = int(rng.integers(0, 5))
            words = words[: S - pre]
            n_resp = len(words)
            if truncate and n_resp > 2:
                n_resp += int(rng.integers(-2, 3))       # mask longer or shorter than the map
                n_resp = max(0, min(n_resp, S - pre))
            m[i, pre:pre + n_resp] = 1
            mp[i, :len(words)] = words
            ln[i] = len(words)
    return src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len


def _valid_tokens(mask_row, map_row, map_len):
    idx = np.nonzero(mask_row == 1)[0]
    L = min(len(idx), int(map_len))
    return idx[:L], np.asarray(map_row[:L])


def test_hand_worked_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "thl_worked_alignment.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = np.array([float(x) for x in v])
    out = thl.word_align_logprobs(rows["src_logp"][None], rows["src_mask"][None].astype(int),
                                  rows["src_word_map"][None].astype(int), [7],
                                  rows["tgt_mask"][None].astype(int), rows["tgt_word_map"][None].astype(int), [7],
                                  IGN)
    assert np.array_equal(out[0], rows["expected"])


@pytest.mark.parametrize("seed", range(6))
def test_word_mass_is_conserved(seed):
    """Thm. 1: for each word with C_w > 0 the aligned values of its target tokens add up to the
    sum of its source log-probs."""
    src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len = _random_case(seed)
    out = thl.word_align_logprobs(src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len, IGN)
    for i in range(src_lp.shape[0]):
        sidx, sw = _valid_tokens(src_m[i], src_map[i], src_len[i])
        tidx, tw = _valid_tokens(tgt_m[i], tgt_map[i], tgt_len[i])
        if not np.any(sw != thl.NONE):
            assert np.all(out[i] == IGN)
            continue
        for w in set(tw.tolist()) - {thl.NONE}:
            Z = src_lp[i, sidx[sw == w]].sum()
            assert abs(out[i, tidx[tw == w]].sum() - Z) < 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_sequence_residual_identity(seed):
    """Thm. 1: (masked source sequence log-prob) - (sum of the aligned values outside
    ignore positions) = R_THL = log-probs of source tokens without a word + totals of the
    words that have source tokens but no target token."""
    src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len = _random_case(seed + 100)
    out = thl.word_align_logprobs(src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len, IGN)
    for i in range(src_lp.shape[0]):
        all_src = np.nonzero(src_m[i] == 1)[0]
        sidx, sw = _valid_tokens(src_m[i], src_map[i], src_len[i])
        tidx, tw = _valid_tokens(tgt_m[i], tgt_map[i], tgt_len[i])
        if not np.any(sw != thl.NONE):
            continue
        L_mu = src_lp[i, all_src].sum()
        L_tilde = out[i][out[i] != IGN].sum()
        tgt_words = set(tw.tolist()) - {thl.NONE}
        R = src_lp[i, all_src[len(sidx):]].sum()                 # response tokens beyond the map
        R += sum(src_lp[i, j] for j, w in zip(sidx, sw) if w == thl.NONE or w not in tgt_words)
        assert abs((L_mu - L_tilde) - R) < 1e-12
        # and its bound: |R| <= sum of |l| over the unplaced tokens
        assert abs(R) <= sum(abs(src_lp[i, j]) for j, w in zip(sidx, sw)
                             if w == thl.NONE or w not in tgt_words) + np.abs(src_lp[i, all_src[len(sidx):]]).sum() + 1e-12


@pytest.mark.parametrize("seed", range(4))
def test_closed_formula_vectorised(seed):
    """Sec. 4.3: aligned value = m_t * Z_{w(t)} / max(1, C_{w(t)}), evaluated with histogram
    sums (bincount) instead of the oracle's indicator-matrix products."""
    src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len = _random_case(seed + 200)
    out = thl.word_align_logprobs(src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len, IGN)
    for i in range(src_lp.shape[0]):
        sidx, sw = _valid_tokens(src_m[i], src_map[i], src_len[i])
        tidx, tw = _valid_tokens(tgt_m[i], tgt_map[i], tgt_len[i])
        expect = np.full(tgt_m.shape[1], IGN)
        if np.any(sw != thl.NONE):
            nw = int(max(sw.max(initial=0), tw.max(initial=0))) + 1
            Z = np.bincount(sw[sw >= 0], weights=src_lp[i, sidx[sw >= 0]], minlength=nw)
            C = np.bincount(tw[tw >= 0], minlength=nw)
            has = tw >= 0
            expect[tidx[has]] = Z[tw[has]] / np.maximum(1, C[tw[has]])
        assert np.allclose(out[i], expect, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", range(3))
def test_per_token_brute_force(seed):
    """For every target position separately: scan all source positions for tokens of the same word
    (Z), scan all target positions for tokens of the same word (C).  Quadratic, no shared
    bookkeeping between positions, walks the masks position by position."""
    src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len = _random_case(seed + 300, B=4, S_src=24, S_tgt=30)
    out = thl.word_align_logprobs(src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len, IGN)

    def word_at(mask_row, map_row, map_len, pos):
        """Word of the token at `pos`, or None when it is not a valid response token."""
        if mask_row[pos] != 1:
            return None
        rank = int(np.sum(mask_row[:pos] == 1))          # it is the rank-th response token
        if rank >= map_len or map_row[rank] == thl.NONE:
            return None
        return int(map_row[rank])

    for i in range(src_lp.shape[0]):
        src_words = [word_at(src_m[i], src_map[i], src_len[i], s) for s in range(src_m.shape[1])]
        any_source = any(w is not None for w in src_words)
        for t in range(tgt_m.shape[1]):
            w = word_at(tgt_m[i], tgt_map[i], tgt_len[i], t)
            if w is None or not any_source:
                assert out[i, t] == IGN
                continue
            Z = sum(src_lp[i, s] for s in range(src_m.shape[1]) if src_words[s] == w)
            C = sum(1 for u in range(tgt_m.shape[1]) if word_at(tgt_m[i], tgt_map[i], tgt_len[i], u) == w)
            assert abs(out[i, t] - Z / max(1, C)) < 1e-12


def test_equal_segmentations_give_the_source_trace_back():
    rng = np.random.default_rng(5)
    S = 30
    lp = -rng.gamma(1.0, 1.0, size=(2, S))
    m = np.zeros((2, S), dtype=np.int64)
    m[0, 3:25] = 1
    m[1, 0:17] = 1
    wmap = np.full((2, S), thl.NONE, dtype=np.int64)
    wmap[0, :22] = np.arange(22)            # one token per word
    wmap[1, :17] = np.arange(17)
    out = thl.word_align_logprobs(lp, m, wmap, [22, 17], m, wmap, [22, 17], IGN)
    assert np.array_equal(out[m == 1], lp[m == 1])
    assert np.all(out[m == 0] == IGN)


def test_one_target_token_per_word_receives_the_word_total():
    lp = np.array([[-0.5, -0.25, -0.125, -1.0, -2.0, 0.0]])
    m_src = np.array([[1, 1, 1, 1, 1, 0]])
    src_map = np.array([[0, 0, 0, 1, 1, -1]])
    m_tgt = np.array([[0, 1, 1, 0]])
    tgt_map = np.array([[0, 1, -1, -1]])
    out = thl.word_align_logprobs(lp, m_src, src_map, [5], m_tgt, tgt_map, [2], IGN)
    assert np.array_equal(out, [[IGN, -0.875, -3.0, IGN]])


def test_maps_are_indexed_by_response_token_not_by_position():
    """The p-th map entry belongs to the p-th position of the response mask (Alg. 2,
    src_idx / tgt_idx), whatever prefix precedes the response."""
    lp = np.array([[7.0, 7.0, 7.0, -1.0, -2.0]])
    m_src = np.array([[0, 0, 0, 1, 1]])
    src_map = np.array([[0, 1, -1, -1, -1]])
    m_tgt = np.array([[0, 0, 1, 1, 1]])
    tgt_map = np.array([[1, 0, 0, -1, -1]])
    out = thl.word_align_logprobs(lp, m_src, src_map, [2], m_tgt, tgt_map, [3], IGN)
    assert np.array_equal(out, [[IGN, IGN, -2.0, -0.5, -0.5]])


def test_truncation_to_the_shorter_of_mask_and_map():
    lp = np.array([[-1.0, -2.0, -4.0, -8.0]])
    m_src = np.array([[1, 1, 1, 1]])
    src_map = np.array([[0, 0, 1, 1]])
    m_tgt = np.array([[1, 1, 1, 0]])
    tgt_map = np.array([[0, 1, 1, 1]])
    # source map shorter than the mask: the last source token is not counted
    out = thl.word_align_logprobs(lp, m_src, src_map, [3], m_tgt, tgt_map, [4], IGN)
    assert np.array_equal(out, [[-3.0, -2.0, -2.0, IGN]])
    # target map shorter than the mask: the last response position stays ignore_value and
    # does not count in C_w
    out = thl.word_align_logprobs(lp, m_src, src_map, [4], m_tgt, tgt_map, [2], IGN)
    assert np.array_equal(out, [[-3.0, -12.0, IGN, IGN]])


def test_source_without_any_word_leaves_the_row_inactive():
    lp = np.array([[-1.0, -2.0]])
    out = thl.word_align_logprobs(lp, np.array([[1, 1]]), np.array([[-1, -1]]), [2],
                                  np.array([[1, 1]]), np.array([[0, 1]]), [2], IGN)
    assert np.all(out == IGN)
    out = thl.word_align_logprobs(lp, np.array([[0, 0]]), np.array([[0, 1]]), [2],
                                  np.array([[1, 1]]), np.array([[0, 1]]), [2], IGN)
    assert np.all(out == IGN)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_aligned_denominator_ratio_envelope(seed):
    """Cor. "Importance-ratio envelope induced by THL" (App. I): the response-level ratio taken
    against the aligned trace is rho * exp(R) with R = L_mu - L~_mu, the source log-prob mass of
    words without target tokens and of tokens without a word; exact refinement gives R = 0.
    Ties the alignment oracle to the loss oracle: the aligned trace goes in as behaviour log-probs
    of the target grid (positions left at ignore_value are masked out) and rho~ is read off the
    surrogate of a single response with a unit advantage and an inactive clip."""
    from oracle import mrl_oracle as orc
    src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len = _random_case(40 + seed, B=6, truncate=False)
    aligned = thl.word_align_logprobs(src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len, IGN)
    rng = np.random.default_rng(seed)
    cfg = dict(orc.default_config(), clip_eps_low=1.0, clip_eps_high=1e30, kl_beta=0.0, ratio_level=1)
    checked = 0
    for i in range(src_lp.shape[0]):
        s_idx, s_w = _valid_tokens(src_m[i], src_map[i], src_len[i])
        t_idx, t_w = _valid_tokens(tgt_m[i], tgt_map[i], tgt_len[i])
        tok_mask = (tgt_m[i] == 1) & (aligned[i] != IGN)
        if not tok_mask.any():
            continue
        T = tgt_m.shape[1]
        logp = -rng.gamma(1.0, 0.3, size=T)                 # the learner's log-probs on the target grid
        out = orc.loss_from_logp(logp, tok_mask[None, :], aligned[i], None, np.array([1.0]), np.array([0]),
                                 None, 1, T, 1, cfg)
        rho_tilde = -out["loss_pg"]                          # one response, A = 1, c sums to 1
        L_theta = logp[tok_mask].sum()
        # ideal ratio: the whole source trace as denominator
        L_mu = src_lp[i, s_idx].sum()
        rho = np.exp(L_theta - L_mu)
        # residual by its definition: words nobody receives on the target side, tokens without a word
        tgt_words = set(int(w) for w in t_w if w != thl.NONE)
        R = sum(src_lp[i, s_idx[p]] for p in range(len(s_idx))
                if s_w[p] == thl.NONE or int(s_w[p]) not in tgt_words)
        assert abs(np.log(rho_tilde) - (np.log(rho) + R)) < 1e-10
        n_mis = sum(1 for p in range(len(s_idx)) if s_w[p] == thl.NONE or int(s_w[p]) not in tgt_words)
        bound = np.max(np.abs(src_lp[i, s_idx])) if len(s_idx) else 0.0
        assert abs(R) <= bound * n_mis + 1e-12
        assert np.exp(-abs(R)) * rho * (1 - 1e-12) <= rho_tilde <= np.exp(abs(R)) * rho * (1 + 1e-12)
        checked += 1
    assert checked >= 3
    # exact refinement: same words on both sides, nothing unmapped => rho~ = rho
    src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len = _random_case(50 + seed, B=4, p_none=0.0,
                                                                            drop_words=False, truncate=False)
    aligned = thl.word_align_logprobs(src_lp, src_m, src_map, src_len, tgt_m, tgt_map, tgt_len, IGN)
    for i in range(4):
        s_idx, s_w = _valid_tokens(src_m[i], src_map[i], src_len[i])
        tok_mask = (tgt_m[i] == 1) & (aligned[i] != IGN)
        if not tok_mask.any() or np.any(s_w == thl.NONE):
            continue
        assert abs(aligned[i][tok_mask].sum() - src_lp[i, s_idx].sum()) < 1e-10
