"""CPU oracle for the THL word-level trace alignment (TEST INFRASTRUCTURE, not the product).

The tokenizer-heterogeneity layer carries a source model's per-token log-probabilities over
to the target model's token grid through the words both tokenizations share (Sec. 4.3):

    Z_w        = sum over source response tokens s that belong to word w of  l_src[s]
    C_w        = number of target response tokens that belong to word w
    l_tilde[t] = Z_w(t) / max(1, C_w(t))        for a target response token t of word w(t)

(Thm. 1 calls a response token valid when the response mask includes it and the word map
assigns it a word; every other position carries no aligned value.)  This module evaluates that
definition with word-membership indicator matrices, one sequence at a time in fp64: the sums
over "tokens of word w" are literally rows of a 0/1 matrix times the log-prob vector.  Building
the word maps themselves (word spans, incremental tokenisation; App. D, Alg. 1 and 3) needs
tokenizers and text and is outside the hot path.

Conventions for the cases the definition leaves open, as stated properties:
  * a word map lists one entry per response token, in order; when the map and the response
    mask disagree in length, only the first min(#response tokens, map length) tokens are valid
    (App. D pairs map entries with response positions one to one);
  * map entry -1 marks a token that belongs to no word (a leading delimiter);
  * a target word no source token belongs to has Z_w = 0, so its tokens receive 0;
  * a sequence whose source side has no valid token at all yields no aligned trace: every
    position keeps `ignore_value`;
  * every position that is not a valid target token keeps `ignore_value`.

Only tests, the smoke check and the bench's CPU-baseline leg may import this module; it shares
no code with the HIP path.

Parity status: pinned by tests/test_thl_oracle_pins.py (a hand-worked instance, per-word
conservation and the residual identity of Thm. 1, an independent evaluation by per-token
loops, identity under equal segmentations, the ratio envelope of the corollary to Thm. 1).
"""
from __future__ import annotations

import numpy as np

NONE = -1   # map entry of a token that belongs to no word


def _valid_tokens(mask_row, map_row, map_len):
    """Positions of the valid response tokens of one sequence and the word of each."""
    pos = np.flatnonzero(np.asarray(mask_row) != 0)
    n = min(pos.size, int(map_len))
    words = np.asarray(map_row[:n], dtype=np.int64)
    has_word = words != NONE
    return pos[:n][has_word], words[has_word]


def _membership(words, n_words):
    """0/1 matrix [n_words, n_tokens]: entry (w, k) is 1 when token k belongs to word w."""
    return (words[None, :] == np.arange(n_words, dtype=np.int64)[:, None]).astype(np.float64)


def word_align_logprobs(source_log_probs, source_response_mask, src_word_map, src_map_len,
                        target_response_mask, tgt_word_map, tgt_map_len, ignore_value):
    """Word-level trace alignment of Sec. 4.3 on integer word maps.

    source_log_probs      [B, S_src] float
    source_response_mask  [B, S_src] 0/1
    src_word_map          [B, S_src] int; entry p (p < src_map_len[i]) is the word of the p-th
                          response token of sequence i, or NONE
    src_map_len           [B] int
    target_*              likewise on the target grid
    Returns l_tilde [B, S_tgt] float64, `ignore_value` wherever no aligned value is defined.
    """
    l_src = np.asarray(source_log_probs, dtype=np.float64)
    tgt_mask = np.asarray(target_response_mask)
    aligned = np.full(tgt_mask.shape, float(ignore_value), dtype=np.float64)
    for i in range(l_src.shape[0]):
        s_pos, s_word = _valid_tokens(source_response_mask[i], src_word_map[i], src_map_len[i])
        t_pos, t_word = _valid_tokens(tgt_mask[i], tgt_word_map[i], tgt_map_len[i])
        if s_pos.size == 0 or t_pos.size == 0:
            continue
        n_words = int(max(s_word.max(), t_word.max())) + 1
        in_src = _membership(s_word, n_words)            # [n_words, valid source tokens]
        in_tgt = _membership(t_word, n_words)            # [n_words, valid target tokens]
        Z = in_src @ l_src[i, s_pos]                     # word mass
        C = in_tgt.sum(axis=1)                           # target tokens per word
        aligned[i, t_pos] = in_tgt.T @ (Z / np.maximum(1.0, C))
    return aligned
