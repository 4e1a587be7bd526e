"""CPU oracle for the THL word-level trace alignment (TEST INFRASTRUCTURE, not the product).

The tokenizer-heterogeneity layer maps a source model's per-token log-probabilities
onto the target model's token positions: source log-probs are summed per textual
word and each word total is spread evenly over the target tokens of that word
(Sec. 4.3; App. D, "THL WordAlignLogProbs", Alg. 2).  This module is the
redistribution part of that routine on integer word maps; producing the maps
(regular-expression spans and incremental tokenization, Alg. 1 and Alg. 3) needs
tokenizers and text and is outside the hot path.

The implementation takes the algorithm's steps in the paper's order and notation,
with plain Python loops and dictionaries (small cases only).  Only tests, the
smoke check and the bench's CPU-baseline leg may import it; it shares no code
with the HIP path.

Parity status: pinned by tests/test_thl_oracle_pins.py (conservation of Thm. 1,
the residual identity of Thm. 1, the closed formula of Sec. 4.3 evaluated by an
independent vectorised routine, identity under equal segmentations, a
hand-worked example, brute force).
"""
from __future__ import annotations

import numpy as np

NONE = -1   # "None" entries of a word map (leading delimiter tokens, App. D)


def word_align_logprobs(source_log_probs, source_response_mask, src_word_map, src_map_len,
                        target_response_mask, tgt_word_map, tgt_map_len, ignore_value):
    """Alg. 2 (App. D) on integer word maps.

    source_log_probs      [B, S_src] float
    source_response_mask  [B, S_src] 0/1
    src_word_map          [B, S_src] int; entry p (p < src_map_len[i]) is the word index of
                          the p-th response token of sequence i, or NONE
    src_map_len           [B] int, the length |src_ids| of the map of sequence i
    target_*              likewise on the target grid
    Returns out [B, S_tgt] float64: ignore_value everywhere except at the target response
    positions that carry a word, which get (sum of the word's source log-probs) / (number
    of target tokens of the word); a word no source token maps to has sum 0.
    A sequence whose source side has no token with a word stays all ignore_value.
    """
    src_lp = np.asarray(source_log_probs, dtype=np.float64)
    src_m = np.asarray(source_response_mask)
    tgt_m = np.asarray(target_response_mask)
    B = src_lp.shape[0]
    out = np.full(tgt_m.shape, float(ignore_value), dtype=np.float64)
    for i in range(B):
        src_idx = [j for j in range(src_m.shape[1]) if src_m[i, j] == 1]
        tgt_idx = [j for j in range(tgt_m.shape[1]) if tgt_m[i, j] == 1]
        L_src = min(len(src_idx), int(src_map_len[i]))
        L_tgt = min(len(tgt_idx), int(tgt_map_len[i]))
        per_word_sum = {}
        for p in range(L_src):
            wid = int(src_word_map[i][p])
            if wid == NONE:
                continue
            per_word_sum[wid] = per_word_sum.get(wid, 0.0) + src_lp[i, src_idx[p]]
        if not per_word_sum:
            continue
        per_word_count = {}
        for p in range(L_tgt):
            wid = int(tgt_word_map[i][p])
            if wid == NONE:
                continue
            per_word_count[wid] = per_word_count.get(wid, 0) + 1
        for p in range(L_tgt):
            wid = int(tgt_word_map[i][p])
            if wid == NONE:
                continue
            cnt = per_word_count.get(wid, 0)
            if cnt <= 0:
                continue
            out[i, tgt_idx[p]] = per_word_sum.get(wid, 0.0) / cnt
    return out

