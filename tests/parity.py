"""Acceptance rule used by the GPU parity tests (helper, not a test module).

Ids must equal the oracle's, rank by rank, except where the oracle itself sees a near-tie:
a different id is accepted at rank j only if the ORACLE's score of the returned row is
within 1e-5 relative of the oracle's rank-j score.  Every returned score must be within 1e-4
relative of the oracle's score of the row that was returned, and a row may not repeat ids.
"""
import numpy as np

ID_TIE_RTOL = 1e-5
SCORE_RTOL = 1e-4


def check_topk(got_ids, got_scores, want_ids, want_scores, oracle_score_of):
    """oracle_score_of(i, ids) -> oracle scores (fp32) of rows `ids` for query i.
    Returns (exact_rank_matches, near_tie_substitutions, total)."""
    got_ids, got_scores = np.asarray(got_ids), np.asarray(got_scores)
    want_ids, want_scores = np.asarray(want_ids), np.asarray(want_scores)
    assert got_ids.shape == want_ids.shape, (got_ids.shape, want_ids.shape)
    Q, k = want_ids.shape
    exact = subs = 0
    for i in range(Q):
        assert len(set(got_ids[i].tolist())) == k, f"query {i}: duplicate ids {got_ids[i]}"
        same = got_ids[i] == want_ids[i]
        exact += int(same.sum())
        mine = oracle_score_of(i, got_ids[i]) if not same.all() else want_scores[i]
        mine = np.where(same, want_scores[i], mine)
        denom = np.maximum(np.abs(want_scores[i]), 1e-30)
        bad = (~same) & (np.abs(mine - want_scores[i]) / denom > ID_TIE_RTOL)
        assert not bad.any(), (f"query {i}: ids differ beyond a near-tie at ranks {np.nonzero(bad)[0]}: "
                               f"got {got_ids[i][bad]} want {want_ids[i][bad]}")
        subs += int((~same).sum())
        rel = np.abs(got_scores[i] - mine) / np.maximum(np.abs(mine), 1e-30)
        assert (rel <= SCORE_RTOL).all(), f"query {i}: score error {rel.max()}"
    return exact, subs, Q * k
