"""Pins for the label-construction oracle (Section III-C): things other than itself."""
import json
import os

import numpy as np
import pytest

import workload as wl
from oracle import labels_oracle as lab

HERE = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(HERE, "golden", "label_cases.json")) as f:
    GOLD = json.load(f)
F, P, X = GOLD["frag_id"], GOLD["pad_id"], GOLD["ignore_id"]


@pytest.mark.parametrize("case", GOLD["cases"], ids=[c["name"] for c in GOLD["cases"]])
@pytest.mark.parametrize("policy", lab.NO_FRAG_POLICIES)
def test_hand_worked_cases(case, policy):
    got = lab.syntax_enriched_labels(np.array(case["l0"]), case["num_heads"], F, P, X, policy)
    assert got.tolist() == case[policy]


def _random_l0(rng, S, p_frag):
    l0 = rng.integers(0, 50, size=S)
    l0[rng.random(S) < p_frag] = F
    return l0.astype(np.int32)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("policy", lab.NO_FRAG_POLICIES)
def test_elementwise_restatement(seed, policy):
    """Entry (i, s) survives iff some [FRAG] sits at l0[s + j] with i <= j <= H inside the sequence;
    survivors equal the shifted label. Columns without any [FRAG] follow the policy."""
    rng = np.random.default_rng(seed)
    S, H = int(rng.integers(1, 40)), int(rng.integers(0, 7))
    l0 = _random_l0(rng, S, [0.0, 0.1, 0.3, 0.6, 0.9, 1.0][seed])
    got = lab.syntax_enriched_labels(l0, H, F, P, X, policy)
    assert got.shape == (H + 1, S)
    for s in range(S):
        window = [int(l0[s + j]) if s + j < S else P for j in range(H + 1)]
        has_frag = F in window
        for i in range(H + 1):
            survives = any(window[j] == F for j in range(i, H + 1))
            if not has_frag:
                survives = True if policy == "keep_all" else i == 0
            assert got[i, s] == (window[i] if survives else X), (s, i)


def test_ignored_share_grows_with_the_head_index():
    """Section III-C: later heads see a larger proportion of [IGNORE]."""
    l0 = wl.frag_filled_labels(4, 2048, 32000, 31999, 31998)
    for row in l0:
        lab_ = lab.syntax_enriched_labels(row, 10, 31999, 31998, X)
        share = (lab_ == X).mean(axis=1)
        assert share[0] == 0.0 and np.all(np.diff(share) >= 0) and share[-1] > share[1] > 0
        # with fragments of mean length 4 plus the marker, head 1 loses roughly the columns whose base label is
        # itself a [FRAG] or that hold none in the window: between a tenth and a half
        assert 0.1 < share[1] < 0.5
        assert np.array_equal(lab_[0], row)


def test_degenerate_inputs():
    l0 = np.array([5, 6, 7, 8], np.int32)
    assert lab.syntax_enriched_labels(l0, 0, F, P, X).tolist() == [l0.tolist()]             # no heads: Labels = L0
    none = lab.syntax_enriched_labels(l0, 3, F, P, X)
    assert np.array_equal(none[0], l0) and (none[1:] == X).all()                             # no [FRAG]: heads ignored
    assert np.array_equal(lab.syntax_enriched_labels(l0, 3, F, P, X, "keep_all"), lab.shifted_labels(l0, 3, P))
    allf = np.full(5, F, np.int32)
    got = lab.syntax_enriched_labels(allf, 2, F, P, X)
    # window (F, F, F) keeps everything; the last two columns run into [PAD], which lies beyond the last [FRAG]
    assert got.tolist() == [[F] * 5, [F, F, F, F, X], [F, F, F, X, X]]
    assert lab.syntax_enriched_labels(np.zeros(0, np.int32), 2, F, P, X).shape == (3, 0)
    with pytest.raises(ValueError):
        lab.syntax_enriched_labels(l0, 1, F, P, X, "other")


@pytest.mark.parametrize("seed", range(4))
def test_vectorised_reverse_cumulative_formulation(seed):
    """Survival mask = reverse cumulative OR of (shifted == [FRAG]) along the head axis."""
    rng = np.random.default_rng(100 + seed)
    S, H = 300, 5
    l0 = _random_l0(rng, S, 0.2)
    shifted = lab.shifted_labels(l0, H, P)
    isf = shifted == F
    surv = np.flip(np.logical_or.accumulate(np.flip(isf, 0), 0), 0)
    nof = ~isf.any(0)
    surv_base = surv.copy()
    surv_base[0, nof] = True
    assert np.array_equal(lab.syntax_enriched_labels(l0, H, F, P, X), np.where(surv_base, shifted, X))
    surv_all = surv.copy()
    surv_all[:, nof] = True
    assert np.array_equal(lab.syntax_enriched_labels(l0, H, F, P, X, "keep_all"), np.where(surv_all, shifted, X))


def test_shift_matches_numpy_roll_with_padding():
    l0 = np.arange(10, 20, dtype=np.int32)
    sh = lab.shifted_labels(l0, 4, P)
    for i in range(5):
        want = np.concatenate([l0[i:], np.full(i, P, np.int32)])
        assert np.array_equal(sh[i], want)


def test_batch_rows_are_independent():
    l0 = wl.frag_filled_labels(3, 64, 100, 99, 98)
    got = lab.syntax_enriched_labels_batch(l0, 4, 99, 98, X)
    assert got.shape == (3, 5, 64)
    for b in range(3):
        assert np.array_equal(got[b], lab.syntax_enriched_labels(l0[b], 4, 99, 98, X))


def test_generator_shape():
    l0 = wl.frag_filled_labels(8, 512, 32000, 31999, 31998)
    assert l0.shape == (8, 512) and l0.dtype == np.int32
    for row in l0:
        n = int((row != 31998).sum())
        assert 256 <= n <= 512 and (row[n:] == 31998).all()
        frag_share = (row[:n] == 31999).mean()
        assert 0.12 < frag_share < 0.3                       # one marker per ~4-token fragment
    assert np.array_equal(l0, wl.frag_filled_labels(8, 512, 32000, 31999, 31998))
