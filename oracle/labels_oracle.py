"""CPU oracle for the construction of syntax-enriched training labels (plain Python / NumPy).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the tests and the benchmark's CPU-baseline
leg may import it. It shares no code with the HIP path and never imports it.

What it computes (Section III-C, Fig. 3 of the paper):
  * L_0, the base model's label row, is the tokenised code with a [FRAG] id inserted at every
    fragment boundary; it has sequence_length entries;
  * the label row of head i is L_0 shifted left by i, L_i = L_0[i:], filled up with [PAD] to
    the same length; the rows 0..num_heads stacked give Labels, (num_heads + 1) x
    sequence_length;
  * per sequence position s (a column of Labels), find the last row that holds [FRAG]; every
    label of that column in a later row is replaced by [IGNORE], so that what remains of a
    column is a run of complete fragments.
The functions below take those steps in that order, one column at a time, with loops.

Readings of what the paper leaves open:
  * the [FRAG] entry itself is kept (only labels BEYOND it are replaced);
  * a column that holds no [FRAG] at all: "keep_base" keeps row 0 and ignores every head row
    (the base model is trained on every token, the heads only on complete fragments);
    "keep_all" leaves the column as it is. "keep_base" is the default;
  * [PAD] entries are ordinary values: they are replaced when they lie beyond the last [FRAG]
    and kept otherwise (only possible under "keep_all");
  * several sequences are independent rows of a batch.

Parity pins (tests/test_oracle_labels.py): hand-worked cases (tests/golden/label_cases.json),
an element-wise restatement (an entry survives iff a [FRAG] sits at or after it within the
window), the monotone growth of the ignored share with the head index that Section III-C
states, degenerate inputs (no heads, no [FRAG], only [FRAG]), and a vectorised
reverse-cumulative formulation.
"""
from __future__ import annotations

import numpy as np

NO_FRAG_POLICIES = ("keep_base", "keep_all")


def shifted_labels(l0: np.ndarray, num_heads: int, pad_id: int) -> np.ndarray:
    """Rows L_i = L_0[i:] + [PAD] * i for i = 0..num_heads (Section III-C)."""
    l0 = np.asarray(l0)
    S = l0.shape[0]
    labels = np.full((num_heads + 1, S), pad_id, dtype=np.int32)
    for i in range(num_heads + 1):
        for s in range(S - i):
            labels[i, s] = l0[s + i]
    return labels


def syntax_enriched_labels(l0: np.ndarray, num_heads: int, frag_id: int, pad_id: int, ignore_id: int,
                           no_frag: str = "keep_base") -> np.ndarray:
    """Labels of one sequence, (num_heads + 1) x sequence_length (Section III-C, Fig. 3)."""
    if no_frag not in NO_FRAG_POLICIES:
        raise ValueError(no_frag)
    labels = shifted_labels(l0, num_heads, pad_id)
    S = labels.shape[1]
    for s in range(S):
        last = -1
        for i in range(num_heads + 1):
            if labels[i, s] == frag_id:
                last = i
        if last < 0:
            if no_frag == "keep_all":
                continue
            last = 0
        for i in range(last + 1, num_heads + 1):
            labels[i, s] = ignore_id
    return labels


def syntax_enriched_labels_batch(l0: np.ndarray, num_heads: int, frag_id: int, pad_id: int, ignore_id: int,
                                 no_frag: str = "keep_base") -> np.ndarray:
    """[batch, seq] -> [batch, num_heads + 1, seq]; sequences are independent."""
    return np.stack([syntax_enriched_labels(row, num_heads, frag_id, pad_id, ignore_id, no_frag) for row in l0])
