"""GPU parity of the syntax-enriched label construction (Section III-C), bit-exact against the oracle."""
import json
import os

import numpy as np
import pytest
import torch

import workload as wl
from oracle import labels_oracle as lab

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
X = -100


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()                       # fails loudly if the library has not been built
    return sd


def _gpu(sd, l0, H, frag, pad, policy):
    out = sd.build_labels(torch.from_numpy(np.ascontiguousarray(l0)).cuda(), H, frag, pad, X, policy)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("policy", lab.NO_FRAG_POLICIES)
def test_hand_worked_cases(sd, policy):
    with open(os.path.join(HERE, "golden", "label_cases.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        l0 = np.array([case["l0"]], np.int32)
        got = _gpu(sd, l0, case["num_heads"], gold["frag_id"], gold["pad_id"], policy)
        assert got[0].tolist() == case[policy], case["name"]


@pytest.mark.parametrize("S", [1, 5, 1023, 1024, 1025, 3000])
@pytest.mark.parametrize("H,batch", [(0, 2), (1, 3), (4, 5), (10, 2), (64, 1)])
def test_ragged_shapes_bit_exact(sd, S, H, batch):
    """Sequence lengths around the 1024-column tile, head counts up to the limit, both policies."""
    rng = np.random.default_rng(S * 100 + H)
    l0 = rng.integers(0, 60, size=(batch, S)).astype(np.int32)
    l0[rng.random((batch, S)) < rng.choice([0.02, 0.2, 0.7], size=(batch, 1))] = 7        # 7 = [FRAG]
    l0[0, S // 2:] = 9 if S > 1 else l0[0, S // 2:]                                           # a padded tail, 9 = [PAD]
    for policy in lab.NO_FRAG_POLICIES:
        got = _gpu(sd, l0, H, 7, 9, policy)
        want = lab.syntax_enriched_labels_batch(l0, H, 7, 9, X, policy)
        assert got.shape == want.shape and np.array_equal(got, want)


def test_training_shaped_batch_bit_exact(sd):
    """Sequences of the paper's CodeLlama token limit (Section IV-A: 8192) with ten heads, fragment lengths from
    the synthetic generator, every element against the oracle."""
    V, frag, pad = 32000, 32001, 32002
    l0 = wl.frag_filled_labels(3, 8192, V, frag, pad)
    got = _gpu(sd, l0, 10, frag, pad, "keep_base")
    want = lab.syntax_enriched_labels_batch(l0, 10, frag, pad, X)
    assert np.array_equal(got, want)
    share = (got == X).mean(axis=(0, 2))
    assert share[0] == 0 and np.all(np.diff(share) > 0)


def test_full_size_launch_on_sampled_columns(sd):
    """The benchmark's launch (256 sequences x 8192 positions x 11 rows): sampled columns against the oracle run on
    the column's own window, plus properties that hold everywhere."""
    V, frag, pad, H, B, S = 32000, 32001, 32002, 10, 256, 8192
    l0 = np.tile(wl.frag_filled_labels(16, S, V, frag, pad), (B // 16, 1))
    rng = np.random.default_rng(0)
    for b in range(B):                                   # decorrelate the copies: rotate each row's real part
        l0[b] = np.roll(l0[b], int(rng.integers(S))) if b >= 16 else l0[b]
    got = _gpu(sd, l0, H, frag, pad, "keep_base")
    assert got.shape == (B, H + 1, S)
    assert np.array_equal(got[:, 0, :], l0)                                     # the base row is L_0
    for i in range(1, H + 1):                                                   # survivors are the shifted labels
        keep = got[:, i, : S - i] != X
        assert np.array_equal(got[:, i, : S - i][keep], l0[:, i:][keep])
    ign = got == X
    assert np.all(ign[:, 1:, :] >= ign[:, :-1, :])                              # once ignored, ignored in later rows
    for _ in range(3000):
        b, s = int(rng.integers(B)), int(rng.integers(S))
        s = S - 1 - int(rng.integers(12)) if rng.random() < 0.1 else s          # some columns at the very end
        window = l0[b, s: s + H + 1]
        want = lab.syntax_enriched_labels(window, H, frag, pad, X)[:, 0]
        assert np.array_equal(got[b, :, s], want), (b, s)


def test_label_errors(sd):
    l0 = torch.zeros((2, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(sd.SpecDecError) as e:
        sd.build_labels(l0, 65, 1, 2)
    assert e.value.name == "SD_ERR_SHAPE"
    with pytest.raises(KeyError):
        sd.build_labels(l0, 2, 1, 2, no_frag="other")
    empty = sd.build_labels(torch.zeros((2, 0), dtype=torch.int32, device="cuda"), 3, 1, 2)
    assert empty.shape == (2, 4, 0)
