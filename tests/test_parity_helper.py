"""The comparison used by the GPU parity tests, exercised on the CPU: it accepts the oracle's own output and a
legitimate near-tie substitution, and rejects planted mistakes (a substituted id that is not among the best, a wrong
value, a wrong order, a repeated id)."""
import numpy as np
import pytest

from oracle import s3_oracle as orc
from paper_2601_17702_amd import synth
from tests import parity


def case():
    rng = np.random.default_rng(2)
    T, d, n_feat, k = 40, 32, 300, 8
    x = synth.to_storage(rng.standard_normal((T, d)).astype(np.float32), "bf16")
    W = synth.to_storage(rng.standard_normal((n_feat, d)).astype(np.float32), "bf16")
    b = rng.standard_normal(n_feat).astype(np.float32)
    o = orc.encode_topk(x, W, b, k, "bf16", want_dense=True)
    return x, W, b, k, o


def test_accepts_the_oracle_and_rejects_planted_mistakes():
    x, W, b, k, o = case()
    ids, vals = o["ids"].copy(), o["vals"].copy()
    assert parity.check_encode(ids[None], vals[None], x[None], W[None], b[None], k, "bf16") == (0, ids.shape[0])

    bad = ids.copy()                                   # the k-th id of row 3 replaced by the worst feature of the row
    bad[3, -1] = int(np.argmin(o["z"][3]))
    with pytest.raises(AssertionError):
        parity.check_encode_rows(bad, vals, x, W, b, k, "bf16")

    bad = ids.copy()                                   # replaced by the (k+1)-th best: value right, set wrong, gap not small
    r = int(np.argmax(o["gap"]))
    nxt = int(np.argsort(-o["z"][r], kind="stable")[k])
    bad[r, -1] = nxt
    v2 = vals.copy()
    v2[r, -1] = max(o["z"][r, nxt], 0)
    assert o["gap"][r] > parity.TIE_GAP
    with pytest.raises(AssertionError):
        parity.check_encode_rows(bad, v2, x, W, b, k, "bf16")

    v2 = vals.copy()                                   # a value off by 1 %
    pos = np.argwhere(vals > 0.1)[0]
    v2[pos[0], pos[1]] *= 1.01
    with pytest.raises(AssertionError):
        parity.check_encode_rows(ids, v2, x, W, b, k, "bf16")

    bad, v2 = ids.copy(), vals.copy()                  # first two entries of a row swapped
    bad[7, [0, 1]] = bad[7, [1, 0]]
    v2[7, [0, 1]] = v2[7, [1, 0]]
    with pytest.raises(AssertionError):
        parity.check_encode_rows(bad, v2, x, W, b, k, "bf16")

    bad = ids.copy()                                   # a repeated id
    bad[9, 1] = bad[9, 0]
    with pytest.raises(AssertionError):
        parity.check_encode_rows(bad, vals, x, W, b, k, "bf16")


def test_near_tie_substitution_is_accepted_and_counted():
    """Two features with pre-activations 1e-6 apart at the k-th/(k+1)-th place: either may be returned."""
    d, n_feat, k = 8, 6, 2
    W = np.zeros((n_feat, d), np.float32)
    W[0, 0], W[1, 1], W[2, 2], W[3, 3] = 1, 1, 1, 1
    x = np.array([[4.0, 2.0, 2.0, 1.0, 0, 0, 0, 0]], np.float32)
    b = np.zeros(n_feat, np.float32)
    b[1] = 1e-6                                       # z = [4, 2 + 1e-6, 2, 1, 0, 0]
    o = orc.encode_topk(x, W, b, k, "fp32")
    assert o["ids"].tolist() == [[0, 1]] and 0 < o["gap"][0] < parity.FLIP_GAP
    gi = np.array([[0, 2]], np.int32)                 # the other one of the near-tied pair
    gv = np.array([[4.0, 2.0]], np.float32)
    assert parity.check_encode_rows(gi, gv, x, W, b, k, "fp32") == (1, 1)
    gi = np.array([[0, 3]], np.int32)                 # not one of the pair
    with pytest.raises(AssertionError):
        parity.check_encode_rows(gi, np.array([[4.0, 1.0]], np.float32), x, W, b, k, "fp32")
