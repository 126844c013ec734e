"""GPU parity of the compact index (16-bit block-relative postings, block-major order, stop-feature pruning) and of
scoring from it.  Both sides start from the same seeded ids: the oracle builds its own index and encodes it itself;
nothing it sees comes from the GPU."""
import numpy as np
import pytest

from oracle import s3_oracle as orc
from tests.test_gpu_index_score import check_score, gpu_index, oracle_score, rand_ids, strided_ids

pytestmark = pytest.mark.gpu


def oracle_compact(ids, n_feat, nblk, prune):
    ix = orc.Index(n_feat)
    ix.append(ids, np.arange(ids.shape[0], dtype=np.int32))
    off, pos = ix.csr()
    return orc.compact_encode(off, pos, nblk, 14, prune)


@pytest.mark.parametrize("H,T,k,n_feat,prune", [
    (2, 3000, 16, 512, 0),          # one block
    (2, 40000, 8, 512, 0),          # three blocks, lists of every length
    (2, 40000, 8, 512, 700),        # with stop-feature pruning
    (1, 100_000, 2, 64, 4000),      # seven blocks, long lists
    (3, 20000, 32, 16384, 0),       # many short lists (most segments empty)
])
def test_compact_arrays_bit_exact_and_scores(H, T, k, n_feat, prune):
    import torch
    rng = np.random.default_rng(T + k + n_feat + prune)
    gen = strided_ids if T >= 100_000 else (lambda r, t, kk, nf: rand_ids(r, t, kk, nf, hot=5 if nf > 5 else None))
    ids = np.stack([gen(rng, T, k, n_feat) for _ in range(H)])
    ix = gpu_index(ids, n_feat, chunks=[8192] * (T // 8192 + 1))
    cx = ix.compact(prune)
    nblk = (T + 16383) // 16384
    assert cx.n_blocks == nblk and cx.max_postings == T * k
    for h in range(H):
        cs, de, cf = cx.arrays(h)
        cs_o, de_o, cf_o = oracle_compact(ids[h], n_feat, nblk, prune)
        assert np.array_equal(cs.cpu().numpy(), cs_o)
        assert np.array_equal(de.cpu().numpy().view(np.uint16), de_o)
        assert np.array_equal(cf.cpu().numpy(), cf_o)
    ix.destroy()                                                   # the compact index does not need the plain one
    nq = 10
    qids = np.stack([rand_ids(rng, nq, k, n_feat) for _ in range(H)])
    qids[:, 0, 0] = 5 if n_feat > 5 else 0                         # the frequent feature is queried
    qvals = rng.random((H, nq, k)).astype(np.float32)
    for max_freq in (0, 300):
        eff = prune if max_freq == 0 else (min(prune, max_freq) if prune else max_freq)   # both rules are strict >
        S, W, st_o, sc_o = oracle_score(ids, qids, qvals, n_feat, T, 64, 8, eff, True)
        st, sc, nf, Sg = cx.coactivate_score(torch.from_numpy(qids).cuda(), torch.from_numpy(qvals).cuda(), T, 64, 8,
                                             max_freq=max_freq, nms=True, want_scores=True)
        torch.cuda.synchronize()
        check_score((st.cpu().numpy(), sc.cpu().numpy(), int(nf.item()), Sg.cpu().numpy()), S, W, st_o, sc_o, 64, True)


def test_compact_needs_a_finalized_index_with_implicit_positions():
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(3)
    ids = torch.from_numpy(rand_ids(rng, 100, 4, 64)[None]).cuda()
    ix = s3.Index(1, 64, 4, 40000)
    ix.append(ids)
    with pytest.raises(s3.S3Error) as e:
        ix.compact()
    assert e.value.code == -2                                      # not finalized
    ix2 = s3.Index(1, 64, 4, 40000)
    ix2.append(ids, positions=torch.arange(100, dtype=torch.int32, device="cuda") * 300)     # explicit positions
    ix2.finalize()
    with pytest.raises(s3.S3Error) as e:
        ix2.compact()
    assert e.value.code == -2
    ix.finalize()
    cx = ix.compact()
    cs, de, cf = cx.arrays(0)
    assert int(cs[-1].item()) == 400 and int(cf.sum().item()) == 400
