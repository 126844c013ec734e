"""GPU parity of the index build (bit-exact) and of co-activation scoring / span selection."""
import json
import os

import numpy as np
import pytest

from oracle import s3_oracle as orc
from tests import parity

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_ids(rng, T, k, n_feat, hot=None):
    """Distinct feature ids per row (as the encoder produces them); optionally one id in every row."""
    ids = np.empty((T, k), np.int32)
    for t in range(T):
        ids[t] = rng.choice(n_feat, k, replace=False)
    if hot is not None:
        for t in range(T):
            if hot not in ids[t]:
                ids[t, rng.integers(k)] = hot
    return ids


def oracle_csr(ids, positions, n_feat, chunks=None):
    ix = orc.Index(n_feat)
    ix.append(ids, positions)
    return ix, ix.csr()


def gpu_index(ids_heads, n_feat, positions=None, chunks=None, base=0):
    """ids_heads [H, T, k] numpy -> finalized s3.Index fed in the given chunk lengths."""
    import torch
    import paper_2601_17702_amd as s3
    H, T, k = ids_heads.shape
    ix = s3.Index(H, n_feat, k, max(T, 1))
    g = torch.from_numpy(ids_heads).cuda()
    a = 0
    for c in (chunks or [T]):
        if a >= T:
            break
        c = min(c, T - a)
        pos = None if positions is None else torch.from_numpy(positions[a:a + c]).cuda()
        ix.append(g[:, a:a + c].contiguous(), pos, base_pos=base + a)
        a += c
    assert a == T
    ix.finalize()
    return ix


def assert_csr_equal(ix, head, off_o, pos_o):
    import torch
    off, pos = ix.csr(head)
    torch.cuda.synchronize()
    assert np.array_equal(off.cpu().numpy(), off_o)
    assert np.array_equal(pos.cpu().numpy(), pos_o)


@pytest.mark.parametrize("T,k,n_feat", [
    (1, 1, 1), (255, 16, 200), (256, 32, 1000), (257, 32, 16384), (1300, 64, 65536),
    (5000, 48, 4096), (700, 7, 33), (900, 128, 16384), (300, 100, 128),
])
def test_index_bit_exact_vs_oracle(T, k, n_feat):
    rng = np.random.default_rng(T + k + n_feat)
    k = min(k, n_feat)
    ids = np.stack([rand_ids(rng, T, k, n_feat) for _ in range(2)])
    ix = gpu_index(ids, n_feat, base=100)
    for h in range(2):
        _, (off_o, pos_o) = oracle_csr(ids[h], np.arange(100, 100 + T, dtype=np.int32), n_feat)
        assert_csr_equal(ix, h, off_o, pos_o)
        assert off_o[-1] == T * k                              # P = tokens * k (Sec. 3.4)


def test_index_is_chunking_invariant_and_keeps_explicit_positions():
    rng = np.random.default_rng(9)
    T, k, n_feat = 3000, 32, 2048
    ids = rand_ids(rng, T, k, n_feat)[None]
    pos = rng.permutation(50000)[:T].astype(np.int32)          # arbitrary, non-monotone positions
    _, (off_o, pos_o) = oracle_csr(ids[0], pos, n_feat)
    for chunks in ([T], [37] * 100, [256, 1, 255, 512, 100, 3000], [2999, 1]):
        ix = gpu_index(ids, n_feat, positions=pos, chunks=chunks)
        assert_csr_equal(ix, 0, off_o, pos_o)


def test_index_hot_feature_spans_several_sort_rounds():
    rng = np.random.default_rng(10)
    T, k, n_feat = 40000, 4, 600                               # feature 77 is in every token: a 40000-entry list
    ids = rand_ids(rng, T, k, n_feat, hot=77)[None]
    ix = gpu_index(ids, n_feat, chunks=[8192] * 5)
    _, (off_o, pos_o) = oracle_csr(ids[0], np.arange(T, dtype=np.int32), n_feat)
    assert off_o[78] - off_o[77] == T
    assert_csr_equal(ix, 0, off_o, pos_o)


def test_one_shot_index_build_matches():
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(12)
    for T, k, n_feat in [(0, 4, 100), (513, 32, 16384), (2048, 16, 4096)]:
        ids = rand_ids(rng, T, k, n_feat) if T else np.zeros((0, k), np.int32)
        off, pos = s3.index_build(torch.from_numpy(ids).cuda(), n_feat)
        torch.cuda.synchronize()
        _, (off_o, pos_o) = oracle_csr(ids, np.arange(T, dtype=np.int32), n_feat)
        assert np.array_equal(off.cpu().numpy(), off_o) and np.array_equal(pos.cpu().numpy(), pos_o)


def test_index_state_and_capacity_errors():
    import torch
    import paper_2601_17702_amd as s3
    ix = s3.Index(1, 64, 4, 10)
    ids = torch.zeros((1, 8, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(s3.S3Error) as e:
        ix.csr(0)
    assert e.value.code == -2
    ix.append(ids)
    with pytest.raises(s3.S3Error) as e:
        ix.append(ids)                                          # 16 > max_tokens 10
    assert e.value.code == -3
    ix.finalize()
    with pytest.raises(s3.S3Error) as e:
        ix.append(ids[:, :1].contiguous())
    assert e.value.code == -2
    with pytest.raises(s3.S3Error):
        ix.finalize()
    assert ix.tokens == 8


# ------------------------------------------------------------------ scoring
def oracle_score(ids_heads, qids, qvals, n_feat, L, span_len, top_b, max_freq, nms, positions=None):
    S = np.zeros(L)
    for h in range(ids_heads.shape[0]):
        ix = orc.Index(n_feat)
        ix.append(ids_heads[h], np.arange(ids_heads.shape[1], dtype=np.int32) if positions is None else positions)
        ix.score_accumulate(qids[h], qvals[h], S, max_freq=max_freq)
    W = orc.pool(S, span_len)
    st, sc = orc.topb(W, span_len, top_b, nms=nms)
    return S, W, st, sc


def check_score(gpu, S, W, st_o, sc_o, span_len, nms):
    """gpu = (starts, scores, n_found, S_gpu) numpy.  Spans may differ from the oracle's only at near-ties."""
    st_g, sc_g, nf, S_g = gpu
    assert np.allclose(S_g, S, rtol=parity.REL_TOL, atol=1e-30)
    assert nf == len(st_o)
    assert np.all(st_g[nf:] == -1) and np.all(sc_g[nf:] == 0)
    for r in range(nf):
        s = int(st_g[r])
        assert 0 <= s < W.shape[0]
        assert abs(sc_g[r] - W[s]) <= parity.REL_TOL * abs(W[s]) + 1e-30      # reported score = oracle score of that window
        if s != st_o[r]:                                                        # a different pick must be a near-tie
            assert abs(W[s] - sc_o[r]) <= parity.REL_TOL * abs(sc_o[r]) + 1e-30, (r, s, st_o[r], W[s], sc_o[r])
    if nms:
        picks = sorted(int(x) for x in st_g[:nf])
        assert all(b - a >= min(span_len, S.shape[0]) for a, b in zip(picks, picks[1:]))
    assert len(set(st_g[:nf].tolist())) == nf


def run_gpu_score(ix, qids, qvals, L, span_len, top_b, max_freq, nms):
    import torch
    st, sc, nf, S = ix.coactivate_score(torch.from_numpy(qids).cuda(), torch.from_numpy(qvals).cuda(), L, span_len,
                                        top_b, max_freq=max_freq, nms=nms, want_scores=True)
    torch.cuda.synchronize()
    return st.cpu().numpy(), sc.cpu().numpy(), int(nf.item()), S.cpu().numpy()


def test_tiny_case_by_hand():
    g = json.load(open(os.path.join(GOLD, "tiny_case.json")))
    ids = np.array(g["ids"], np.int32)[None]
    ix = gpu_index(ids, 8)
    assert_csr_equal(ix, 0, np.array(g["offsets"], np.int32), np.array(g["csr_positions"], np.int32))
    qids, qvals = np.array(g["qids"], np.int32)[None], np.array(g["qvals"], np.float32)[None]
    for nms, want in ((True, g["span_start_nms"]), (False, g["span_start_no_nms"])):
        st, sc, nf, S = run_gpu_score(ix, qids, qvals, 6, g["span_len"], g["top_b"], 0, nms)
        assert nf == 2 and st.tolist() == want
        assert np.allclose(S, np.array(g["S_in_idf3_units"]) * g["idf3"], rtol=1e-6)
        assert np.allclose(sc, (np.array(g["W_in_idf3_units"]) * g["idf3"])[st], rtol=1e-6)
    st, _, nf, _ = run_gpu_score(ix, qids, qvals, 6, g["span_len"], 3, 0, True)
    assert st.tolist() == g["top_b3_nms"]


@pytest.mark.parametrize("H,T,k,n_feat,nq,span_len,top_b,max_freq,nms", [
    (1, 2048, 16, 4096, 8, 32, 8, 0, True),
    (3, 3000, 32, 1024, 40, 64, 16, 0, True),
    (3, 3000, 32, 1024, 40, 64, 16, 100, True),      # stop-feature threshold prunes the frequent lists
    (2, 1500, 64, 8192, 30, 32, 32, 0, False),
    (1, 300, 8, 64, 5, 1, 40, 0, True),              # span of one token
    (1, 90, 8, 64, 5, 500, 4, 0, True),              # span longer than the context: a single window
    (2, 1000, 4, 50, 6, 128, 64, 0, True),           # more spans asked for than disjoint windows exist
    (2, 1000, 4, 50, 6, 512, 4, 0, True),            # long windows over few heads: the windows' fixed-point sums need
    (1, 3000, 8, 16, 4, 2048, 2, 0, True),           # the span length in their headroom (frequent queried features)
    (2, 1200, 128, 16384, 6, 48, 40, 0, True),       # k = 128 (the paper's SAE sparsity), 40 spans of 48 (App. B.3)
])
def test_score_and_spans_vs_oracle(H, T, k, n_feat, nq, span_len, top_b, max_freq, nms):
    rng = np.random.default_rng(H * T + k + nq + span_len)
    ids = np.stack([rand_ids(rng, T, k, n_feat) for _ in range(H)])
    qids = np.stack([rand_ids(rng, nq, k, n_feat) for _ in range(H)])
    qids[:, -1] = qids[:, 0]                                   # duplicate query pairs add up
    qvals = rng.random((H, nq, k)).astype(np.float32) * 3
    qvals[:, 0, 0] = 0.0                                       # a zero activation adds nothing
    ix = gpu_index(ids, n_feat)
    S, W, st_o, sc_o = oracle_score(ids, qids, qvals, n_feat, T, span_len, top_b, max_freq, nms)
    out = run_gpu_score(ix, qids, qvals, T, span_len, top_b, max_freq, nms)
    check_score(out, S, W, st_o, sc_o, span_len, nms)
    again = run_gpu_score(ix, qids, qvals, T, span_len, top_b, max_freq, nms)
    for a, b in zip(out, again):                               # bit-identical from run to run
        assert np.array_equal(a, b)
    # forward-index identity (App. D.2): S[t] = sum_j qw[ids[t, j]]
    if max_freq == 0 and H == 1:
        freq = np.bincount(ids[0].ravel(), minlength=n_feat)
        qw = np.zeros(n_feat)
        np.add.at(qw, qids[0].ravel(), qvals[0].ravel().astype(np.float64))
        qw /= (np.log1p(freq) + 1)
        assert np.allclose(out[3], qw[ids[0]].sum(axis=1), rtol=parity.REL_TOL)


def test_window_score_is_exactly_the_sum_of_its_members_and_empty_query():
    rng = np.random.default_rng(77)
    T, k, n_feat, nq, span = 4096, 32, 2048, 16, 64
    ids = rand_ids(rng, T, k, n_feat)[None]
    ix = gpu_index(ids, n_feat)
    qids = rand_ids(rng, nq, k, n_feat)[None]
    qvals = rng.random((1, nq, k)).astype(np.float32)
    st, sc, nf, S = run_gpu_score(ix, qids, qvals, T, span, 8, 0, True)
    for r in range(nf):
        member_sum = S[st[r]:st[r] + span].astype(np.float64).sum()
        assert abs(sc[r] - member_sum) <= 1e-5 * member_sum
    st, sc, nf, S = run_gpu_score(ix, qids[:, :0], qvals[:, :0], T, span, 4, 0, True)   # no query vectors
    assert np.all(S == 0) and nf == 4 and st.tolist() == [0, span, 2 * span, 3 * span] and np.all(sc == 0)


def test_end_to_end_small_streams():
    """encode -> index -> query encode -> score on shrunken workloads.  The oracle runs its own chain end to end
    (its ids feed its index, its query activations feed its scores); nothing it sees comes from the GPU."""
    import torch
    import paper_2601_17702_amd as s3
    from paper_2601_17702_amd import synth
    for name, L, T, n_feat, heads in [("c1_tiny", 2048, 2048, 4096, [0]),
                                      ("c2_llama8b", 1024, 256, 4096, [0, 100]),
                                      ("c3_long", 768, 300, 2048, [1]),
                                      ("c4_qwen7b", 512, 128, 4096, [2, 3])]:
        w = synth.shrink(synth.WORKLOADS[name], L=L, T=T, n_feat=n_feat, nq=min(synth.WORKLOADS[name].nq, 32))
        W = np.stack([synth.gen_w_enc(w, h) for h in heads])
        b = np.stack([synth.gen_b_enc(w, h) for h in heads])
        Wg, bg = parity.to_gpu(W, w.dtype), parity.to_gpu(b, "fp32")
        ix = s3.Index(len(heads), n_feat, w.k, L)
        o_ids, ties = [], 0
        for c in range(w.n_chunks):
            x = np.stack([synth.gen_keys(w, h, c) for h in heads])
            ids, vals = s3.sae_encode_topk(parity.to_gpu(x, w.dtype), Wg, bg, w.k)
            ix.append(ids, base_pos=c * w.T)
            torch.cuda.synchronize()
            ties += parity.check_encode(ids.cpu().numpy(), vals.cpu().numpy(), x, W, b, w.k, w.dtype)[0]
            o_ids.append(np.stack([orc.encode_topk(x[i], W[i], b[i], w.k, w.dtype)["ids"] for i in range(len(heads))]))
        ix.finalize()
        o_ids = np.concatenate(o_ids, axis=1)
        q = np.stack([synth.gen_queries(w, h) for h in heads])
        qids, qvals = s3.sae_encode_topk(parity.to_gpu(q, w.dtype), Wg, bg, w.k)
        torch.cuda.synchronize()
        ties += parity.check_encode(qids.cpu().numpy(), qvals.cpu().numpy(), q, W, b, w.k, w.dtype)[0]
        oq = [orc.encode_topk(q[i], W[i], b[i], w.k, w.dtype) for i in range(len(heads))]
        oq_ids, oq_vals = np.stack([o["ids"] for o in oq]), np.stack([o["vals"] for o in oq]).astype(np.float32)
        assert ties == 0, "pick another seed/size: a near-tie row makes the two chains select different features"
        for i in range(len(heads)):
            _, (off_o, pos_o) = oracle_csr(o_ids[i], np.arange(L, dtype=np.int32), n_feat)
            assert_csr_equal(ix, i, off_o, pos_o)
        qi, qv = qids.cpu().numpy(), qvals.cpu().numpy()
        for max_freq in (0, 50):
            S, Wd, st_o, sc_o = oracle_score(o_ids, oq_ids, oq_vals, n_feat, L, w.span_len, w.top_b, max_freq, True)
            out = run_gpu_score(ix, qi, qv, L, w.span_len, w.top_b, max_freq, True)
            check_score(out, S, Wd, st_o, sc_o, w.span_len, True)


def test_scatter_position_blocks_long_lists_sorted_and_unsorted():
    """More than one LDS block of positions, posting lists long enough to be narrowed by binary search, and the
    same index fed with explicit positions in a scrambled order (lists unsorted: every posting is filtered)."""
    rng = np.random.default_rng(1234)
    H, T, k, n_feat, nq = 2, 40000, 8, 512, 12
    ids = np.stack([rand_ids(rng, T, k, n_feat, hot=5) for _ in range(H)])
    qids = np.stack([rand_ids(rng, nq, k, n_feat) for _ in range(H)])
    qids[:, 0, 0] = 5                                          # the hot feature (a list of T postings) is queried
    qvals = rng.random((H, nq, k)).astype(np.float32)
    ix = gpu_index(ids, n_feat, chunks=[4096] * 10)
    S, W, st_o, sc_o = oracle_score(ids, qids, qvals, n_feat, T, 64, 8, 0, True)
    check_score(run_gpu_score(ix, qids, qvals, T, 64, 8, 0, True), S, W, st_o, sc_o, 64, True)
    perm = rng.permutation(T).astype(np.int32)
    ix2 = gpu_index(ids, n_feat, positions=perm, chunks=[4096] * 10)
    S2, W2, st2, sc2 = oracle_score(ids, qids, qvals, n_feat, T, 64, 8, 0, True, positions=perm)
    check_score(run_gpu_score(ix2, qids, qvals, T, 64, 8, 0, True), S2, W2, st2, sc2, 64, True)


def strided_ids(rng, T, k, n_feat):
    """Distinct ids per row without a Python loop over rows (rows of 10^6 tokens)."""
    stride = n_feat // k
    return ((rng.integers(0, n_feat, T)[:, None] + np.arange(k)[None, :] * stride) % n_feat).astype(np.int32)


@pytest.mark.parametrize("T", [150_000, 64 * 16384 + 5000])
def test_scoring_of_long_contexts(T):
    """Ten position blocks (segments from the index's block table) and a context beyond the 64 blocks a table covers
    (every list walked whole by every block's workgroup and filtered)."""
    rng = np.random.default_rng(T)
    H, k, n_feat, nq = 2, 2, 64, 4
    ids = np.stack([strided_ids(rng, T, k, n_feat) for _ in range(H)])
    qids = np.stack([strided_ids(rng, nq, k, n_feat) for _ in range(H)])
    qvals = rng.random((H, nq, k)).astype(np.float32)
    ix = gpu_index(ids, n_feat, chunks=[50_000] * (T // 50_000 + 1))
    S, W, st_o, sc_o = oracle_score(ids, qids, qvals, n_feat, T, 128, 16, 0, True)
    check_score(run_gpu_score(ix, qids, qvals, T, 128, 16, 0, True), S, W, st_o, sc_o, 128, True)


def test_scoring_with_shifted_positions_and_index_reuse():
    """Positions that start at an offset: inside the range the index's block table covers (table used), beyond it
    (lists are searched instead), and the same index object reset and fed another stream (table rebuilt)."""
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(99)
    H, T, k, n_feat, nq = 2, 20000, 8, 256, 10
    ix = s3.Index(H, n_feat, k, 40000)                         # capacity: three blocks of 16384 positions
    for base in (0, 12000, 30000, 5):                          # 30000 + 20000 lies beyond the three blocks
        ids = np.stack([rand_ids(rng, T, k, n_feat, hot=3) for _ in range(H)])
        qids = np.stack([rand_ids(rng, nq, k, n_feat) for _ in range(H)])
        qids[:, 0, 0] = 3
        qvals = rng.random((H, nq, k)).astype(np.float32)
        ix.reset()
        g = torch.from_numpy(ids).cuda()
        for a in range(0, T, 3000):
            ix.append(g[:, a:a + 3000].contiguous(), base_pos=base + a)
        ix.finalize()
        L = base + T + 7
        pos = np.arange(base, base + T, dtype=np.int32)
        for h in range(H):
            _, (off_o, pos_o) = oracle_csr(ids[h], pos, n_feat)
            assert_csr_equal(ix, h, off_o, pos_o)
        S, W, st_o, sc_o = oracle_score(ids, qids, qvals, n_feat, L, 48, 8, 0, True, positions=pos)
        check_score(run_gpu_score(ix, qids, qvals, L, 48, 8, 0, True), S, W, st_o, sc_o, 48, True)
        if base + T <= 3 * 16384:                              # the compact form needs the table's range
            cx = ix.compact(0)
            st, sc, nf, Sg = cx.coactivate_score(torch.from_numpy(qids).cuda(), torch.from_numpy(qvals).cuda(), L, 48, 8,
                                                 want_scores=True)
            torch.cuda.synchronize()
            check_score((st.cpu().numpy(), sc.cpu().numpy(), int(nf.item()), Sg.cpu().numpy()), S, W, st_o, sc_o, 48, True)
        else:
            with pytest.raises(s3.S3Error):
                ix.compact(0)
