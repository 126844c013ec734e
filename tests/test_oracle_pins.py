"""Pins of the CPU oracle against things other than itself: the values the paper fixes, closed
forms, a hand-computed case, brute force on tiny inputs and library routines (numpy)."""
import json
import math
import os

import numpy as np
import pytest

from oracle import s3_oracle as orc
from paper_2601_17702_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def paper_values():
    out = {}
    for line in open(os.path.join(GOLD, "paper_values.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [s.strip() for s in line.split("=")]
            out[k] = float(v)
    return out


def tiny():
    return json.load(open(os.path.join(GOLD, "tiny_case.json")))


def np_topk_rows(z, k):
    """Library route: stable argsort of -z gives (z desc, id asc)."""
    order = np.argsort(-z, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


# ------------------------------------------------------------------ encoder + Top-k (Sec. 3.3)
def test_tiny_case_encode_by_hand():
    g = tiny()
    x = np.array(g["x"], np.float32)
    w = np.array(g["w_enc"], np.float32)
    b = np.array(g["b_enc"], np.float32)
    r = orc.encode_topk(x, w, b, g["k"], "fp32", want_dense=True)
    assert np.array_equal(r["z"], np.array(g["z"], np.float64))
    assert np.array_equal(r["ids"], np.array(g["ids"], np.int32))
    assert np.array_equal(r["vals"], np.array(g["vals"], np.float32))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_encode_matches_numpy_matmul_and_sort(dtype):
    rng = np.random.default_rng(7)
    T, d, n_feat, k = 48, 96, 320, 12          # non-square, so a transposed operand cannot pass
    x = synth.to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    w = synth.to_storage(rng.standard_normal((n_feat, d)).astype(np.float32), dtype)
    b = rng.standard_normal(n_feat).astype(np.float32)
    r = orc.encode_topk(x, w, b, k, dtype, want_dense=True)
    z = synth.storage_to_f64(x, dtype) @ synth.storage_to_f64(w, dtype).T + b.astype(np.float64)
    assert np.allclose(r["z"], z, rtol=1e-13, atol=1e-13)
    ids = np_topk_rows(r["z"], k)
    assert np.array_equal(r["ids"], ids)
    zs = np.take_along_axis(r["z"], ids, axis=1)
    assert np.array_equal(r["zsel"], zs)
    assert np.array_equal(r["vals"], np.maximum(zs, 0).astype(np.float32))
    srt = -np.sort(-r["z"], axis=1)
    assert np.allclose(r["gap"], (srt[:, k - 1] - srt[:, k]) / np.abs(srt[:, k - 1]))


def test_bf16_storage_is_widened_exactly():
    # 1 + 2^-7 is a bf16 value; 1 + 2^-9 is not and must already have been rounded by the generator
    v = np.array([[1.0 + 2.0 ** -7, 3.0]], np.float32)
    bits = synth.f32_to_bf16_bits(v)
    assert np.array_equal(synth.bf16_bits_to_f32(bits), v)
    w = synth.f32_to_bf16_bits(np.array([[1.0, 0.0], [0.0, 1.0]], np.float32))
    r = orc.encode_topk(bits, w, np.zeros(2, np.float32), 2, "bf16", want_dense=True)
    assert np.array_equal(r["z"], np.array([[1.0 + 2.0 ** -7, 3.0]]))
    assert np.array_equal(synth.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -9], np.float32)),
                          synth.f32_to_bf16_bits(np.array([1.0], np.float32)))
    # round-to-nearest-even at the halfway point: 1 + 2^-8 -> 1 (even), 1 + 3*2^-8 -> 1 + 2^-6
    h = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8], np.float32)))
    assert np.array_equal(h, np.array([1.0, 1 + 2.0 ** -6], np.float32))


def test_one_hot_dictionary_selects_largest_channels():
    # W = [I; -I], b = 0: z = [x, -x], so the Top-k features are the k largest |x_c| with the sign's half
    rng = np.random.default_rng(3)
    d, k = 16, 5
    x = rng.standard_normal((10, d)).astype(np.float32)
    w = np.concatenate([np.eye(d), -np.eye(d)]).astype(np.float32)
    r = orc.encode_topk(x, w, np.zeros(2 * d, np.float32), k, "fp32")
    for t in range(x.shape[0]):
        ch = np.argsort(-np.abs(x[t]), kind="stable")[:k]
        want = [c if x[t, c] > 0 else c + d for c in ch]
        assert r["ids"][t].tolist() == want
        assert np.array_equal(r["vals"][t], np.abs(x[t, ch]))


def test_k_equals_n_feat_returns_every_feature_sorted():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 8)).astype(np.float32)
    w = rng.standard_normal((24, 8)).astype(np.float32)
    b = rng.standard_normal(24).astype(np.float32)
    r = orc.encode_topk(x, w, b, 24, "fp32", want_dense=True)
    assert np.array_equal(np.sort(r["ids"], axis=1), np.tile(np.arange(24, dtype=np.int32), (4, 1)))
    assert np.all(np.diff(r["zsel"], axis=1) <= 0)
    assert np.all(np.isinf(r["gap"]))


def test_exact_ties_take_lower_feature_id_and_negative_rows_keep_k_ids():
    w = np.array([[1, 0], [1, 0], [0, 1], [1, 0], [-1, -1]], np.float32)   # features 0, 1, 3 identical
    x = np.array([[2, 1], [-1, -3]], np.float32)
    r = orc.encode_topk(x, w, np.zeros(5, np.float32), 2, "fp32")
    assert r["ids"][0].tolist() == [0, 1]                # z = [2, 2, 1, 2, -3]
    assert r["ids"][1].tolist() == [4, 0]                # z = [-1, -1, -3, -1, 4]
    # every pre-activation negative: still exactly k ids (largest z), activations are ReLU -> 0
    r = orc.encode_topk(x, w, np.full(5, -100, np.float32), 2, "fp32", want_dense=True)
    assert np.all(r["vals"] == 0) and np.all(r["z"] < 0)
    assert np.array_equal(r["ids"], np_topk_rows(r["z"], 2))
    assert all(len(set(row)) == 2 for row in r["ids"].tolist())


def test_decoder_bias_folding_identity():
    # encoder equation W(x - b_dec) + b_enc == W x + (b_enc - W b_dec); small integers keep fp exact
    rng = np.random.default_rng(11)
    x = rng.integers(-8, 9, (6, 4)).astype(np.float32)
    w = rng.integers(-4, 5, (10, 4)).astype(np.float32)
    b_enc = rng.integers(-3, 4, 10).astype(np.float32)
    b_dec = rng.integers(-2, 3, 4).astype(np.float32)
    direct = (x - b_dec) @ w.T + b_enc
    r = orc.encode_topk(x, w, (b_enc - w @ b_dec).astype(np.float32), 3, "fp32", want_dense=True)
    assert np.array_equal(r["z"], direct.astype(np.float64))


def test_selected_set_dominates_the_rest():
    w = synth.shrink(synth.WORKLOADS["c1_tiny"], n_feat=512, L=64, T=64)
    x, W, b = synth.gen_keys(w, 0, 0), synth.gen_w_enc(w, 0), synth.gen_b_enc(w, 0)
    r = orc.encode_topk(x, W, b, w.k, w.dtype, want_dense=True)
    for t in range(x.shape[0]):
        sel = set(r["ids"][t].tolist())
        assert len(sel) == w.k
        rest = np.array([f for f in range(w.n_feat) if f not in sel])
        assert r["z"][t, list(sel)].min() >= r["z"][t, rest].max()
    # generated rows are unit-norm (fp32 storage)
    assert np.allclose(np.linalg.norm(W.astype(np.float64), axis=1), 1.0, atol=1e-6)


# ------------------------------------------------------------------ inverted index (Sec. 3.4)
def brute_lists(ids, positions, n_feat):
    lists = {f: [] for f in range(n_feat)}
    for t in range(ids.shape[0]):
        for f in ids[t]:
            lists[int(f)].append(int(positions[t]))
    return lists


def test_tiny_case_index_by_hand():
    g = tiny()
    ix = orc.Index(8)
    ix.append(np.array(g["ids"], np.int32), np.array(g["positions"], np.int32))
    off, pos = ix.csr()
    assert off.tolist() == g["offsets"]
    assert pos.tolist() == g["csr_positions"]


def test_index_matches_brute_force_and_is_chunking_invariant():
    rng = np.random.default_rng(2)
    T, k, n_feat = 300, 6, 50
    ids = np.stack([rng.choice(n_feat, k, replace=False) for _ in range(T)]).astype(np.int32)
    pos = np.arange(1000, 1000 + T, dtype=np.int32)
    one = orc.Index(n_feat)
    one.append(ids, pos)
    off, p = one.csr()
    lists = brute_lists(ids, pos, n_feat)
    assert off[0] == 0 and np.all(np.diff(off) >= 0) and off[-1] == T * k == one.n_postings
    for f in range(n_feat):
        seg = p[off[f]:off[f + 1]].tolist()
        assert seg == lists[f] and seg == sorted(set(seg))     # ascending, each (f, t) once
    # inverse check: rebuild every row's feature set from the postings
    back = [set() for _ in range(T)]
    for f in range(n_feat):
        for t in p[off[f]:off[f + 1]]:
            back[t - 1000].add(f)
    assert back == [set(r) for r in ids.tolist()]
    many = orc.Index(n_feat)
    for a in range(0, T, 37):                                   # ragged chunks
        many.append(ids[a:a + 37], pos[a:a + 37])
    off2, p2 = many.csr()
    assert np.array_equal(off, off2) and np.array_equal(p, p2)


def test_index_keeps_insertion_order_for_explicit_positions():
    ix = orc.Index(3)
    ix.append(np.array([[0, 1], [0, 2], [1, 0]], np.int32), np.array([9, 4, 7], np.int32))
    off, p = ix.csr()
    assert off.tolist() == [0, 3, 5, 6] and p.tolist() == [9, 4, 7, 9, 7, 4]


def test_posting_count_closed_form_and_paper_worked_example():
    v = paper_values()
    L, layers, k = int(v["index_size_L"]), int(v["index_size_layers"]), int(v["index_size_k"])
    assert L * layers * k == int(v["index_size_postings"])
    assert 4 * L * layers * k == int(v["index_size_bytes"]) == 256 * 2 ** 20
    # the oracle's own count at the paper's worked size, one index per instrumented layer
    rng = np.random.default_rng(0)
    total = 0
    for _ in range(layers):
        ix = orc.Index(16384)
        for a in range(0, L, 16384):
            ids = rng.integers(0, 16384, (16384, k), dtype=np.int32)
            ix.append(ids, np.arange(a, a + 16384, dtype=np.int32))
        off, _ = ix.csr()
        assert off[-1] == ix.n_postings == L * k
        total += ix.n_postings
    assert total == int(v["index_size_postings"])


# ------------------------------------------------------------------ scoring (Sec. 3.5, App. D.2, App. E)
def test_idf_closed_forms():
    v = paper_values()
    assert orc.idf(0) == v["idf_freq0"] == 1.0
    assert orc.idf(1) == pytest.approx(v["idf_freq1"], rel=1e-15)
    assert orc.idf(1) == pytest.approx(1 / (math.log(2) + 1), rel=1e-15)
    assert orc.idf(3) == pytest.approx(v["idf_freq3"], rel=1e-15)
    # natural log: IDF = 1/2 exactly where 1 + freq = e; integers on either side bracket it
    assert orc.idf(1) > 0.5 > orc.idf(2)
    assert all(orc.idf(f) > orc.idf(f + 1) for f in range(0, 50))


def test_tiny_case_scores_spans_by_hand():
    g = tiny()
    ix = orc.Index(8)
    ix.append(np.array(g["ids"], np.int32), np.array(g["positions"], np.int32))
    q = orc.encode_topk(np.array(g["query"], np.float32), np.array(g["w_enc"], np.float32),
                        np.array(g["b_enc"], np.float32), g["k"], "fp32")
    assert q["ids"].tolist() == g["qids"] and q["vals"].tolist() == g["qvals"]
    S = np.zeros(6)
    ix.score_accumulate(q["ids"], q["vals"], S)
    assert np.allclose(S, np.array(g["S_in_idf3_units"]) * g["idf3"], rtol=1e-15)
    W = orc.pool(S, g["span_len"])
    assert np.allclose(W, np.array(g["W_in_idf3_units"]) * g["idf3"], rtol=1e-15)
    st, sc = orc.topb(W, g["span_len"], g["top_b"], nms=True)
    assert st.tolist() == g["span_start_nms"] and np.array_equal(sc, W[st])
    st, _ = orc.topb(W, g["span_len"], g["top_b"], nms=False)
    assert st.tolist() == g["span_start_no_nms"]
    st, _ = orc.topb(W, g["span_len"], 3, nms=True)
    assert st.tolist() == g["top_b3_nms"]


def test_score_equals_set_intersection_brute_force():
    """App. D.2: s(t) = sum over f in F_Q ∩ F_t of a_f * IDF(f), straight from the forward lists."""
    rng = np.random.default_rng(4)
    T, k, n_feat, nq = 200, 5, 40, 7
    ids = np.stack([rng.choice(n_feat, k, replace=False) for _ in range(T)]).astype(np.int32)
    qids = np.stack([rng.choice(n_feat, k, replace=False) for _ in range(nq)]).astype(np.int32)
    qvals = rng.random((nq, k)).astype(np.float32)
    qvals[0, 0] = 0.0                                           # a zero activation adds nothing
    ix = orc.Index(n_feat)
    ix.append(ids, np.arange(T, dtype=np.int32))
    freq = np.bincount(ids.ravel(), minlength=n_feat)
    for max_freq in (0, int(np.median(freq))):
        S = np.zeros(T)
        ix.score_accumulate(qids, qvals, S, max_freq=max_freq)
        want = np.zeros(T)
        for t in range(T):
            Ft = set(ids[t].tolist())
            for q in range(nq):
                for j in range(k):
                    f = int(qids[q, j])
                    if f in Ft and not (max_freq > 0 and freq[f] > max_freq):   # strict ">"
                        want[t] += float(qvals[q, j]) / (math.log(1 + freq[f]) + 1)
        assert np.allclose(S, want, rtol=1e-12, atol=0)
    # a feature whose freq equals max_freq is kept, freq = max_freq + 1 is dropped
    f0 = int(qids[1, 1])
    S_keep, S_drop = np.zeros(T), np.zeros(T)
    ix.score_accumulate(qids[1:2, 1:2], qvals[1:2, 1:2], S_keep, max_freq=int(freq[f0]))
    ix.score_accumulate(qids[1:2, 1:2], qvals[1:2, 1:2], S_drop, max_freq=int(freq[f0]) - 1)
    assert S_keep.sum() > 0 and S_drop.sum() == 0


def test_query_equal_to_a_context_token_scores_its_own_features():
    rng = np.random.default_rng(6)
    T, k, n_feat = 64, 4, 30
    ids = np.stack([rng.choice(n_feat, k, replace=False) for _ in range(T)]).astype(np.int32)
    ix = orc.Index(n_feat)
    ix.append(ids, np.arange(T, dtype=np.int32))
    freq = np.bincount(ids.ravel(), minlength=n_feat)
    S = np.zeros(T)
    ix.score_accumulate(ids[17:18], np.ones((1, k), np.float32), S)
    assert S[17] == pytest.approx(sum(1 / (math.log(1 + freq[f]) + 1) for f in ids[17]), rel=1e-14)
    assert S[17] == S.max()
    # scores add over (layer, head) indexes and over duplicate query pairs
    S2 = np.zeros(T)
    ix.score_accumulate(np.concatenate([ids[17:18]] * 2), np.ones((2, k), np.float32), S2)
    assert np.allclose(S2, 2 * S)


def test_pool_is_a_box_sum_over_valid_windows():
    rng = np.random.default_rng(8)
    S = rng.random(97)
    for span in (1, 8, 48, 97):
        W = orc.pool(S, span)
        assert W.shape[0] == 97 - span + 1
        assert np.allclose(W, np.convolve(S, np.ones(span), mode="valid"), rtol=1e-13)
        if span < 97:
            assert np.allclose(W[1:] - W[:-1], S[span:] - S[:-span], atol=1e-12)
    W = orc.pool(S, 500)                                        # span longer than the context
    assert W.shape == (1,) and W[0] == pytest.approx(S.sum(), rel=1e-13)


def test_topb_hand_cases():
    span = 4
    S = np.zeros(40)
    S[10] = 1.0                                                 # one spike
    W = orc.pool(S, span)
    st, sc = orc.topb(W, span, 3, nms=True)
    # windows 7..10 all hold the spike and tie; smallest start wins, the others overlap it
    assert st[0] == 7 and sc[0] == 1.0
    assert all(abs(int(a) - int(b)) >= span for i, a in enumerate(st) for b in st[:i])
    assert sc[1] == 0.0 and st[1] == 0                          # next best is an all-zero window
    S[30] = 2.0                                                 # a second, larger spike far away
    W = orc.pool(S, span)
    st, sc = orc.topb(W, span, 2, nms=True)
    assert st.tolist() == [27, 7] and sc.tolist() == [2.0, 1.0]
    st, sc = orc.topb(W, span, 5, nms=False)                    # without suppression: plain top-5
    assert st.tolist() == [27, 28, 29, 30, 7]
    # more spans asked for than disjoint windows exist
    W = orc.pool(np.ones(10), 4)
    st, _ = orc.topb(W, 4, 8, nms=True)
    assert st.tolist() == [0, 4]
    st, _ = orc.topb(W, 4, 100, nms=False)
    assert st.tolist() == list(range(7))


def test_preact_at_closed_forms():
    """Sec. 3.3 encoder equation at single entries: the hand case's z table, and z = +-x_c + b for a one-hot
    dictionary [I; -I] (the feature row picks the channel, so a transposed or shifted index cannot pass)."""
    g = tiny()
    x, w, b = np.array(g["x"], np.float32), np.array(g["w_enc"], np.float32), np.array(g["b_enc"], np.float32)
    all_ids = np.broadcast_to(np.arange(8, dtype=np.int32)[::-1], (6, 8))            # every feature, in reversed order
    assert np.array_equal(orc.preact_at(x, w, b, all_ids, "fp32"), np.array(g["z"], np.float64)[:, ::-1])
    rng = np.random.default_rng(21)
    d, T = 16, 9
    xb = synth.to_storage(rng.standard_normal((T, d)).astype(np.float32), "bf16")
    wb = synth.to_storage(np.concatenate([np.eye(d), -np.eye(d)]).astype(np.float32), "bf16")
    bias = rng.standard_normal(2 * d).astype(np.float32)
    ids = rng.integers(0, 2 * d, (T, 5)).astype(np.int32)
    xf = synth.storage_to_f64(xb, "bf16")
    want = np.where(ids < d, 1.0, -1.0) * np.take_along_axis(xf, ids % d, axis=1) + bias[ids].astype(np.float64)
    assert np.array_equal(orc.preact_at(xb, wb, bias, ids, "bf16"), want)
    with pytest.raises(ValueError):
        orc.preact_at(xb, wb, bias, np.full((T, 1), 2 * d, np.int32), "bf16")


def test_score_dense_hand_case_and_set_intersection():
    """The token-wise form of the scoring equation against things other than the oracle: the hand-computed case
    (scores in units of IDF(3)), and App. D.2's set-intersection sum written out with Python sets, for several
    heads, duplicate query pairs, a zero activation and the strict freq > max_freq rule."""
    g = tiny()
    ids = np.array(g["ids"], np.int32)[None]
    S = orc.score_dense(ids, np.array(g["qids"], np.int32)[None], np.array(g["qvals"], np.float32)[None], 8)
    assert np.allclose(S, np.array(g["S_in_idf3_units"]) * g["idf3"], rtol=1e-15)
    rng = np.random.default_rng(13)
    H, L, k, n_feat, nq = 2, 120, 4, 30, 6
    ids = np.stack([np.stack([rng.choice(n_feat, k, replace=False) for _ in range(L)]) for _ in range(H)]).astype(np.int32)
    qids = np.stack([np.stack([rng.choice(n_feat, k, replace=False) for _ in range(nq)]) for _ in range(H)]).astype(np.int32)
    qids[:, -1] = qids[:, 0]
    qvals = rng.random((H, nq, k)).astype(np.float32)
    qvals[0, 0, 0] = 0.0
    freq = [np.bincount(ids[h].ravel(), minlength=n_feat) for h in range(H)]
    for max_freq in (0, int(np.median(freq[0]))):
        want = np.zeros(L)
        for h in range(H):
            for t in range(L):
                Ft = set(ids[h, t].tolist())
                for q in range(nq):
                    for j in range(k):
                        f = int(qids[h, q, j])
                        if f in Ft and not (max_freq > 0 and freq[h][f] > max_freq):
                            want[t] += float(qvals[h, q, j]) / (math.log(1 + freq[h][f]) + 1)
        assert np.allclose(orc.score_dense(ids, qids, qvals, n_feat, max_freq=max_freq), want, rtol=1e-12, atol=0)


def test_score_dense_equals_postings_form():
    """The token-wise evaluation of the scoring equation (Sec. 3.5) and the postings traversal are the same sum."""
    rng = np.random.default_rng(11)
    H, L, k, n_feat, nq = 3, 200, 4, 37, 5
    ids = np.stack([np.stack([rng.choice(n_feat, k, replace=False) for _ in range(L)]) for _ in range(H)]).astype(np.int32)
    qids = np.stack([np.stack([rng.choice(n_feat, k, replace=False) for _ in range(nq)]) for _ in range(H)]).astype(np.int32)
    qvals = rng.random((H, nq, k)).astype(np.float32)
    for max_freq in (0, 25):
        S = np.zeros(L)
        for h in range(H):
            ix = orc.Index(n_feat)
            ix.append(ids[h], np.arange(L, dtype=np.int32))
            ix.score_accumulate(qids[h], qvals[h], S, max_freq=max_freq)
        D = orc.score_dense(ids, qids, qvals, n_feat, max_freq=max_freq)
        assert np.allclose(S, D, rtol=1e-12, atol=1e-12)
        assert max_freq == 0 or not np.allclose(D, orc.score_dense(ids, qids, qvals, n_feat, max_freq=0))
