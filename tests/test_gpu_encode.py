"""GPU parity of s3_sae_encode_topk against the fp64 oracle (element by element)."""
import numpy as np
import pytest

from paper_2601_17702_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


def run(x, W, b, k, dtype):
    import torch
    import paper_2601_17702_amd as s3
    ids, vals = s3.sae_encode_topk(parity.to_gpu(x, dtype), parity.to_gpu(W, dtype), parity.to_gpu(b, "fp32"), k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), vals.cpu().numpy()


def test_c1_tiny_full():
    w = synth.WORKLOADS["c1_tiny"]
    x, W, b = parity.head_inputs(w, [0])
    ids, vals = run(x, W, b, w.k, w.dtype)
    ties, rows = parity.check_encode(ids, vals, x, W, b, w.k, w.dtype)
    print(f"c1_tiny: {ties} near-tie rows of {rows}")


@pytest.mark.parametrize("name,T,n_feat,heads", [
    ("c2_llama8b", 300, 16384, [0, 255]),      # ragged token tail, two heads in one launch
    ("c3_long", 257, 16384, [0]),              # Zipf-biased b_enc (hot features)
    ("c4_qwen7b", 130, 32768, [5]),            # k = 64
    ("c5_wide", 96, 65536, [7]),               # widest SAE, k = 64
])
def test_workload_shapes_sampled(name, T, n_feat, heads):
    w = synth.shrink(synth.WORKLOADS[name], T=T, L=T, n_feat=n_feat)
    x, W, b = parity.head_inputs(w, heads)
    ids, vals = run(x, W, b, w.k, w.dtype)
    ties, rows = parity.check_encode(ids, vals, x, W, b, w.k, w.dtype)
    print(f"{name}: {ties} near-tie rows of {rows}")


@pytest.mark.parametrize("dtype,d,n_feat,k,T", [
    ("bf16", 64, 1000, 64, 129),     # n_feat not a multiple of the feature tile
    ("bf16", 256, 520, 7, 33),
    ("fp32", 64, 96, 1, 5),
    ("fp32", 256, 300, 33, 64),
    ("bf16", 128, 48, 48, 70),       # k == n_feat: every feature is returned
    ("fp32", 128, 64, 64, 1),        # single token
    ("bf16", 128, 16384, 128, 200),  # the paper's SAE setting: expansion 128, k = 128 (App. B.3)
    ("fp32", 64, 700, 128, 70),      # k = 128 in fp32
    ("bf16", 256, 1024, 121, 40),    # the largest k that fits beside the 256-wide tiles
    ("bf16", 128, 128, 128, 33),     # k == n_feat == 128
    ("fp32", 256, 500, 78, 35),      # half-tile headroom below k = 64's usual setting (fp32, d_head 256)
])
def test_odd_shapes(dtype, d, n_feat, k, T):
    rng = np.random.default_rng(d + n_feat + k + T)
    x = synth.to_storage(rng.standard_normal((2, T, d)).astype(np.float32), dtype)
    W = synth.to_storage((rng.standard_normal((2, n_feat, d)) / np.sqrt(d)).astype(np.float32), dtype)
    b = (0.1 * rng.standard_normal((2, n_feat))).astype(np.float32)
    ids, vals = run(x, W, b, k, dtype)
    ties, rows = parity.check_encode(ids, vals, x, W, b, k, dtype)
    if k == n_feat:
        assert np.array_equal(np.sort(ids, axis=2), np.broadcast_to(np.arange(n_feat, dtype=np.int32), ids.shape))


def test_exact_ties_take_lower_id_and_negative_rows():
    d, n_feat, k, T = 128, 256, 32, 40
    rng = np.random.default_rng(0)
    base = rng.integers(-2, 3, (8, d)).astype(np.float32)          # small integers: every product is exact
    W = base[rng.integers(0, 8, n_feat)][None]                     # many duplicate rows -> many exact ties
    x = rng.integers(-2, 3, (1, T, d)).astype(np.float32)
    b = np.zeros((1, n_feat), np.float32)
    for dtype in ("fp32", "bf16"):
        xs, Ws = synth.to_storage(x, dtype), synth.to_storage(W, dtype)
        ids, vals = run(xs, Ws, b, k, dtype)
        from oracle import s3_oracle as orc
        o = orc.encode_topk(xs[0], Ws[0], b[0], k, dtype)
        assert np.array_equal(ids[0], o["ids"]) and np.array_equal(vals[0], o["vals"])
    # all pre-activations negative: ids still the k largest z, activations are ReLU -> 0
    bneg = np.full((1, n_feat), -1000, np.float32)
    Wr = synth.to_storage(rng.standard_normal((1, n_feat, d)).astype(np.float32), "bf16")
    xr = synth.to_storage(rng.standard_normal((1, T, d)).astype(np.float32), "bf16")
    ids, vals = run(xr, Wr, bneg, k, "bf16")
    assert np.all(vals == 0)
    parity.check_encode(ids, vals, xr, Wr, bneg, k, "bf16")
    # all-equal pre-activations (W = 0): the k lowest ids win
    ids, vals = run(xr, np.zeros_like(Wr), np.ones((1, n_feat), np.float32), k, "bf16")
    assert np.array_equal(ids[0], np.broadcast_to(np.arange(k, dtype=np.int32), (T, k))) and np.all(vals == 1)


def test_one_hot_dictionary():
    d, k, T = 128, 9, 50
    rng = np.random.default_rng(1)
    x = synth.to_storage(rng.standard_normal((1, T, d)).astype(np.float32), "bf16")
    W = synth.to_storage(np.concatenate([np.eye(d), -np.eye(d)]).astype(np.float32)[None], "bf16")
    ids, vals = run(x, W, np.zeros((1, 2 * d), np.float32), k, "bf16")
    xf = synth.bf16_bits_to_f32(x[0])
    for t in range(T):
        z = np.concatenate([xf[t], -xf[t]])                     # z is the input itself: no rounding anywhere
        want = np.argsort(-z, kind="stable")[:k]                # (z descending, id ascending)
        assert ids[0, t].tolist() == want.tolist()
        assert np.array_equal(vals[0, t], z[want])
        # the selected features are the k largest |x_c|, each in the half that matches its sign
        assert np.array_equal(np.sort(np.abs(xf[t]))[-k:], np.sort(vals[0, t]))


def test_bitwise_deterministic():
    w = synth.shrink(synth.WORKLOADS["c2_llama8b"], T=256, L=256, n_feat=4096)
    x, W, b = parity.head_inputs(w, [3])
    a = run(x, W, b, w.k, w.dtype)
    c = run(x, W, b, w.k, w.dtype)
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])


def test_streamed_calls_equal_plain_calls_whatever_the_carried_threshold_holds():
    """Chunks of one stream through s3_sae_encode_topk_stream: bit-identical to s3_sae_encode_topk with the
    thresholds carried from chunk to chunk, with no carried threshold, and with one that is absurdly high
    (every token is then selected again from scratch inside the call)."""
    import torch
    import paper_2601_17702_amd as s3
    from oracle import s3_oracle as orc
    w = synth.shrink(synth.WORKLOADS["c2_llama8b"], L=3 * 600, T=600, n_feat=2048)
    heads = [0, 3, 9]
    W, b = np.stack([synth.gen_w_enc(w, h) for h in heads]), np.stack([synth.gen_b_enc(w, h) for h in heads])
    Wg, bg = parity.to_gpu(W, w.dtype), parity.to_gpu(b, "fp32")
    hint = s3.new_tau_hint(len(heads))
    seen = []
    for c in range(w.n_chunks):
        x = np.stack([synth.gen_keys(w, h, c) for h in heads])
        xg = parity.to_gpu(x, w.dtype)
        ids0, vals0 = s3.sae_encode_topk(xg, Wg, bg, w.k)
        before = hint.clone()
        ids1, vals1 = s3.sae_encode_topk_stream(xg, Wg, bg, w.k, hint)
        torch.cuda.synchronize()
        assert torch.equal(ids0, ids1) and torch.equal(vals0, vals1)
        h_now = hint.cpu().numpy()
        assert np.all(np.isfinite(h_now).sum(axis=1) == 1) and not torch.equal(before, hint)   # one bound per head is carried
        # the carried values are lower bounds of this chunk's thresholds: tau_t >= k-th largest oracle value - rounding
        o = orc.encode_topk(x[0], W[0], b[0], w.k, w.dtype)
        kth = o["zsel"][:, -1]
        nx = np.linalg.norm(synth.storage_to_f64(x[0], w.dtype), axis=1)
        assert h_now[0, 1] <= kth.min() * (1 + 1e-3) + 1e-6 and h_now[0, 0] <= (kth / nx).min() * (1 + 1e-3) + 1e-6
        assert np.isfinite(h_now[0, 0])                        # W x dominates here: the |x|-scaled bound is the tighter one
        seen.append(h_now.copy())
        for bad in (1e30, -1e30, float("nan")):
            hb = torch.full_like(hint, bad)
            ids2, vals2 = s3.sae_encode_topk_stream(xg, Wg, bg, w.k, hb)
            torch.cuda.synchronize()
            assert torch.equal(ids0, ids2) and torch.equal(vals0, vals2), bad
    assert np.allclose(seen[1][:, 0], seen[2][:, 0], rtol=0.2)          # the statistic is stable from chunk to chunk
    # the k <= 64 build of the kernel (4 wavefronts per workgroup, one token per sort step), streamed as well
    w4 = synth.shrink(synth.WORKLOADS["c4_qwen7b"], L=2 * 300, T=300, n_feat=4096)
    W4, b4 = np.stack([synth.gen_w_enc(w4, h) for h in (0, 1)]), np.stack([synth.gen_b_enc(w4, h) for h in (0, 1)])
    W4g, b4g = parity.to_gpu(W4, w4.dtype), parity.to_gpu(b4, "fp32")
    h4 = s3.new_tau_hint(2)
    for c in range(w4.n_chunks):
        x = np.stack([synth.gen_keys(w4, h, c) for h in (0, 1)])
        xg = parity.to_gpu(x, w4.dtype)
        a0 = s3.sae_encode_topk(xg, W4g, b4g, w4.k)
        a1 = s3.sae_encode_topk_stream(xg, W4g, b4g, w4.k, h4)
        a2 = s3.sae_encode_topk_stream(xg, W4g, b4g, w4.k, torch.full_like(h4, 1e30))
        torch.cuda.synchronize()
        assert torch.equal(a0[0], a1[0]) and torch.equal(a0[1], a1[1]) and torch.equal(a0[0], a2[0]) and torch.equal(a0[1], a2[1])
        ties, rows = parity.check_encode(a1[0].cpu().numpy(), a1[1].cpu().numpy(), x, W4, b4, w4.k, w4.dtype)
    # shapes outside the threshold-carrying kernel: same results, hint untouched
    w4 = synth.shrink(synth.WORKLOADS["c4_qwen7b"], L=200, T=200, n_feat=1000)
    x, W4, b4 = parity.head_inputs(w4, [0])
    h4 = s3.new_tau_hint(1)
    a = s3.sae_encode_topk(parity.to_gpu(x, w4.dtype), parity.to_gpu(W4, w4.dtype), parity.to_gpu(b4, "fp32"), w4.k)
    bb = s3.sae_encode_topk_stream(parity.to_gpu(x, w4.dtype), parity.to_gpu(W4, w4.dtype), parity.to_gpu(b4, "fp32"), w4.k, h4)
    torch.cuda.synchronize()
    assert torch.equal(a[0], bb[0]) and torch.equal(a[1], bb[1]) and torch.all(torch.isinf(h4))


@pytest.mark.parametrize("T,n_feat,k,heads", [
    (1, 128, 32, 1),        # a single token, the smallest dictionary the fast kernel takes
    (33, 256, 64, 3),       # k = 64 build, heads not a multiple of 8, ragged wavefront
    (257, 128, 64, 9),      # half of all features are selected; one token in the second workgroup
    (40, 384, 17, 2),
])
def test_fast_kernel_edge_shapes_plain_and_streamed(T, n_feat, k, heads):
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(T * 7 + n_feat + k)
    x = synth.to_storage(rng.standard_normal((heads, T, 128)).astype(np.float32) * 3, "bf16")
    W = synth.to_storage((rng.standard_normal((heads, n_feat, 128)) / np.sqrt(128)).astype(np.float32), "bf16")
    b = (0.1 * rng.standard_normal((heads, n_feat))).astype(np.float32)
    xg, Wg, bg = parity.to_gpu(x, "bf16"), parity.to_gpu(W, "bf16"), parity.to_gpu(b, "fp32")
    ids0, vals0 = s3.sae_encode_topk(xg, Wg, bg, k)
    torch.cuda.synchronize()
    ties, rows = parity.check_encode(ids0.cpu().numpy(), vals0.cpu().numpy(), x, W, b, k, "bf16")
    hint = s3.new_tau_hint(heads)
    for _ in range(3):                                    # same chunk again and again: the carried bound is as tight as it gets
        ids1, vals1 = s3.sae_encode_topk_stream(xg, Wg, bg, k, hint)
        torch.cuda.synchronize()
        assert torch.equal(ids0, ids1) and torch.equal(vals0, vals1)
