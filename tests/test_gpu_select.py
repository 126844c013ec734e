"""GPU parity of the rest of Phase 2 (density curve, peak selection, variable-length spans) and of the Phase-3 set
operations against the CPU oracle.  Inputs are seeded synthetic score arrays with the look of position scores: sparse,
non-negative, with a few dense clusters.  The oracle follows the same precision steps as the library (fp64 sum of
fp32 products rounded to fp32 once; decisions on those values), so centres, spans and index lists must be equal."""
import numpy as np
import pytest

from oracle import s3_oracle as orc

pytestmark = pytest.mark.gpu


def synth_scores(rng, L, clusters=6):
    S = rng.random(L).astype(np.float32) * (rng.random(L) < 0.05)
    for _ in range(clusters):
        c, w = int(rng.integers(0, L)), int(rng.integers(1, 80))
        a, b = max(0, c - w), min(L, c + w)
        S[a:b] += (rng.random(b - a) * 3 * (rng.random(b - a) < 0.6)).astype(np.float32)
    return S.astype(np.float32)


def oracle_select(S32, g32, n_centers, radius, rel, max_half):
    D64 = orc.conv1d(S32.astype(np.float64), g32.astype(np.float64))
    D32 = D64.astype(np.float32)                                  # the one rounding
    Dd = D32.astype(np.float64)                                   # every decision is taken on the fp32 values
    centers, peak = orc.nms_peaks(Dd, n_centers, radius)
    lo, hi = orc.grow_spans(Dd, centers, float(np.float32(rel)), max_half)
    return D32, centers, peak, lo, hi


@pytest.mark.parametrize("L,kind,K,n_centers,radius,rel,max_half", [
    (5000, "box", 48, 40, 24, 0.5, 64),            # the paper's sizes: kernel 48, 40 centres
    (5000, "box", 8, 40, 4, 0.5, 16),              # kernel 8 (QA setting)
    (100_000, "gaussian", 48, 40, 48, 0.25, 200),  # many tiles, spans longer than a wavefront step
    (100_000, "triangular", 9, 64, 0, 0.75, 5),    # odd kernel, no suppression radius
    (1500, "gaussian", 7, 10, 3000, 0.0, 4000),    # radius and half length beyond the context: one centre, whole context
    (37, "box", 48, 5, 2, 0.5, 3),                 # context shorter than the kernel
    (1, "box", 1, 3, 0, 1.0, 0),                   # a single position
    (3000, "box", 48, 4096, 1, 1.0, 0),            # more centres asked for than there are peaks
])
def test_select_spans_vs_oracle(L, kind, K, n_centers, radius, rel, max_half):
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(L + K + n_centers)
    S = synth_scores(rng, L) if L > 1 else np.array([2.0], np.float32)
    g = s3.smoothing_kernel({"box": 0, "triangular": 1, "gaussian": 2}[kind], K)
    g32 = g.cpu().numpy()
    assert np.allclose(g32, orc.smoothing_kernel(kind, K), rtol=1e-6, atol=0)       # the library's weights are the oracle's
    c, dc, lo, hi, nf, D = s3.select_spans(torch.from_numpy(S).cuda(), g, n_centers, radius, rel, max_half, want_density=True)
    torch.cuda.synchronize()
    D32, c_o, pk_o, lo_o, hi_o = oracle_select(S, g32, n_centers, radius, rel, max_half)
    assert np.array_equal(D.cpu().numpy(), D32)
    n = int(nf.item())
    assert n == len(c_o) and n >= 1
    assert np.array_equal(c.cpu().numpy()[:n], c_o) and np.array_equal(dc.cpu().numpy()[:n], pk_o.astype(np.float32))
    assert np.array_equal(lo.cpu().numpy()[:n], lo_o) and np.array_equal(hi.cpu().numpy()[:n], hi_o)
    assert np.all(c.cpu().numpy()[n:] == -1) and np.all(lo.cpu().numpy()[n:] == -1) and np.all(hi.cpu().numpy()[n:] == -1)
    # same result again, and without the density output (the curve then lives in the workspace)
    c2, _, lo2, hi2, nf2, _ = s3.select_spans(torch.from_numpy(S).cuda(), g, n_centers, radius, rel, max_half)
    torch.cuda.synchronize()
    assert torch.equal(c, c2) and torch.equal(lo, lo2) and torch.equal(hi, hi2) and torch.equal(nf, nf2)


def test_select_spans_without_evidence_and_argument_errors():
    import torch
    import paper_2601_17702_amd as s3
    g = s3.smoothing_kernel(s3.KERNEL_BOX, 8)
    c, dc, lo, hi, nf, D = s3.select_spans(torch.zeros(1000, device="cuda"), g, 5, 4, 0.5, 10, want_density=True)
    torch.cuda.synchronize()
    assert int(nf.item()) == 0 and torch.all(c == -1) and torch.all(D == 0)
    S = torch.ones(10, device="cuda")
    for bad in (dict(n_centers=0), dict(nms_radius=-1), dict(rel_threshold=1.5), dict(max_half_len=-1)):
        kw = dict(n_centers=3, nms_radius=1, rel_threshold=0.5, max_half_len=2)
        kw.update(bad)
        with pytest.raises(s3.S3Error) as e:
            s3.select_spans(S, g, kw["n_centers"], kw["nms_radius"], kw["rel_threshold"], kw["max_half_len"])
        assert e.value.code == -1


@pytest.mark.parametrize("L,lead,tail,n_extra", [(5000, 16, 16, 100), (100_000, 0, 0, 0), (70_000, 128, 64, 5000), (9, 20, 0, 3)])
def test_fuse_indices_vs_oracle(L, lead, tail, n_extra):
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(L + lead + n_extra)
    ns = 40
    lo = rng.integers(0, L, ns).astype(np.int32)
    hi = (lo + rng.integers(0, 300, ns)).astype(np.int32)                      # some run past the end
    extra = rng.integers(-10, L + 10, n_extra).astype(np.int32)
    for n_used in (ns, 7, 0):
        nsp = torch.tensor([n_used], dtype=torch.int32, device="cuda")
        mask, idx, n_out = s3.fuse_indices(L, torch.from_numpy(lo).cuda(), torch.from_numpy(hi).cuda(), nsp,
                                           torch.from_numpy(extra).cuda() if n_extra else None, lead, tail)
        torch.cuda.synchronize()
        m_o, idx_o = orc.fuse(L, lo[:n_used], hi[:n_used], extra, lead, tail)
        n = int(n_out.item())
        assert n == len(idx_o)
        assert np.array_equal(mask.cpu().numpy(), m_o) and np.array_equal(idx.cpu().numpy()[:n], idx_o)


def test_scores_to_fused_indices_chain():
    """The chain s3_coactivate_score (scores_out) -> s3_select_spans -> s3_fuse_indices on one small index against the
    oracle's own chain (its scores, rounded to fp32 as the library hands them on, feed its selection; nothing it sees
    comes from the GPU): scores within 2e-3, centres and the fused index list equal (a seed without a near-tie)."""
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(5)
    H, T, k, n_feat, nq = 2, 3000, 16, 512, 12
    ids = np.stack([np.stack([rng.choice(n_feat, k, replace=False) for _ in range(T)]) for _ in range(H)]).astype(np.int32)
    qids = np.stack([np.stack([rng.choice(n_feat, k, replace=False) for _ in range(nq)]) for _ in range(H)]).astype(np.int32)
    qvals = rng.random((H, nq, k)).astype(np.float32)
    ix = s3.Index(H, n_feat, k, T)
    ix.append(torch.from_numpy(ids).cuda())
    ix.finalize()
    _, _, _, S = ix.coactivate_score(torch.from_numpy(qids).cuda(), torch.from_numpy(qvals).cuda(), T, 32, 4, want_scores=True)
    S_o = np.zeros(T)
    for h in range(H):
        oi = orc.Index(n_feat)
        oi.append(ids[h], np.arange(T, dtype=np.int32))
        oi.score_accumulate(qids[h], qvals[h], S_o)
    torch.cuda.synchronize()
    S32 = S.cpu().numpy()
    assert np.allclose(S32, S_o, rtol=2e-3)
    g = s3.smoothing_kernel(s3.KERNEL_TRIANGULAR, 48)
    c, dc, lo, hi, nf, _ = s3.select_spans(S, g, 40, 24, 0.5, 32)
    mask, idx, n_out = s3.fuse_indices(T, lo, hi, nf, None, 16, 16)
    torch.cuda.synchronize()
    _, c_o, _, lo_o, hi_o = oracle_select(S_o.astype(np.float32), g.cpu().numpy(), 40, 24, 0.5, 32)
    n = int(nf.item())
    assert n == len(c_o) and np.array_equal(c.cpu().numpy()[:n], c_o)
    m_o, idx_o = orc.fuse(T, lo_o, hi_o, np.zeros(0, np.int32), 16, 16)
    assert np.array_equal(idx.cpu().numpy()[:int(n_out.item())], idx_o) and np.array_equal(mask.cpu().numpy(), m_o)
