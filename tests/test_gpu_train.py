"""GPU parity of s3_sae_train_step (one Adam step of the Top-K SAE on the reconstruction error) against the fp64
oracle: selection checked like every encoder output, loss / gradients / updated parameters against the oracle run on
the same selection."""
import numpy as np
import pytest

from oracle import s3_oracle as orc
from paper_2601_17702_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

NAMES = ("g_w_enc", "g_b_enc", "g_w_dec", "g_b_dec")


def make_problem(seed, B, n_feat, d=128):
    rng = np.random.default_rng(seed)
    basis = rng.standard_normal((24, d)) / np.sqrt(24)
    x = (rng.standard_normal((B, 24)) @ basis + 0.3 * rng.standard_normal((B, d))).astype(np.float32)
    w = rng.standard_normal((n_feat, d)).astype(np.float32)
    w /= np.linalg.norm(w, axis=1, keepdims=True)
    w_enc = w.copy()
    w_dec = (w + 0.05 * rng.standard_normal((n_feat, d))).astype(np.float32)
    b_enc = (0.02 * rng.standard_normal(n_feat)).astype(np.float32)
    b_dec = (0.05 * rng.standard_normal(d)).astype(np.float32)
    return x, [w_enc, b_enc, w_dec, b_dec]


def unpack(flat, n_feat, d):
    a, b = n_feat * d, n_feat * d + n_feat
    return [flat[:a].reshape(n_feat, d), flat[a:b], flat[b:b + a].reshape(n_feat, d), flat[b + a:]]


def check_step(tr, x, P64, M, V, k, step, lr, sample_rows=None):
    """One GPU step on x against the oracle; P64 / M / V are the oracle's fp64 parameters and moments (updated)."""
    import torch
    n_feat, d = P64[0].shape
    before = [p.copy() for p in P64]
    loss, ids, grads = tr.step(torch.from_numpy(x).cuda(), want_ids=True, want_grads=True)
    torch.cuda.synchronize()
    gi = ids.cpu().numpy()
    # selection: the encoder's operands as the step defines them, checked like any encoder output
    u = synth.to_storage(x - before[3].astype(np.float32), "bf16")
    wb = synth.to_storage(before[0].astype(np.float32), "bf16")
    rows = np.arange(x.shape[0]) if sample_rows is None else sample_rows
    o = orc.encode_topk(u[rows], wb, before[1].astype(np.float32), k, "bf16")
    same = np.sort(gi[rows], 1) == np.sort(o["ids"], 1)
    for r in np.flatnonzero(~same.all(axis=1)):
        assert o["gap"][r] < parity.TIE_GAP, f"row {rows[r]}: selection differs at gap {o['gap'][r]:.2e}"
    assert np.all(np.diff(np.sort(gi, 1), axis=1) > 0) and gi.min() >= 0 and gi.max() < n_feat
    # everything else on the GPU's own selection
    r = orc.sae_loss_grad(x, *before, k, round_bf16=True, ids_in=gi)
    assert float(loss.item()) == pytest.approx(r["loss"], rel=2e-5)
    got = unpack(grads.cpu().numpy().astype(np.float64), n_feat, d)
    tols = []
    for name, g in zip(NAMES, got):
        want = r[name]
        # fp32 sums of up to B terms against fp64: relative to the entry and to the size of the terms around it
        tol = 2e-4 * np.abs(want) + 2e-5 * np.sqrt(np.mean(want ** 2)) + 1e-12
        tols.append(tol)
        bad = np.abs(g - want) > tol
        assert not bad.any(), f"{name}: {int(bad.sum())} entries off, worst {np.abs(g - want).max():.3e} (rms {np.sqrt(np.mean(want**2)):.3e})"
    for p, m, v, name in zip(P64, M, V, NAMES):
        orc.adam(p, m, v, r[name], lr, 0.9, 0.999, 1e-8, step)
    now = [tr.w_enc, tr.b_enc, tr.w_dec, tr.b_dec]
    eps = 1e-8
    for p, t, name, tol in zip(P64, now, NAMES, tols):
        gp = t.cpu().numpy().astype(np.float64)
        g = np.abs(r[name])
        # Adam divides by |g| + eps (step 1; about that later on): where a gradient is as small as eps, an error dg in
        # it moves the update by lr * dg * eps / (|g| + eps)^2 -- the update itself is never more than about lr
        ptol = lr * np.minimum(2.0, 1e-5 + 4.0 * tol * eps / (g + eps) ** 2) + 1e-7
        bad = np.abs(gp - p) > ptol
        assert not bad.any(), f"parameters behind {name}: {int(bad.sum())} off, worst {np.abs(gp - p).max():.3e}"
    return r["loss"]


@pytest.mark.parametrize("B,n_feat,k", [(256, 1024, 16), (130, 512, 128), (64, 128, 1), (300, 2048, 33)])
def test_two_steps_against_oracle(B, n_feat, k):
    import torch
    import paper_2601_17702_amd as s3
    lr = 1e-3
    x1, P32 = make_problem(B + n_feat + k, B, n_feat)
    x2, _ = make_problem(B + n_feat + k + 1, B, n_feat)
    tr = s3.SaeTrainer(*[torch.from_numpy(p.copy()).cuda() for p in P32], k=k, batch=B, lr=lr)
    P64 = [p.astype(np.float64) for p in P32]
    M = [np.zeros_like(p) for p in P64]
    V = [np.zeros_like(p) for p in P64]
    check_step(tr, x1, P64, M, V, k, 1, lr)
    # the oracle goes on from the GPU's fp32 parameters, so that the second step is compared on equal inputs
    P64 = [t.cpu().numpy().astype(np.float64) for t in (tr.w_enc, tr.b_enc, tr.w_dec, tr.b_dec)]
    check_step(tr, x2, P64, M, V, k, 2, lr)


def test_paper_configuration_full_batch():
    """App. B.3: expansion 128 (16384 latents), k = 128, 4096 tokens per batch: selection on sampled rows, loss,
    gradients and parameters everywhere."""
    import torch
    import paper_2601_17702_amd as s3
    B, n_feat, k, lr = 4096, 16384, 128, 1e-3
    x, P32 = make_problem(7, B, n_feat)
    tr = s3.SaeTrainer(*[torch.from_numpy(p.copy()).cuda() for p in P32], k=k, batch=B, lr=lr)
    P64 = [p.astype(np.float64) for p in P32]
    M = [np.zeros_like(p) for p in P64]
    V = [np.zeros_like(p) for p in P64]
    rows = np.random.default_rng(0).choice(B, 48, replace=False)
    check_step(tr, x, P64, M, V, k, 1, lr, sample_rows=np.sort(rows))


def test_step_is_bit_reproducible_and_loss_goes_down():
    import torch
    import paper_2601_17702_amd as s3
    B, n_feat, k = 512, 1024, 8
    outs = []
    for rep in range(2):
        x, P32 = make_problem(11, B, n_feat)
        tr = s3.SaeTrainer(*[torch.from_numpy(p.copy()).cuda() for p in P32], k=k, batch=B, lr=3e-3)
        losses = []
        for s in range(40):
            xb, _ = make_problem(1000 + s, B, n_feat)
            losses.append(float(tr.step(torch.from_numpy(xb).cuda())[0].item()))
        outs.append((losses, tr.w_enc.cpu().numpy().copy(), tr.w_dec.cpu().numpy().copy()))
    assert outs[0][0] == outs[1][0] and np.array_equal(outs[0][1], outs[1][1]) and np.array_equal(outs[0][2], outs[1][2])
    assert np.mean(outs[0][0][-5:]) < 0.9 * np.mean(outs[0][0][:5])


def test_errors():
    import torch
    import paper_2601_17702_amd as s3
    x, P32 = make_problem(3, 64, 256)
    with pytest.raises(s3.S3Error):
        s3.SaeTrainer(*[torch.from_numpy(p[..., :64].copy() if p.ndim == 2 else (p[:64].copy() if p.shape[0] == 128 else p.copy())).cuda()
                        for p in P32], k=8, batch=64)                      # d_head 64: not supported
    tr = s3.SaeTrainer(*[torch.from_numpy(p.copy()).cuda() for p in P32], k=8, batch=64)
    tr.ws = tr.ws[:1024]
    with pytest.raises(s3.S3Error):
        tr.step(torch.from_numpy(x).cuda())
