"""Pins of the oracle's SAE training step (Sec. 3.3 equations, App. B.3 optimiser) against things other than
itself: finite differences of its own loss, the matrix form of the dense (k = n_feat, all active) case written with
library matmuls, Adam's closed form for a constant gradient, the rounding rule against numpy integer arithmetic,
the pinned encoder, and the behaviour the objective must have (the loss goes down on data drawn from a dictionary)."""
import numpy as np
import pytest

from oracle import s3_oracle as orc
from paper_2601_17702_amd import synth


def small_problem(seed, B=7, d=8, n_feat=24):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, d)).astype(np.float32)
    w_enc = rng.standard_normal((n_feat, d)) / np.sqrt(d)
    b_enc = 0.1 * rng.standard_normal(n_feat)
    w_dec = rng.standard_normal((n_feat, d)) / np.sqrt(d)
    b_dec = 0.1 * rng.standard_normal(d)
    return x, w_enc, b_enc, w_dec, b_dec


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_gradients_match_central_differences(seed):
    x, w_enc, b_enc, w_dec, b_dec = small_problem(seed)
    k = 5
    base = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, k, round_bf16=False)
    rng = np.random.default_rng(100 + seed)
    params = {"g_w_enc": w_enc, "g_b_enc": b_enc, "g_w_dec": w_dec, "g_b_dec": b_dec}
    h = 1e-6
    checked = 0
    for name, arr in params.items():
        flat = arr.reshape(-1)
        # entries that matter: for the per-feature parameters, features that some token selected
        used = np.unique(base["ids"])
        cand = [int(f) * (arr.size // len(b_enc)) + int(rng.integers(arr.size // len(b_enc))) for f in used[:6]] \
            if arr.shape[0] == len(b_enc) else list(range(arr.size))
        for i in cand[:8]:
            old = flat[i]
            flat[i] = old + h
            lp = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, k, round_bf16=False)
            flat[i] = old - h
            lm = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, k, round_bf16=False)
            flat[i] = old
            if not (np.array_equal(lp["ids"], base["ids"]) and np.array_equal(lm["ids"], base["ids"])):
                continue                       # the perturbation moved the selection: not a point where L is smooth
            fd = (lp["loss"] - lm["loss"]) / (2 * h)
            an = base[name].reshape(-1)[i]
            assert abs(fd - an) <= 1e-7 + 1e-5 * abs(an), (name, i, fd, an)
            checked += 1
    assert checked >= 20


def test_dense_case_equals_the_linear_autoencoder_in_matrix_form():
    """k = n_feat with a bias that keeps every pre-activation positive: the SAE is z = U W_enc^T + b, xhat = z W_dec +
    b_dec, whose gradients are textbook matrix products."""
    x, w_enc, b_enc, w_dec, b_dec = small_problem(5, B=9, d=6, n_feat=10)
    b_enc = b_enc + 50.0
    r = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, k=10, round_bf16=False)
    X = x.astype(np.float64)
    U = X - b_dec
    Z = U @ w_enc.T + b_enc
    assert Z.min() > 0
    R = Z @ w_dec + b_dec - X
    n = X.size
    G = 2 * R / n
    np.testing.assert_allclose(r["loss"], (R ** 2).sum() / n, rtol=1e-13)
    dZ = G @ w_dec.T
    np.testing.assert_allclose(r["g_w_dec"], Z.T @ G, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(r["g_w_enc"], dZ.T @ U, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(r["g_b_enc"], dZ.sum(0), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(r["g_b_dec"], G.sum(0) - (dZ @ w_enc).sum(0), rtol=1e-11, atol=1e-14)


def test_relu_and_topk_gate_the_gradient():
    """One token, hand-built: feature 0 selected and positive, feature 1 selected with a negative pre-activation
    (ReLU gives 0: it adds nothing and receives no gradient), feature 2 not selected."""
    x = np.array([[1.0, 2.0]], np.float32)
    w_enc = np.array([[1.0, 0.0], [-1.0, 0.0], [-5.0, -5.0]])
    b_enc = np.zeros(3)
    w_dec = np.array([[0.5, 0.25], [7.0, 7.0], [9.0, 9.0]])
    b_dec = np.zeros(2)
    r = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, k=2, round_bf16=False)
    assert r["ids"].tolist() == [[0, 1]]                       # z = (1, -1, -15)
    xhat = np.array([0.5, 0.25])                               # 1 * w_dec[0] + 0 * w_dec[1]
    res = xhat - np.array([1.0, 2.0])
    assert r["loss"] == pytest.approx((res ** 2).sum() / 2)
    g = 2 * res / 2
    np.testing.assert_allclose(r["g_w_dec"], [1.0 * g, 0 * g, 0 * g], atol=1e-15)
    dz0 = g @ w_dec[0]
    np.testing.assert_allclose(r["g_w_enc"], [dz0 * np.array([1.0, 2.0]), [0, 0], [0, 0]], atol=1e-15)
    np.testing.assert_allclose(r["g_b_enc"], [dz0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(r["g_b_dec"], g - dz0 * w_enc[0], atol=1e-15)


def test_given_selection_is_used():
    x, w_enc, b_enc, w_dec, b_dec = small_problem(3)
    own = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, 4, round_bf16=False)
    same = orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, 4, round_bf16=False, ids_in=own["ids"][:, ::-1].copy())
    assert same["loss"] == pytest.approx(own["loss"], rel=1e-14)          # the order inside a row does not matter
    np.testing.assert_allclose(same["g_w_dec"], own["g_w_dec"], rtol=1e-12, atol=1e-16)
    other = own["ids"].copy()
    other[0, 0] = [f for f in range(24) if f not in own["ids"][0]][0]
    assert orc.sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, 4, False, ids_in=other)["loss"] != own["loss"]


def test_bf16_rounding_is_round_to_nearest_even():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(500).astype(np.float32) * 10.0 ** rng.integers(-5, 5, 500).astype(np.float32),
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38], np.float32)])
    want = synth.to_storage(a, "bf16").astype(np.uint32) << 16        # the generators' rounding: integer arithmetic in numpy
    got = orc.bf16_round(a).view(np.uint32)
    assert np.array_equal(got, want)
    assert orc.bf16_round(np.float32(1.00390625)) == np.float32(1.0)           # halfway, even mantissa below
    assert orc.bf16_round(np.float32(1.01171875)) == np.float32(1.015625)      # halfway, odd mantissa below: up


def test_rounded_forward_selects_what_the_pinned_encoder_selects():
    x, w_enc, b_enc, w_dec, b_dec = small_problem(8, B=20, d=16, n_feat=64)
    w_enc32, b_enc32, b_dec32 = w_enc.astype(np.float32), b_enc.astype(np.float32), b_dec.astype(np.float32)
    r = orc.sae_loss_grad(x, w_enc32.astype(np.float64), b_enc32.astype(np.float64), w_dec, b_dec32.astype(np.float64),
                          6, round_bf16=True)
    u = synth.to_storage(x - b_dec32, "bf16")
    e = orc.encode_topk(u, synth.to_storage(w_enc32, "bf16"), b_enc32, 6, "bf16")
    assert np.array_equal(r["ids"], e["ids"])


def test_adam_closed_form_for_a_constant_gradient():
    rng = np.random.default_rng(1)
    g = rng.standard_normal(50) * 10.0 ** rng.integers(-6, 2, 50)
    p = rng.standard_normal(50)
    p0, m, v = p.copy(), np.zeros(50), np.zeros(50)
    lr, eps = 1e-3, 1e-8
    for step in (1, 2, 3):
        orc.adam(p, m, v, g, lr, 0.9, 0.999, eps, step)
        # bias-corrected moments of a constant gradient are the gradient and its square at every step
        np.testing.assert_allclose(p, p0 - step * lr * g / (np.abs(g) + eps), rtol=1e-12, atol=1e-15)
    with pytest.raises(ValueError):
        orc.adam(p, m, v, g, lr, 0.9, 0.999, eps, 0)


def test_training_lowers_the_loss_on_data_from_a_dictionary():
    rng = np.random.default_rng(4)
    d, n_feat, k, B = 16, 48, 4, 256
    D = rng.standard_normal((n_feat, d))
    D /= np.linalg.norm(D, axis=1, keepdims=True)
    def batch():
        x = np.zeros((B, d))
        for t in range(B):
            f = rng.choice(n_feat, k, replace=False)
            x[t] = (1.0 + rng.random(k)) @ D[f]
        return x.astype(np.float32)
    w_dec = D + 0.3 * rng.standard_normal((n_feat, d))
    w_enc = w_dec.copy()
    b_enc, b_dec = np.zeros(n_feat), np.zeros(d)
    P = [w_enc, b_enc, w_dec, b_dec]
    M = [np.zeros_like(a) for a in P]
    V = [np.zeros_like(a) for a in P]
    losses = []
    for step in range(1, 61):
        r = orc.sae_loss_grad(batch(), w_enc, b_enc, w_dec, b_dec, k, round_bf16=False)
        losses.append(r["loss"])
        for a, m, v, name in zip(P, M, V, ("g_w_enc", "g_b_enc", "g_w_dec", "g_b_dec")):
            orc.adam(a, m, v, r[name], 1e-2, 0.9, 0.999, 1e-8, step)
    assert np.mean(losses[-5:]) < 0.5 * np.mean(losses[:5])
