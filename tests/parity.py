"""Helpers shared by the GPU parity tests: move generated inputs to the GPU, compare with the oracle."""
import numpy as np

from oracle import s3_oracle as orc
from paper_2601_17702_amd import synth

REL_TOL = 2e-3        # activations and scores: bf16 inputs, fp32 accumulation
TIE_GAP = 1e-3        # a row may differ from the oracle only if its k-th/(k+1)-th relative gap is below this


def to_gpu(a: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16" and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def head_inputs(w: synth.Workload, heads, chunk=0):
    x = np.stack([synth.gen_keys(w, h, chunk) for h in heads])
    W = np.stack([synth.gen_w_enc(w, h) for h in heads])
    b = np.stack([synth.gen_b_enc(w, h) for h in heads])
    return x, W, b


def check_encode(ids_g, vals_g, x, W, b, k, dtype, want_dense=False):
    """ids_g/vals_g [H, T, k] numpy from the GPU; x/W/b stored host arrays.  Returns (tie_rows, rows)."""
    H, T = ids_g.shape[:2]
    ties = 0
    for h in range(H):
        o = orc.encode_topk(x[h], W[h], b[h], k, dtype, want_dense=want_dense)
        for t in range(T):
            gi, oi = ids_g[h, t], o["ids"][t]
            assert len(set(gi.tolist())) == k, f"head {h} row {t}: ids not distinct"
            assert np.all(np.diff(vals_g[h, t]) <= 0), f"head {h} row {t}: values not in descending order"
            if not np.array_equal(gi, oi):
                if set(gi.tolist()) == set(oi.tolist()):
                    # same set, different order: only allowed among (near-)equal values
                    zo = dict(zip(oi.tolist(), o["zsel"][t].tolist()))
                    zg = np.array([zo[f] for f in gi.tolist()])
                    assert np.all(np.diff(zg) <= REL_TOL * np.abs(zg[:-1]) + 1e-6), f"head {h} row {t}: wrong order"
                else:
                    assert o["gap"][t] < TIE_GAP, (
                        f"head {h} row {t}: id set differs, gap {o['gap'][t]:.3e}: gpu {sorted(gi.tolist())} "
                        f"oracle {sorted(oi.tolist())}")
                    ties += 1
                    if want_dense:   # whatever was picked instead must be as good as the k-th value within the gap
                        zk = o["zsel"][t, -1]
                        assert o["z"][t, gi].min() >= zk - TIE_GAP * abs(zk)
            common = {f: j for j, f in enumerate(oi.tolist())}
            for j, f in enumerate(gi.tolist()):
                if f in common:
                    ov = o["vals"][t, common[f]]
                    assert abs(vals_g[h, t, j] - ov) <= REL_TOL * abs(ov) + 1e-6, (
                        f"head {h} row {t} feature {f}: {vals_g[h, t, j]} vs {ov}")
    return ties, H * T
