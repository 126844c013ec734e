"""ctypes loader for the CPU oracle (oracle/s3_oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg; never by the
product package.  Argument marshalling for the C++ file, which holds the arithmetic -- with one exception,
score_dense at the end: the scoring equation of Sec. 3.5 evaluated token by token in numpy, for contexts
where building every head's std::map postings on the host would take too long.  It is pinned by the
hand-computed case, by App. D.2's set-intersection sum written out with Python sets, and against the
postings form (tests/test_oracle_pins.py).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s3_oracle.cpp")
_LIB = os.path.join(_HERE, "libs3oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (g++, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", _LIB, _SRC])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.orc_encode_topk.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, vp, C.c_int, C.c_int, vp, vp, vp, vp, vp]
        L.orc_encode_topk.restype = C.c_int
        L.orc_preact_at.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, vp, C.c_int, vp, C.c_int, vp]
        L.orc_preact_at.restype = C.c_int
        L.orc_index_new.restype = vp
        L.orc_index_free.argtypes = [vp]
        L.orc_index_append.argtypes = [vp, vp, vp, C.c_int, C.c_int]
        L.orc_index_postings.argtypes = [vp]
        L.orc_index_postings.restype = i64
        L.orc_index_export.argtypes = [vp, C.c_int, vp, vp]
        L.orc_idf.argtypes = [i64]
        L.orc_idf.restype = C.c_double
        L.orc_score_accumulate.argtypes = [vp, vp, vp, C.c_int, C.c_int, i32, vp, i64]
        L.orc_pool.argtypes = [vp, i64, C.c_int, vp]
        L.orc_pool.restype = i64
        L.orc_topb.argtypes = [vp, i64, C.c_int, C.c_int, C.c_int, vp, vp]
        L.orc_threads.restype = C.c_int
        L.orc_compact_encode.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, i32, vp, vp, vp]
        L.orc_compact_encode.restype = i64
        L.orc_compact_decode.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, vp, vp]
        L.orc_compact_decode.restype = i64
        L.orc_smoothing_kernel.argtypes = [C.c_int, C.c_int, vp]
        L.orc_conv1d.argtypes = [vp, i64, vp, C.c_int, vp]
        L.orc_nms_peaks.argtypes = [vp, i64, C.c_int, C.c_int, vp, vp]
        L.orc_grow_span.argtypes = [vp, i64, i32, C.c_double, C.c_int, vp, vp]
        L.orc_grow_span.restype = None
        L.orc_fuse.argtypes = [i64, vp, vp, C.c_int, vp, i64, C.c_int, C.c_int, vp, vp]
        L.orc_fuse.restype = i64
        L.orc_bf16_round.argtypes = [C.c_float]
        L.orc_bf16_round.restype = C.c_float
        L.orc_sae_loss_grad.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, C.c_int, vp, vp, vp,
                                        vp, vp, vp, vp]
        L.orc_adam.argtypes = [vp, vp, vp, vp, i64, C.c_double, C.c_double, C.c_double, C.c_double, C.c_int]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dt(dtype: str) -> int:
    return {"bf16": 0, "fp32": 1}[dtype]


def encode_topk(x, w, b, k, dtype, want_dense=False):
    """x [T, d], w [n_feat, d] as stored (uint16 bf16 bits or float32), b [n_feat] float32.
    Returns dict(ids [T,k] int32, vals [T,k] float32, zsel [T,k] f64, gap [T] f64, z [T,n_feat] f64|None)."""
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    b = np.ascontiguousarray(b, dtype=np.float32)
    want = np.float32 if dtype == "fp32" else np.uint16
    assert x.dtype == want and w.dtype == want
    T, d = x.shape
    n_feat = w.shape[0]
    ids = np.empty((T, k), np.int32)
    vals = np.empty((T, k), np.float32)
    zsel = np.empty((T, k), np.float64)
    gap = np.empty((T,), np.float64)
    z = np.empty((T, n_feat), np.float64) if want_dense else None
    rc = lib().orc_encode_topk(_p(x), _dt(dtype), T, d, _p(w), _p(b), n_feat, k, _p(ids), _p(vals), _p(zsel),
                               _p(gap), _p(z))
    if rc != 0:
        raise ValueError("orc_encode_topk: invalid arguments")
    return {"ids": ids, "vals": vals, "zsel": zsel, "gap": gap, "z": z}


def preact_at(x, w, b, ids, dtype):
    """Pre-activations z[t, j] of the features ids[t, j] (int32 [T, m]) for the stored x [T, d], w [n_feat, d],
    b [n_feat] float32: float64 [T, m]."""
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    b = np.ascontiguousarray(b, dtype=np.float32)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    want = np.float32 if dtype == "fp32" else np.uint16
    assert x.dtype == want and w.dtype == want and ids.ndim == 2 and ids.shape[0] == x.shape[0]
    z = np.empty(ids.shape, np.float64)
    rc = lib().orc_preact_at(_p(x), _dt(dtype), x.shape[0], x.shape[1], _p(w), _p(b), w.shape[0], _p(ids),
                             ids.shape[1], _p(z))
    if rc != 0:
        raise ValueError("orc_preact_at: invalid arguments or feature id outside [0, n_feat)")
    return z


class Index:
    """Inverted index of one (layer, head): feature id -> positions in insertion order."""

    def __init__(self, n_feat: int):
        self.n_feat = n_feat
        self._h = lib().orc_index_new()

    def append(self, ids, positions):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        positions = np.ascontiguousarray(positions, dtype=np.int32)
        assert ids.ndim == 2 and positions.shape == (ids.shape[0],)
        lib().orc_index_append(self._h, _p(ids), _p(positions), ids.shape[0], ids.shape[1])

    @property
    def n_postings(self) -> int:
        return int(lib().orc_index_postings(self._h))

    def csr(self):
        offsets = np.empty(self.n_feat + 1, np.int32)
        positions = np.empty(max(self.n_postings, 1), np.int32)
        rc = lib().orc_index_export(self._h, self.n_feat, _p(offsets), _p(positions))
        if rc != 0:
            raise ValueError("feature id outside [0, n_feat)")
        return offsets, positions[: self.n_postings]

    def score_accumulate(self, qids, qvals, S, max_freq=0):
        qids = np.ascontiguousarray(qids, dtype=np.int32)
        qvals = np.ascontiguousarray(qvals, dtype=np.float32)
        assert S.dtype == np.float64 and S.flags.c_contiguous
        rc = lib().orc_score_accumulate(self._h, _p(qids), _p(qvals), qids.shape[0], qids.shape[1], int(max_freq),
                                        _p(S), S.shape[0])
        if rc != 0:
            raise ValueError("position outside [0, L)")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_index_free(self._h)
            self._h = None


def idf(freq: int) -> float:
    return float(lib().orc_idf(int(freq)))


def pool(S, span_len):
    S = np.ascontiguousarray(S, dtype=np.float64)
    L = S.shape[0]
    W = np.empty(L - min(span_len, L) + 1, np.float64)
    nw = lib().orc_pool(_p(S), L, int(span_len), _p(W))
    assert nw == W.shape[0]
    return W


def topb(W, span_len, top_b, nms=True):
    W = np.ascontiguousarray(W, dtype=np.float64)
    starts = np.empty(top_b, np.int32)
    scores = np.empty(top_b, np.float64)
    n = lib().orc_topb(_p(W), W.shape[0], int(span_len), int(top_b), int(bool(nms)), _p(starts), _p(scores))
    return starts[:n].copy(), scores[:n].copy()


def compact_encode(offsets, positions, nblk, block_log2=14, prune_freq=0):
    """Plain CSR -> (cstart [nblk * n_feat + 1], delta uint16 [kept], cfreq [n_feat])."""
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    positions = np.ascontiguousarray(positions, dtype=np.int32)
    n_feat = offsets.shape[0] - 1
    cstart = np.empty(nblk * n_feat + 1, np.int32)
    delta = np.empty(max(positions.shape[0], 1), np.uint16)
    cfreq = np.empty(n_feat, np.int32)
    n = lib().orc_compact_encode(_p(offsets), _p(positions), n_feat, int(nblk), int(block_log2), int(prune_freq),
                                 _p(cstart), _p(delta), _p(cfreq))
    if n < 0:
        raise ValueError("orc_compact_encode: a list does not ascend or leaves the block range")
    return cstart, delta[:n].copy(), cfreq


def compact_decode(cstart, delta, n_feat, nblk, block_log2=14):
    cstart = np.ascontiguousarray(cstart, dtype=np.int32)
    delta = np.ascontiguousarray(delta, dtype=np.uint16)
    offsets = np.empty(n_feat + 1, np.int32)
    positions = np.empty(max(delta.shape[0], 1), np.int32)
    n = lib().orc_compact_decode(_p(cstart), _p(delta), n_feat, int(nblk), int(block_log2), _p(offsets), _p(positions))
    return offsets, positions[:n].copy()


KERNEL_KINDS = {"box": 0, "triangular": 1, "gaussian": 2}


def smoothing_kernel(kind: str, K: int):
    g = np.empty(K, np.float64)
    if lib().orc_smoothing_kernel(KERNEL_KINDS[kind], int(K), _p(g)) != 0:
        raise ValueError("orc_smoothing_kernel: invalid arguments")
    return g


def conv1d(S, g):
    S = np.ascontiguousarray(S, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float64)
    D = np.empty_like(S)
    lib().orc_conv1d(_p(S), S.shape[0], _p(g), g.shape[0], _p(D))
    return D


def nms_peaks(D, n_centers, radius):
    D = np.ascontiguousarray(D, dtype=np.float64)
    c = np.empty(n_centers, np.int32)
    v = np.empty(n_centers, np.float64)
    n = lib().orc_nms_peaks(_p(D), D.shape[0], int(n_centers), int(radius), _p(c), _p(v))
    return c[:n].copy(), v[:n].copy()


def grow_spans(D, centers, rel, max_half):
    D = np.ascontiguousarray(D, dtype=np.float64)
    lo = np.empty(len(centers), np.int32)
    hi = np.empty(len(centers), np.int32)
    a, b = C.c_int32(), C.c_int32()
    for i, c in enumerate(centers):
        lib().orc_grow_span(_p(D), D.shape[0], int(c), float(rel), int(max_half), C.byref(a), C.byref(b))
        lo[i], hi[i] = a.value, b.value
    return lo, hi


def fuse(L, lo, hi, extra, lead, tail):
    lo = np.ascontiguousarray(lo, dtype=np.int32)
    hi = np.ascontiguousarray(hi, dtype=np.int32)
    extra = np.ascontiguousarray(extra, dtype=np.int32)
    mask = np.empty(L, np.uint8)
    idx = np.empty(max(L, 1), np.int32)
    n = lib().orc_fuse(int(L), _p(lo), _p(hi), len(lo), _p(extra), extra.shape[0], int(lead), int(tail), _p(mask), _p(idx))
    return mask, idx[:n].copy()


def threads() -> int:
    return int(lib().orc_threads())


def score_dense(ids, qids, qvals, n_feat, max_freq=0):
    """Position scores of Sec. 3.5 written token by token instead of posting by posting.

    ids [H, L, k]: row t of head h holds the features active at position t; qids/qvals [H, nq, k].
    S[t] = sum over heads h and features f active at (h, t) of IDF_h(f) * (sum of the query
    activations of head h that name f); features with more than max_freq postings are skipped
    (max_freq > 0).  Same sum as Index.score_accumulate over all heads, in another order: used where
    building every head's postings on the host would take too long.
    """
    ids = np.asarray(ids)
    H, L, k = ids.shape
    S = np.zeros(L, np.float64)
    for h in range(H):
        freq = np.bincount(ids[h].reshape(-1), minlength=n_feat)
        act = np.zeros(n_feat, np.float64)
        np.add.at(act, np.asarray(qids[h]).reshape(-1), np.asarray(qvals[h], np.float64).reshape(-1))
        # one IDF value per distinct list length (the C++ orc_idf), 0 for lists the rule skips and for empty ones
        lengths, which = np.unique(freq, return_inverse=True)
        table = np.array([idf(int(fr)) if fr > 0 and not (max_freq > 0 and fr > max_freq) else 0.0 for fr in lengths])
        w = act * table[which.reshape(-1)]
        S += w[ids[h]].sum(axis=1)
    return S


def bf16_round(a):
    """float32 array rounded to the nearest bf16 value (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    f = lib().orc_bf16_round
    return np.array([f(float(v)) for v in a.ravel()], np.float32).reshape(a.shape)


def sae_loss_grad(x, w_enc, b_enc, w_dec, b_dec, k, round_bf16, ids_in=None):
    """Mean squared reconstruction error of the Top-K SAE on the batch x [B, d] (float32) and its gradients with
    the selection held fixed.  Parameters are float64 arrays (w_enc, w_dec [n_feat, d]; b_enc [n_feat]; b_dec [d]).
    Returns dict(loss, ids [B, k], g_w_enc, g_b_enc, g_w_dec, g_b_dec)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w_enc, b_enc, w_dec, b_dec = (np.ascontiguousarray(a, dtype=np.float64) for a in (w_enc, b_enc, w_dec, b_dec))
    B, d = x.shape
    n_feat = w_enc.shape[0]
    assert w_enc.shape == (n_feat, d) and w_dec.shape == (n_feat, d) and b_enc.shape == (n_feat,) and b_dec.shape == (d,)
    ids = np.empty((B, k), np.int32)
    loss = np.zeros(1, np.float64)
    g = [np.empty_like(w_enc), np.empty_like(b_enc), np.empty_like(w_dec), np.empty_like(b_dec)]
    if ids_in is not None:
        ids_in = np.ascontiguousarray(ids_in, dtype=np.int32)
        assert ids_in.shape == (B, k)
    rc = lib().orc_sae_loss_grad(_p(x), B, d, n_feat, k, _p(w_enc), _p(b_enc), _p(w_dec), _p(b_dec), int(round_bf16),
                                 _p(ids_in), _p(ids), _p(loss), _p(g[0]), _p(g[1]), _p(g[2]), _p(g[3]))
    if rc != 0:
        raise ValueError("orc_sae_loss_grad: invalid arguments")
    return {"loss": float(loss[0]), "ids": ids, "g_w_enc": g[0], "g_b_enc": g[1], "g_w_dec": g[2], "g_b_dec": g[3]}


def adam(p, m, v, grad, lr, b1, b2, eps, step):
    """One Adam update in place on float64 arrays of one shape."""
    for a in (p, m, v, grad):
        assert a.dtype == np.float64 and a.flags.c_contiguous and a.shape == p.shape
    rc = lib().orc_adam(_p(p), _p(m), _p(v), _p(grad), p.size, lr, b1, b2, eps, int(step))
    if rc != 0:
        raise ValueError("orc_adam: step must be >= 1")
