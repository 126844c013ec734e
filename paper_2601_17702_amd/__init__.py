"""Thin Python binding of libs3attn.so (C ABI in include/s3attn.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the library.
PyTorch supplies device memory and the current stream.  There is no CPU fallback: if the
library is not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs3attn.so")
_lib = None

S3_BF16, S3_FP32 = 0, 1
MAX_K, MAX_FEAT = 128, 65536


class S3Error(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"s3attn error {code}: {msg}")
        self.code = code


def lib():
    """Load the HIP library (built in-tree by paper_2601_17702_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_17702_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, ci, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_int, C.c_size_t
        L.s3_last_error.restype = C.c_char_p
        L.s3_sae_encode_topk.argtypes = [vp, ci, ci, ci, vp, vp, ci, ci, ci, vp, vp, vp]
        L.s3_sae_encode_topk_stream.argtypes = [vp, ci, ci, ci, vp, vp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
        L.s3_sae_encode_topk_stream_workspace.argtypes = [ci, ci]
        L.s3_sae_encode_topk_stream_workspace.restype = sz
        L.s3_index_create.argtypes = [ci, ci, ci, i64, C.POINTER(vp)]
        L.s3_index_destroy.argtypes = [vp]
        L.s3_index_destroy.restype = None
        L.s3_index_append.argtypes = [vp, vp, ci, vp, i32, vp]
        L.s3_index_finalize.argtypes = [vp, vp]
        L.s3_index_csr.argtypes = [vp, ci, C.POINTER(vp), C.POINTER(vp), C.POINTER(i64)]
        L.s3_index_export.argtypes = [vp, ci, vp, vp, vp]
        L.s3_index_export.restype = ci
        L.s3_index_reset.argtypes = [vp]
        L.s3_index_reset.restype = ci
        L.s3_index_tokens.argtypes = [vp]
        L.s3_index_tokens.restype = i64
        L.s3_index_build_workspace.argtypes = [ci, ci, ci]
        L.s3_index_build_workspace.restype = sz
        L.s3_index_build.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, sz, vp]
        L.s3_index_build_static.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp]
        L.s3_index_build_static.restype = ci
        L.s3_coactivate_score_workspace.argtypes = [vp, i64]
        L.s3_coactivate_score_workspace.restype = sz
        L.s3_coactivate_score.argtypes = [vp, vp, vp, ci, i64, ci, ci, i32, ci, vp, vp, vp, vp, vp, sz, vp]
        L.s3_smoothing_kernel.argtypes = [ci, ci, vp]
        L.s3_smoothing_kernel.restype = ci
        L.s3_select_spans_workspace.argtypes = [i64]
        L.s3_select_spans_workspace.restype = sz
        L.s3_select_spans.argtypes = [vp, i64, vp, ci, ci, ci, C.c_float, ci, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.s3_select_spans.restype = ci
        L.s3_fuse_indices_workspace.argtypes = [i64]
        L.s3_fuse_indices_workspace.restype = sz
        L.s3_fuse_indices.argtypes = [i64, vp, vp, vp, ci, vp, i64, ci, ci, vp, vp, vp, vp, sz, vp]
        L.s3_fuse_indices.restype = ci
        L.s3_index_compact_bytes.argtypes = [vp]
        L.s3_index_compact_bytes.restype = sz
        L.s3_index_compact.argtypes = [vp, i32, vp, sz, C.POINTER(vp), vp]
        L.s3_index_compact.restype = ci
        L.s3_cindex_destroy.argtypes = [vp]
        L.s3_cindex_destroy.restype = None
        L.s3_cindex_info.argtypes = [vp, C.POINTER(ci), C.POINTER(i64)]
        L.s3_cindex_info.restype = ci
        L.s3_cindex_export.argtypes = [vp, ci, vp, vp, vp, vp]
        L.s3_cindex_export.restype = ci
        L.s3_coactivate_score_compact_workspace.argtypes = [vp, i64]
        L.s3_coactivate_score_compact_workspace.restype = sz
        L.s3_coactivate_score_compact.argtypes = [vp, vp, vp, ci, i64, ci, ci, i32, ci, vp, vp, vp, vp, vp, sz, vp]
        L.s3_coactivate_score_compact.restype = ci
        L.s3_sae_train_workspace.argtypes = [ci, ci, ci, ci]
        L.s3_sae_train_workspace.restype = sz
        cf = C.c_float
        L.s3_sae_train_step.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, cf, cf, cf, cf, ci, vp, vp, vp, vp, sz, vp]
        L.s3_sae_train_step.restype = ci
        for name in ("s3_sae_encode_topk", "s3_sae_encode_topk_stream", "s3_index_create", "s3_index_append", "s3_index_finalize",
                     "s3_index_csr", "s3_index_build", "s3_coactivate_score"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise S3Error(rc, lib().s3_last_error().decode())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return S3_BF16
    if t.dtype == torch.float32:
        return S3_FP32
    raise TypeError(f"x must be bfloat16 or float32, got {t.dtype}")


def sae_encode_topk(x, w_enc, b_enc, k: int, ids=None, vals=None):
    """x [n_heads, T, d_head], w_enc [n_heads, n_feat, d_head] (same dtype), b_enc [n_heads, n_feat] fp32,
    all on the GPU and contiguous.  Returns (ids int32 [n_heads, T, k], vals fp32 [n_heads, T, k])."""
    import torch
    assert x.is_cuda and x.is_contiguous() and w_enc.is_contiguous() and b_enc.is_contiguous()
    assert x.dim() == 3 and w_enc.dim() == 3 and b_enc.dim() == 2
    n_heads, T, d = x.shape
    n_feat = w_enc.shape[1]
    assert w_enc.shape == (n_heads, n_feat, d) and b_enc.shape == (n_heads, n_feat)
    assert w_enc.dtype == x.dtype and b_enc.dtype == torch.float32
    if ids is None:
        ids = torch.empty((n_heads, T, k), dtype=torch.int32, device=x.device)
    if vals is None:
        vals = torch.empty((n_heads, T, k), dtype=torch.float32, device=x.device)
    assert ids.is_contiguous() and vals.is_contiguous() and ids.dtype == torch.int32 and vals.dtype == torch.float32
    assert ids.numel() == n_heads * T * k and vals.numel() == n_heads * T * k
    _check(lib().s3_sae_encode_topk(_ptr(x), _dtype_code(x), T, d, _ptr(w_enc), _ptr(b_enc), n_feat, k, n_heads,
                                    _ptr(ids), _ptr(vals), _stream()))
    return ids, vals


def new_tau_hint(n_heads: int, device="cuda"):
    """Carried thresholds of a stream before its first chunk: [n_heads, 2] fp32 filled with -inf."""
    import torch
    return torch.full((n_heads, 2), float("-inf"), dtype=torch.float32, device=device)


def sae_encode_topk_stream_workspace(n_heads: int, T: int) -> int:
    return int(lib().s3_sae_encode_topk_stream_workspace(n_heads, T))


def sae_encode_topk_stream(x, w_enc, b_enc, k: int, tau_hint, ws=None, ids=None, vals=None):
    """sae_encode_topk for the chunks of one stream: tau_hint [n_heads, 2] fp32 (new_tau_hint) is read and updated;
    the results are the same as sae_encode_topk's whatever it holds."""
    import torch
    assert x.is_cuda and x.is_contiguous() and w_enc.is_contiguous() and b_enc.is_contiguous()
    assert x.dim() == 3 and w_enc.dim() == 3 and b_enc.dim() == 2
    n_heads, T, d = x.shape
    n_feat = w_enc.shape[1]
    assert w_enc.shape == (n_heads, n_feat, d) and b_enc.shape == (n_heads, n_feat)
    assert w_enc.dtype == x.dtype and b_enc.dtype == torch.float32
    assert tau_hint.is_cuda and tau_hint.is_contiguous() and tau_hint.dtype == torch.float32
    assert tau_hint.numel() == 2 * n_heads
    need = sae_encode_topk_stream_workspace(n_heads, T)
    if ws is None:
        ws = torch.empty(max(need, 1), dtype=torch.uint8, device=x.device)
    assert ws.numel() >= need
    if ids is None:
        ids = torch.empty((n_heads, T, k), dtype=torch.int32, device=x.device)
    if vals is None:
        vals = torch.empty((n_heads, T, k), dtype=torch.float32, device=x.device)
    assert ids.is_contiguous() and vals.is_contiguous() and ids.dtype == torch.int32 and vals.dtype == torch.float32
    assert ids.numel() == n_heads * T * k and vals.numel() == n_heads * T * k
    _check(lib().s3_sae_encode_topk_stream(_ptr(x), _dtype_code(x), T, d, _ptr(w_enc), _ptr(b_enc), n_feat, k, n_heads,
                                           _ptr(ids), _ptr(vals), _ptr(tau_hint), _ptr(ws), ws.numel(), _stream()))
    return ids, vals


class Index:
    """n_heads inverted indexes (feature -> positions) living on the GPU (s3_index_* calls)."""

    def __init__(self, n_heads: int, n_feat: int, k: int, max_tokens: int):
        h = C.c_void_p()
        _check(lib().s3_index_create(n_heads, n_feat, k, max_tokens, C.byref(h)))
        self._h = h
        self.n_heads, self.n_feat, self.k, self.max_tokens = n_heads, n_feat, k, max_tokens

    def append(self, ids, positions=None, base_pos: int = 0):
        import torch
        assert ids.is_cuda and ids.is_contiguous() and ids.dtype == torch.int32 and ids.dim() == 3
        assert ids.shape[0] == self.n_heads and ids.shape[2] == self.k
        if positions is not None:
            assert positions.is_cuda and positions.dtype == torch.int32 and positions.numel() == ids.shape[1]
        _check(lib().s3_index_append(self._h, _ptr(ids), ids.shape[1], _ptr(positions), base_pos, _stream()))

    def finalize(self):
        _check(lib().s3_index_finalize(self._h, _stream()))

    def reset(self):
        _check(lib().s3_index_reset(self._h))

    @property
    def tokens(self) -> int:
        return int(lib().s3_index_tokens(self._h))

    def csr(self, head: int):
        """Copies of one head's (offsets [n_feat + 1], positions [P]) as torch int32 tensors."""
        import torch
        off, pos, n = C.c_void_p(), C.c_void_p(), C.c_int64()
        _check(lib().s3_index_csr(self._h, head, C.byref(off), C.byref(pos), C.byref(n)))
        o = torch.empty(self.n_feat + 1, dtype=torch.int32, device="cuda")
        p = torch.empty(n.value, dtype=torch.int32, device="cuda")
        _check(lib().s3_index_export(self._h, head, _ptr(o), _ptr(p) if n.value else None, _stream()))
        return o, p

    def csr_offsets(self, head: int):
        """Copy of one head's offsets [n_feat + 1] only."""
        import torch
        o = torch.empty(self.n_feat + 1, dtype=torch.int32, device="cuda")
        _check(lib().s3_index_export(self._h, head, _ptr(o), None, _stream()))
        return o

    def score_workspace(self, n_positions: int) -> int:
        return int(lib().s3_coactivate_score_workspace(self._h, n_positions))

    def coactivate_score(self, qids, qvals, n_positions: int, span_len: int, top_b: int, max_freq: int = 0,
                         nms: bool = True, want_scores: bool = False, ws=None):
        """Returns (span_start int32 [top_b], span_score fp32 [top_b], n_found int32 [1], scores fp32 [L] | None)."""
        import torch
        assert qids.is_cuda and qids.is_contiguous() and qvals.is_contiguous()
        assert qids.dtype == torch.int32 and qvals.dtype == torch.float32 and qids.dim() == 3
        assert qids.shape[0] == self.n_heads and qids.shape[2] == self.k and qvals.shape == qids.shape
        dev = qids.device
        need = self.score_workspace(n_positions)
        if ws is None:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        assert ws.numel() >= need
        starts = torch.empty(top_b, dtype=torch.int32, device=dev)
        scores = torch.empty(top_b, dtype=torch.float32, device=dev)
        found = torch.empty(1, dtype=torch.int32, device=dev)
        S = torch.empty(n_positions, dtype=torch.float32, device=dev) if want_scores else None
        _check(lib().s3_coactivate_score(self._h, _ptr(qids), _ptr(qvals), qids.shape[1], n_positions, span_len,
                                         top_b, max_freq, int(bool(nms)), _ptr(S), _ptr(starts), _ptr(scores),
                                         _ptr(found), _ptr(ws), ws.numel(), _stream()))
        return starts, scores, found, S

    def compact(self, prune_freq: int = 0):
        """s3_index_compact: the compact form of this (finalized) index in a buffer of its own."""
        return CompactIndex(self, prune_freq)

    def destroy(self):
        if getattr(self, "_h", None) and lib is not None:    # module globals are gone at interpreter shutdown
            lib().s3_index_destroy(self._h)
            self._h = None

    def __del__(self):
        self.destroy()


class CompactIndex:
    """Compact form of a finalized Index (s3_index_compact): 16-bit block-relative postings in block-major order, a
    segment table, optional stop-feature pruning.  Owns its buffer; independent of the Index it was built from."""

    def __init__(self, index: "Index", prune_freq: int = 0):
        import torch
        need = int(lib().s3_index_compact_bytes(index._h))
        self.buf = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        _check(lib().s3_index_compact(index._h, prune_freq, _ptr(self.buf), self.buf.numel(), C.byref(h), _stream()))
        self._h = h
        self.n_heads, self.n_feat, self.k = index.n_heads, index.n_feat, index.k
        nb, mp = C.c_int(), C.c_int64()
        _check(lib().s3_cindex_info(self._h, C.byref(nb), C.byref(mp)))
        self.n_blocks, self.max_postings = nb.value, mp.value
        self.nbytes = need

    def arrays(self, head: int):
        """Copies of one head's (cstart int32 [n_blocks * n_feat + 1], delta int16-view-of-uint16 [kept], cfreq [n_feat])."""
        import torch
        cs = torch.empty(self.n_blocks * self.n_feat + 1, dtype=torch.int32, device="cuda")
        de = torch.empty(max(self.max_postings, 1), dtype=torch.int16, device="cuda")
        cf = torch.empty(self.n_feat, dtype=torch.int32, device="cuda")
        _check(lib().s3_cindex_export(self._h, head, _ptr(cs), _ptr(de), _ptr(cf), _stream()))
        torch.cuda.synchronize()
        return cs, de[: int(cs[-1].item())], cf

    def score_workspace(self, n_positions: int) -> int:
        return int(lib().s3_coactivate_score_compact_workspace(self._h, n_positions))

    def coactivate_score(self, qids, qvals, n_positions: int, span_len: int, top_b: int, max_freq: int = 0,
                         nms: bool = True, want_scores: bool = False, ws=None):
        """As Index.coactivate_score, reading the compact index."""
        import torch
        assert qids.is_cuda and qids.is_contiguous() and qvals.is_contiguous()
        assert qids.dtype == torch.int32 and qvals.dtype == torch.float32 and qids.dim() == 3
        assert qids.shape[0] == self.n_heads and qids.shape[2] == self.k and qvals.shape == qids.shape
        dev = qids.device
        need = self.score_workspace(n_positions)
        if ws is None:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        assert ws.numel() >= need
        starts = torch.empty(top_b, dtype=torch.int32, device=dev)
        scores = torch.empty(top_b, dtype=torch.float32, device=dev)
        found = torch.empty(1, dtype=torch.int32, device=dev)
        S = torch.empty(n_positions, dtype=torch.float32, device=dev) if want_scores else None
        _check(lib().s3_coactivate_score_compact(self._h, _ptr(qids), _ptr(qvals), qids.shape[1], n_positions, span_len,
                                                 top_b, max_freq, int(bool(nms)), _ptr(S), _ptr(starts), _ptr(scores),
                                                 _ptr(found), _ptr(ws), ws.numel(), _stream()))
        return starts, scores, found, S

    def destroy(self):
        if getattr(self, "_h", None) and lib is not None:
            lib().s3_cindex_destroy(self._h)
            self._h = None

    def __del__(self):
        self.destroy()


def index_build(ids, n_feat: int, positions=None):
    """One-shot CSR of a single index: ids [T, k] int32 -> (offsets [n_feat + 1], positions [T * k])."""
    import torch
    assert ids.is_cuda and ids.is_contiguous() and ids.dtype == torch.int32 and ids.dim() == 2
    T, k = ids.shape
    need = int(lib().s3_index_build_workspace(T, k, n_feat))
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device=ids.device)
    off = torch.empty(n_feat + 1, dtype=torch.int32, device=ids.device)
    pos = torch.empty(T * k, dtype=torch.int32, device=ids.device)
    _check(lib().s3_index_build(_ptr(ids), _ptr(positions), T, k, n_feat, _ptr(off), _ptr(pos), _ptr(ws),
                                ws.numel(), _stream()))
    return off, pos


STATIC_SCRATCH_BYTES = 16 << 20


def index_build_static(ids, n_feat: int, off, pos, positions=None):
    """s3_index_build_static: one-shot CSR into the caller's off [n_feat + 1] / pos [T * k]; allocates nothing."""
    import torch
    assert ids.is_cuda and ids.is_contiguous() and ids.dtype == torch.int32 and ids.dim() == 2
    T, k = ids.shape
    assert off.is_cuda and off.dtype == torch.int32 and off.numel() >= n_feat + 1 and off.is_contiguous()
    assert pos.is_cuda and pos.dtype == torch.int32 and pos.numel() >= T * k and pos.is_contiguous()
    _check(lib().s3_index_build_static(_ptr(ids), _ptr(positions), T, k, n_feat, _ptr(off), _ptr(pos), _stream()))
    return off, pos


KERNEL_BOX, KERNEL_TRIANGULAR, KERNEL_GAUSSIAN = 0, 1, 2


def smoothing_kernel(kind: int, K: int):
    """Weights of a smoothing kernel (s3_smoothing_kernel, computed by the library on the host) as a float32 GPU tensor."""
    import torch
    host = (C.c_float * K)()
    _check(lib().s3_smoothing_kernel(kind, K, host))
    return torch.tensor(list(host), dtype=torch.float32).cuda()


def select_spans(scores, kernel, n_centers: int, nms_radius: int, rel_threshold: float, max_half_len: int,
                 want_density: bool = False):
    """s3_select_spans: scores [L] fp32, kernel [K] fp32 (GPU).  Returns (center, center_density, span_lo, span_hi,
    n_found, density | None)."""
    import torch
    assert scores.is_cuda and scores.is_contiguous() and scores.dtype == torch.float32 and scores.dim() == 1
    assert kernel.is_cuda and kernel.is_contiguous() and kernel.dtype == torch.float32 and kernel.dim() == 1
    L, dev = scores.numel(), scores.device
    ws = torch.empty(max(int(lib().s3_select_spans_workspace(L)), 1), dtype=torch.uint8, device=dev)
    center = torch.empty(n_centers, dtype=torch.int32, device=dev)
    dens_c = torch.empty(n_centers, dtype=torch.float32, device=dev)
    lo = torch.empty(n_centers, dtype=torch.int32, device=dev)
    hi = torch.empty(n_centers, dtype=torch.int32, device=dev)
    found = torch.empty(1, dtype=torch.int32, device=dev)
    D = torch.empty(L, dtype=torch.float32, device=dev) if want_density else None
    _check(lib().s3_select_spans(_ptr(scores), L, _ptr(kernel), kernel.numel(), n_centers, nms_radius, rel_threshold,
                                 max_half_len, _ptr(D), _ptr(center), _ptr(dens_c), _ptr(lo), _ptr(hi), _ptr(found),
                                 _ptr(ws), ws.numel(), _stream()))
    return center, dens_c, lo, hi, found, D


def fuse_indices(n_positions: int, span_lo, span_hi, n_spans, extra=None, lead: int = 0, tail: int = 0):
    """s3_fuse_indices: returns (mask uint8 [L], idx int32 [L], n_out int32 [1]); n_spans is a GPU int32 [1] or None."""
    import torch
    dev = span_lo.device
    ws = torch.empty(max(int(lib().s3_fuse_indices_workspace(n_positions)), 1), dtype=torch.uint8, device=dev)
    mask = torch.empty(n_positions, dtype=torch.uint8, device=dev)
    idx = torch.empty(n_positions, dtype=torch.int32, device=dev)
    n_out = torch.empty(1, dtype=torch.int32, device=dev)
    assert span_lo.dtype == torch.int32 and span_hi.dtype == torch.int32 and span_lo.numel() == span_hi.numel()
    if extra is not None:
        assert extra.is_cuda and extra.dtype == torch.int32 and extra.is_contiguous()
    _check(lib().s3_fuse_indices(n_positions, _ptr(span_lo), _ptr(span_hi), _ptr(n_spans), span_lo.numel(), _ptr(extra),
                                 0 if extra is None else extra.numel(), lead, tail, _ptr(mask), _ptr(idx), _ptr(n_out),
                                 _ptr(ws), ws.numel(), _stream()))
    return mask, idx, n_out


class SaeTrainer:
    """Parameters, Adam moments and workspace of one Top-K SAE on the GPU; step(x) is one s3_sae_train_step.
    w_enc, w_dec [n_feat, d] / b_enc [n_feat] / b_dec [d]: float32 GPU tensors, updated in place."""

    def __init__(self, w_enc, b_enc, w_dec, b_dec, k: int, batch: int, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
        import torch
        for t in (w_enc, b_enc, w_dec, b_dec):
            assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32
        self.n_feat, self.d = w_enc.shape
        assert w_dec.shape == w_enc.shape and b_enc.shape == (self.n_feat,) and b_dec.shape == (self.d,)
        self.w_enc, self.b_enc, self.w_dec, self.b_dec = w_enc, b_enc, w_dec, b_dec
        self.k, self.batch, self.hyper, self.steps = k, batch, (lr, beta1, beta2, eps), 0
        self.P = 2 * self.n_feat * self.d + self.n_feat + self.d
        self.m = torch.zeros(self.P, dtype=torch.float32, device=w_enc.device)
        self.v = torch.zeros_like(self.m)
        need = int(lib().s3_sae_train_workspace(batch, self.d, self.n_feat, k))
        if need == 0:
            raise S3Error(1, f"s3_sae_train_workspace: shape not supported (batch {batch}, d {self.d}, n_feat {self.n_feat}, k {k})")
        self.ws = torch.empty(need, dtype=torch.uint8, device=w_enc.device)
        self.loss = torch.empty(1, dtype=torch.float32, device=w_enc.device)

    def step(self, x, want_ids=False, want_grads=False):
        """x [batch, d] float32 on the GPU.  Returns (loss tensor [1], ids or None, grads [P] or None)."""
        import torch
        assert x.is_cuda and x.is_contiguous() and x.dtype == torch.float32 and x.shape == (self.batch, self.d)
        ids = torch.empty((self.batch, self.k), dtype=torch.int32, device=x.device) if want_ids else None
        grads = torch.empty(self.P, dtype=torch.float32, device=x.device) if want_grads else None
        self.steps += 1
        lr, b1, b2, eps = self.hyper
        _check(lib().s3_sae_train_step(_ptr(x), self.batch, self.d, self.n_feat, self.k, _ptr(self.w_enc), _ptr(self.b_enc),
                                       _ptr(self.w_dec), _ptr(self.b_dec), _ptr(self.m), _ptr(self.v), lr, b1, b2, eps,
                                       self.steps, _ptr(self.loss), _ptr(ids), _ptr(grads), _ptr(self.ws), self.ws.numel(),
                                       _stream()))
        return self.loss, ids, grads
