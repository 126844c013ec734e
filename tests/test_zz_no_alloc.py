"""s3_index_build_static (the entry point that allocates nothing: its workspace is a buffer built into the library)
against s3_index_build, through the C ABI: two calls in a row, the second with a smaller input, then the size limit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _ids(rng, T, k, n_feat):
    start = rng.integers(0, n_feat, (T, 1), dtype=np.int64)
    stride = rng.integers(0, n_feat // 2, (T, 1), dtype=np.int64) * 2 + 1
    return ((start + stride * np.arange(k, dtype=np.int64)) % n_feat).astype(np.int32)      # distinct per row


def test_static_scratch_build_equals_workspace_build_twice_in_a_row():
    import torch
    import paper_2601_17702_amd as s3
    rng = np.random.default_rng(42)
    n_feat = 16384
    off = torch.empty(n_feat + 1, dtype=torch.int32, device="cuda")
    pos = torch.empty(20000 * 32, dtype=torch.int32, device="cuda")
    for T, k, explicit in [(20000, 32, False), (777, 32, True), (0, 32, False), (4096, 8, False)]:
        ids = torch.from_numpy(_ids(rng, T, k, n_feat)).cuda() if T else torch.zeros((0, k), dtype=torch.int32, device="cuda")
        positions = torch.from_numpy(rng.permutation(100000)[:T].astype(np.int32)).cuda() if explicit else None
        off.fill_(-7)
        pos.fill_(-7)
        s3.index_build_static(ids, n_feat, off, pos, positions)
        want_off, want_pos = s3.index_build(ids, n_feat, positions)
        torch.cuda.synchronize()
        assert torch.equal(off, want_off), (T, k)
        assert torch.equal(pos[:T * k], want_pos), (T, k)
        assert int(off[-1]) == T * k
    # beyond the built-in buffer: a clear error, nothing launched
    big = torch.zeros((200000, 32), dtype=torch.int32, device="cuda")
    with pytest.raises(s3.S3Error) as e:
        s3.index_build_static(big, n_feat, off, torch.empty(200000 * 32, dtype=torch.int32, device="cuda"))
    assert e.value.code == -3 and "scratch" in str(e.value)
