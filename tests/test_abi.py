"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments on the host before anything touches a GPU."""
import ctypes as C
import os
import re

import paper_2601_17702_amd as s3

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "s3attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(s3_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert "s3_sae_encode_topk" in names and "s3_index_finalize" in names and "s3_coactivate_score" in names
    lib = C.CDLL(s3.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/s3attn.h but not exported"


def test_library_exports_nothing_but_the_declared_symbols():
    """Every dynamic symbol the library defines with the s3 prefix (in any case, mangled or not) is declared in the
    header: no tuning hook, no internal helper leaks out."""
    import subprocess
    out = subprocess.check_output(["nm", "-D", "--defined-only", s3.LIB_PATH], text=True)
    exported = sorted(line.split()[-1] for line in out.splitlines() if "s3_" in line.lower())
    assert exported == declared_symbols()


def test_no_environment_reads_in_the_product_sources():
    """Tuning knobs exist only under -DS3_TUNING: outside such blocks no source reads the environment."""
    import glob
    for path in glob.glob(os.path.join(ROOT, "paper_2601_17702_amd", "csrc", "*")):
        if not path.endswith((".hip", ".h", ".inc")):
            continue
        depth, tuning = [], 0
        for line in open(path):
            t = line.strip()
            if t.startswith("#if"):
                depth.append("S3_TUNING" in t)
                tuning += depth[-1]
            elif t.startswith("#endif") and depth:
                tuning -= depth.pop()
            elif not tuning:
                assert "getenv" not in t and "env_int" not in t, f"{path}: {t}"


def test_host_side_argument_validation():
    L = s3.lib()
    one = C.c_void_p(256)           # non-null, never dereferenced: validation fails first
    bad = [
        L.s3_sae_encode_topk(None, 0, 8, 128, one, one, 64, 4, 1, one, one, None),        # null x
        L.s3_sae_encode_topk(one, 2, 8, 128, one, one, 64, 4, 1, one, one, None),         # dtype
        L.s3_sae_encode_topk(one, 0, 8, 96, one, one, 64, 4, 1, one, one, None),          # d_head
        L.s3_sae_encode_topk(one, 0, 8, 128, one, one, 256, 129, 1, one, one, None),      # k > S3_MAX_K
        L.s3_sae_encode_topk(one, 0, 8, 128, one, one, 16, 32, 1, one, one, None),        # k > n_feat
        L.s3_sae_encode_topk(one, 0, 8, 128, one, one, 70000, 4, 1, one, one, None),      # n_feat
        L.s3_sae_encode_topk(one, 0, -1, 128, one, one, 64, 4, 1, one, one, None),        # T
        L.s3_sae_encode_topk(C.c_void_p(264), 0, 8, 128, one, one, 64, 4, 1, one, one, None),   # alignment
    ]
    assert all(rc == -1 for rc in bad)
    assert b"s3_sae_encode_topk" in L.s3_last_error()
    h = C.c_void_p()
    assert L.s3_index_create(0, 64, 4, 10, C.byref(h)) == -1
    assert L.s3_index_create(1, 256, 129, 10, C.byref(h)) == -1
    assert L.s3_index_create(1, 64, 4, 1 << 25, C.byref(h)) == -1
    assert L.s3_index_append(None, one, 1, None, 0, None) == -1
    assert L.s3_index_finalize(None, None) == -1
    assert L.s3_index_build(one, None, 8, 4, 64, one, one, one, 16, None) == -3          # workspace too small
    assert L.s3_index_build_workspace(8, 4, 64) > 0 and L.s3_index_build_workspace(8, 129, 256) == 0
    assert L.s3_coactivate_score(None, one, one, 1, 10, 4, 2, 0, 1, None, one, one, one, one, 1 << 20, None) == -1
    need = L.s3_sae_encode_topk_stream_workspace(2, 512)
    assert need >= 2 * 512 * 4 and L.s3_sae_encode_topk_stream_workspace(0, 512) == 0
    args = (one, 0, 512, 128, one, one, 2048, 32, 2, one, one)
    assert L.s3_sae_encode_topk_stream(*args, None, one, need, None) == -1                 # null tau_hint
    assert L.s3_sae_encode_topk_stream(*args, one, None, need, None) == -1                 # null workspace
    assert L.s3_sae_encode_topk_stream(*args, one, C.c_void_p(264), need, None) == -1      # workspace alignment
    assert L.s3_sae_encode_topk_stream(*args, one, one, need - 1, None) == -3              # workspace too small
    assert b"s3_sae_encode_topk_stream" in L.s3_last_error()
    # training step: shapes, hyper-parameters, pointers and the workspace are checked before anything is launched
    need = L.s3_sae_train_workspace(256, 128, 1024, 16)
    assert need > 0 and L.s3_sae_train_workspace(256, 64, 1024, 16) == 0 and L.s3_sae_train_workspace(256, 128, 1000, 16) == 0
    assert L.s3_sae_train_workspace(1 << 20, 128, 1024, 128) == 0                            # B * k > 2^24
    hyp = (1e-3, 0.9, 0.999, 1e-8)
    ptrs = (one,) * 6

    def train(B=256, d=128, nf=1024, k=16, hyp=hyp, step=1, x=one, ws=one, ws_bytes=need):
        return L.s3_sae_train_step(x, B, d, nf, k, *ptrs, *hyp, step, one, None, None, ws, ws_bytes, None)
    assert train(d=64) == -1 and train(k=129) == -1 and train(nf=1000) == -1 and train(x=None) == -1
    assert train(step=0) == -1 and train(hyp=(1e-3, 1.0, 0.999, 1e-8)) == -1 and train(hyp=(1e-3, 0.9, 0.999, 0.0)) == -1
    assert train(ws=C.c_void_p(264)) == -1 and train(ws_bytes=need - 1) == -3
    assert b"s3_sae_train_step" in L.s3_last_error()
    assert s3.MAX_K == 128 and s3.MAX_FEAT == 65536
