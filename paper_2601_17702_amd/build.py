"""Build libs3attn.so (hand-written HIP for gfx950 behind the C ABI of include/s3attn.h)."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libs3attn.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result"]


def build(verbose: bool = False, tuning_lib: str | None = None) -> str:
    """Compile every csrc/*.hip and link libs3attn.so.  tuning_lib: path of a second library to build instead, with
    -DS3_TUNING (environment knobs, kernels with parts compiled out, cycle counters: measurement tooling only)."""
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    objs = []
    procs = []
    extra = ["-DS3_TUNING"] if tuning_lib else []
    for s in srcs:
        o = s[:-4] + (".tuning.o" if tuning_lib else ".o")
        objs.append(o)
        procs.append((s, subprocess.Popen(["hipcc", *FLAGS, *extra, "-c", s, "-o", o], stderr=subprocess.PIPE, text=True)))
    for s, p in procs:
        _, err = p.communicate()
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {s}:\n{err}")
        if verbose and err.strip():
            print(err)
    check_fast_encoder_asm(extra)
    out = tuning_lib or LIB
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs])
    return out


def check_fast_encoder_asm(extra=()) -> None:
    """Compile the fast encoder to assembly once more and scan it (asm_check): its inline-assembly MFMA chains rely on
    distances that the compiler does not know about, so a build whose generated code breaks them is rejected."""
    import tempfile
    from . import asm_check
    src = os.path.join(CSRC, "encode_topk_fast.hip")
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "encode_topk_fast.s")
        p = subprocess.run(["hipcc", *FLAGS, *extra, "-S", "--cuda-device-only", src, "-o", asm], stderr=subprocess.PIPE, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src}:\n{p.stderr}")
        res = asm_check.scan_file(asm, "sae_encode_topk_")
    if len(res) < 6:
        raise RuntimeError(f"asm check: expected the six fast-encoder kernels, found {sorted(res)}")
    bad = {k: v for k, v in res.items() if v}
    if bad:
        lines = [f"{k}: {len(v)} finding(s), first: {v[0]}" for k, v in bad.items()]
        raise RuntimeError("asm check of the fast encoder failed:\n" + "\n".join(lines))


if __name__ == "__main__":
    print(build(verbose=True))
