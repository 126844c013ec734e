#!/usr/bin/env python3
"""Benchmark of the S3-Attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic context: for every chunk
sae_encode_topk -> index_append, then index_finalize, then the query encode and
coactivate_score (position scores, span pooling, Top-B).  Inputs are resident in HBM before the
timed region starts.  Prints ONE JSON line (see the design doc for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2601_17702_amd import synth  # noqa: E402

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp32": 157.3}   # MI355X dense matrix peaks
HBM_PEAK_GBS = 8000.0


def measured_traffic(workload: str):
    """HBM bytes per chunk call of the encoder from the committed counter summary of this workload, if there is one
    (profiles/encode_<workload>_hbm_traffic.txt, written from two rocprofv3 --pmc runs: counters cannot be read from
    inside this script).  The file carries a line `traffic_bytes_per_chunk_call = N`; None without the file."""
    path = os.path.join(ROOT, "profiles", f"encode_{workload}_hbm_traffic.txt")
    if os.path.exists(path):
        for line in open(path):
            if line.lstrip("# ").startswith("traffic_bytes_per_chunk_call"):
                return int(float(line.split("=")[1].split()[0])), os.path.relpath(path, ROOT)
    return None, None


def train_leg(torch, s3, steps):
    """One Adam step of the Top-K SAE at App. B.3's configuration (4096 tokens per batch, expansion 128 -> 16384
    latents, k = 128, d_head 128) on synthetic activations (a 24-dimensional Gaussian subspace plus noise; unit-norm
    Gaussian dictionary, decoder initialised next to the encoder): not part of a hot-path step, reported beside it."""
    Bt, nf, d, k = 4096, 16384, 128, 128
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    basis = torch.randn(24, d, generator=g, device="cuda") / 24 ** 0.5
    xs = [torch.randn(Bt, 24, generator=g, device="cuda") @ basis + 0.3 * torch.randn(Bt, d, generator=g, device="cuda")
          for _ in range(4)]
    w_enc = torch.randn(nf, d, generator=g, device="cuda")
    w_enc /= w_enc.norm(dim=1, keepdim=True)
    w_dec = w_enc + 0.05 * torch.randn(nf, d, generator=g, device="cuda")
    tr = s3.SaeTrainer(w_enc.contiguous(), torch.zeros(nf, device="cuda"), w_dec.contiguous(), torch.zeros(d, device="cuda"),
                       k=k, batch=Bt)
    for i in range(2):
        tr.step(xs[i])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    first = float(tr.loss.item())
    e0.record()
    for i in range(steps):
        tr.step(xs[i % 4])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return {"config": {"batch_tokens": Bt, "n_feat": nf, "k": k, "d_head": d, "optimizer": "adam"}, "steps": steps,
            "ms_per_step": ms, "tokens_per_s": Bt / (ms * 1e-3),
            "encoder_gemm_tflops": 2.0 * Bt * nf * d / (ms * 1e-3) / 1e12, "loss_first": first, "loss_last": float(tr.loss.item())}


def gen_inputs(w, torch, threads=16):
    """All chunks of all heads, W_enc, b_enc and the queries, generated on the host and moved to HBM."""
    from concurrent.futures import ThreadPoolExecutor
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    H, C = w.n_heads, w.n_chunks
    assert w.L % w.T == 0
    K = torch.empty((C, H, w.T, w.d_head), dtype=tdt, device="cuda")
    W = torch.empty((H, w.n_feat, w.d_head), dtype=tdt, device="cuda")
    B = torch.empty((H, w.n_feat), dtype=torch.float32, device="cuda")
    Q = torch.empty((H, w.nq, w.d_head), dtype=tdt, device="cuda")

    def as_t(a):
        t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
        return t.view(torch.bfloat16) if a.dtype == np.uint16 else t

    def one_head(h):
        return (h, [synth.gen_keys(w, h, c) for c in range(C)], synth.gen_w_enc(w, h), synth.gen_b_enc(w, h),
                synth.gen_queries(w, h))

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for h, ks, wh, bh, qh in ex.map(one_head, range(H)):
            for c in range(C):
                K[c, h].copy_(as_t(ks[c]))
            W[h].copy_(as_t(wh))
            B[h].copy_(torch.from_numpy(bh))
            Q[h].copy_(as_t(qh))
    torch.cuda.synchronize()
    return K, W, B, Q


def cpu_baseline(w, sample_tokens, sample_heads):
    """The oracle, as it stands, on a bounded sample of the same workload (host cores, OpenMP over rows)."""
    from oracle import s3_oracle as orc
    sw = synth.shrink(w, L=sample_tokens, T=min(w.T, sample_tokens))
    dt, S = 0.0, np.zeros(sample_tokens)
    for h in range(sample_heads):
        x = np.concatenate([synth.gen_keys(sw, h, c) for c in range(sw.n_chunks)])
        W, b, q = synth.gen_w_enc(sw, h), synth.gen_b_enc(sw, h), synth.gen_queries(sw, h)
        t0 = time.perf_counter()
        enc = orc.encode_topk(x, W, b, w.k, w.dtype)
        ix = orc.Index(w.n_feat)
        ix.append(enc["ids"], np.arange(x.shape[0], dtype=np.int32))
        ix.csr()
        qe = orc.encode_topk(q, W, b, w.k, w.dtype)
        ix.score_accumulate(qe["ids"], qe["vals"], S)
        dt += time.perf_counter() - t0
    t0 = time.perf_counter()
    orc.topb(orc.pool(S, w.span_len), w.span_len, w.top_b, nms=True)
    dt += time.perf_counter() - t0
    return {"value": sample_heads * sample_tokens / dt, "unit": "tokens\u00b7heads/s", "cores": orc.threads(),
            "kind": "oracle", "sample": f"{sample_heads} heads x {sample_tokens} tokens of {w.name} "
            f"(encode+Top-k+index+score), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_llama8b", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = min(L, 32768)")
    ap.add_argument("--cpu-sample-heads", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--train-steps", type=int, default=10,
                    help="SAE training steps timed beside the hot path (App. B.3's configuration; 0 = skip)")
    ap.add_argument("--train-only", action="store_true", help="time the SAE training steps alone (for profiles)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 256 MiB device copy (a kernel of known traffic, for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    import torch
    import paper_2601_17702_amd as s3
    s3.lib()                                   # fail loudly if the HIP library is not built
    if args.train_only:
        print(json.dumps({"sae_train_step": train_leg(torch, s3, max(args.train_steps, 1))}))
        return
    w = synth.WORKLOADS[args.workload]
    H = w.n_heads
    K, W, B, Q = gen_inputs(w, torch)
    ids = torch.empty((H, w.T, w.k), dtype=torch.int32, device="cuda")
    vals = torch.empty((H, w.T, w.k), dtype=torch.float32, device="cuda")
    qids = torch.empty((H, w.nq, w.k), dtype=torch.int32, device="cuda")
    qvals = torch.empty((H, w.nq, w.k), dtype=torch.float32, device="cuda")
    index = s3.Index(H, w.n_feat, w.k, w.L)
    ws = torch.empty(index.score_workspace(w.L), dtype=torch.uint8, device="cuda")
    enc_ws = torch.empty(max(s3.sae_encode_topk_stream_workspace(H, w.T), 1), dtype=torch.uint8, device="cuda")
    tau_hint = s3.new_tau_hint(H)
    # every event of the timed steps exists before the timed region starts; per step: 3 per chunk + 4
    nev = 3 * w.n_chunks + 4
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(nev)] for _ in range(args.steps)]

    def step(ev=None):
        """ev: this step's events (chunk c: 3c = before encode, 3c + 1 = after encode, 3c + 2 = after append; then
        before finalize, after finalize, after query encode, after scoring) or None for an untimed step."""
        index.reset()
        tau_hint.fill_(float("-inf"))            # a new stream: no threshold is carried into its first chunk
        for c in range(w.n_chunks):
            if ev:
                ev[3 * c].record()
            s3.sae_encode_topk_stream(K[c], W, B, w.k, tau_hint, enc_ws, ids, vals)
            if ev:
                ev[3 * c + 1].record()
            index.append(ids, base_pos=c * w.T)
            if ev:
                ev[3 * c + 2].record()
        if ev:
            ev[-4].record()
        index.finalize()
        if ev:
            ev[-3].record()
        s3.sae_encode_topk(Q, W, B, w.k, qids, qvals)
        if ev:
            ev[-2].record()
        out = index.coactivate_score(qids, qvals, w.L, w.span_len, w.top_b, max_freq=0, nms=True, ws=ws)
        if ev:
            ev[-1].record()
        return out

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        out = step(events[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # outside the timed steps: the compact form of the same index (16-bit block-relative postings) and scoring from it
    cev = [torch.cuda.Event(enable_timing=True) for _ in range(2 + 2 * args.steps)]
    cev[0].record()
    cindex = index.compact(0)
    cev[1].record()
    cws = torch.empty(cindex.score_workspace(w.L), dtype=torch.uint8, device="cuda")
    cindex.coactivate_score(qids, qvals, w.L, w.span_len, w.top_b, max_freq=0, nms=True, ws=cws)
    for i in range(args.steps):
        cev[2 + 2 * i].record()
        cout = cindex.coactivate_score(qids, qvals, w.L, w.span_len, w.top_b, max_freq=0, nms=True, ws=cws)
        cev[3 + 2 * i].record()
    torch.cuda.synchronize()
    compact_build_ms = cev[0].elapsed_time(cev[1])
    compact_score_ms = float(np.mean([cev[2 + 2 * i].elapsed_time(cev[3 + 2 * i]) for i in range(args.steps)]))
    assert torch.equal(cout[0], out[0]) and torch.equal(cout[2], out[2])      # same spans as from the plain index

    if args.calibrate_copy:          # reads 256 MiB, writes 256 MiB: scales the FETCH_SIZE / WRITE_SIZE counters
        src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    nc = w.n_chunks
    enc_ms = [e[3 * c].elapsed_time(e[3 * c + 1]) for e in events for c in range(nc)]
    app_ms = [e[3 * c + 1].elapsed_time(e[3 * c + 2]) for e in events for c in range(nc)]
    fin_ms = [e[-4].elapsed_time(e[-3]) for e in events]
    qenc_ms = [e[-3].elapsed_time(e[-2]) for e in events]
    score_ms = [e[-2].elapsed_time(e[-1]) for e in events]
    scan_ms = float(np.mean([e[0].elapsed_time(e[-3]) for e in events]))    # encode + Top-k + index of one context
    enc_avg = float(np.mean(enc_ms))
    flop_per_launch = 2.0 * w.d_head * w.n_feat * w.T * H       # encoder GEMM of one chunk, all heads
    achieved = flop_per_launch / (enc_avg * 1e-3) / 1e12
    peak = MFMA_PEAK_TFLOPS[w.dtype]
    ms_per_step = dt / args.steps * 1e3

    # algorithmic HBM bytes of the index build and of scoring (every byte that has to move once)
    idx_bytes = 2.0 * H * w.L * w.k * 4 + 4.0 * H * (w.n_feat + 1)   # ids in, postings and offsets out
    post_bytes = 0.0
    qh = qids.cpu().numpy()
    for h in range(H):
        off = index.csr(h)[0].cpu().numpy()
        f = np.unique(qh[h])
        post_bytes += 4.0 * float((off[f + 1] - off[f]).sum())   # posting lists named by this head's queries
    score_bytes = post_bytes + 2.0 * H * w.nq * w.k * 4 + 4.0 * w.L
    idx_ms = float(np.sum(app_ms)) / args.steps + float(np.mean(fin_ms))
    traffic, traffic_src = measured_traffic(w.name)
    fast = w.dtype == "bf16" and w.d_head == 128 and w.k <= 64 and w.n_feat % 128 == 0      # shapes the fast kernel takes
    enc_kernel = (("k32" if w.k <= 32 else "k64") + "::sae_encode_topk_fast_kernel<0>") if fast else "sae_encode_topk_kernel"

    def hbm(nbytes, ms):
        return {"bound": "hbm", "bytes": nbytes, "ms": ms, "achieved": nbytes / ms / 1e6, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": nbytes / ms / 1e6 / HBM_PEAK_GBS}

    res = {
        "metric": "scanned tokens\u00b7heads/sec (encode+TopK+index) at Llama-8B shape; % MFMA/HBM peak",
        # the metric's own stages: every chunk's encode + Top-k + append, then finalize (events inside the timed steps);
        # the query encode and the scoring that complete a step are timed and reported separately below
        "value": w.token_heads / (scan_ms * 1e-3),
        "unit": "tokens\u00b7heads/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": w.layers, "kv_heads": w.kv_heads, "tokens": w.L, "chunk": w.T,
                   "d_head": w.d_head, "n_feat": w.n_feat, "k": w.k, "queries_per_kv_head": w.nq,
                   "span_len": w.span_len, "top_b": w.top_b},
        "scan_ms_per_step": scan_ms,
        "whole_path_tokens_heads_per_s": w.token_heads / (ms_per_step * 1e-3),
        "stages_ms": {"encode_topk": float(np.sum(enc_ms)) / args.steps, "index_append": float(np.sum(app_ms)) / args.steps,
                      "index_finalize": float(np.mean(fin_ms)), "query_encode": float(np.mean(qenc_ms)),
                      "coactivate_score": float(np.mean(score_ms))},
        "roofline": {"kernel": enc_kernel, "bound": "mfma", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic, "traffic_source": traffic_src,
                     "launch_ms": enc_avg, "flop_per_launch": flop_per_launch},
        "stage_rooflines": {
            "encode_topk": {"bound": "mfma", "flop": flop_per_launch * nc, "ms": float(np.sum(enc_ms)) / args.steps,
                            "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak},
            "index_build": hbm(idx_bytes, idx_ms),
            "coactivate_score": hbm(score_bytes, float(np.mean(score_ms))),
            # not part of a step: the same scoring from the compact index (half the posting bytes really move;
            # the fraction is still taken on the plain 4-byte postings so that the two lines compare)
            "coactivate_score_compact": hbm(score_bytes, compact_score_ms)},
        "compact_index": {"build_ms": compact_build_ms, "bytes": cindex.nbytes,
                          "plain_csr_bytes": H * (w.L * w.k + w.n_feat + 1) * 4},
        "spans_found": int(out[2].item()),
    }
    if args.train_steps > 0:
        res["sae_train_step"] = train_leg(torch, s3, args.train_steps)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_tokens or min(w.L, 32768), args.cpu_sample_heads)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
