// Generation-time co-activation scoring (Sec. 3.5 scoring equation; App. D.2 / App. E weights;
// Sec. 3.5 "Adaptive Granularity" read as box pooling + fixed-length spans with NMS).
//
//   1. query weights   qw[h][f] = IDF_h(f) * sum of the query activations that name f
//   2. postings gather S[t] += qw[h][f] for every t in I_h[f], all heads into one S (per block of positions
//      in LDS; global atomics only for contexts longer than 64 blocks = 1 Mi positions)
//   3. span pooling    W[s] = S[s] + ... + S[s + len - 1]
//   4. Top-B           greedy best window, optional suppression of overlapping windows
//
// Every sum is carried in 64-bit fixed point (power-of-two scales derived on the device from the
// largest query activation / largest weight), so additions commute exactly: the result does not
// depend on the order in which wavefronts reach a position, run-to-run output is bit-identical,
// and a window's score is exactly the sum of its members.  Values are rounded to fp32 once, on
// output.
#include "s3_common.h"

#include <math.h>

namespace {

struct Scal {
    unsigned int qmax_bits;          // bits of the largest query activation (>= 0)
    unsigned int pad;
    unsigned long long qwmax_bits;   // bits (as double) of the largest query weight
};

// A posting list with a non-zero query weight: CSR bounds and the weight.
struct alignas(16) ActiveList {
    double w;
    int32_t b, e;
};

struct ScoreArgs {
    const int32_t* qids;
    const float* qvals;
    const int32_t* offsets;
    const int32_t* positions;
    int64_t off_stride, pos_stride;
    int n_heads, n_feat, k, nq;
    int64_t L, nW;
    int len, top_b, nms, hb;
    int32_t max_freq;
    Scal* sc;
    unsigned long long* qacc;        // [n_heads * n_feat] fixed-point sums, then doubles (query weights)
    ActiveList* act;                 // [n_heads * n_feat] lists with a non-zero weight, packed per head (LDS scatter)
    int* nact;                       // [n_heads] their number
    unsigned long long* sfix;        // [L]
    unsigned long long* part;        // [ngroup][L] partial sums of head groups (ngroup > 1)
    int pb, npb, heads_per, ngroup, sorted;   // position blocks / head groups of the LDS scatter
    long long* wfix;                 // [nW]
    unsigned char* dead;             // [nW]
    long long* tmaxv;                // [ntile]
    int* tmaxi;                      // [ntile]
    int ntile;
    float* scores_out;
    int32_t* span_start;
    float* span_score;
    int32_t* n_found;
};

constexpr int kTileW = 1024;

__device__ __forceinline__ int exp_q(const Scal* sc) {   // activations are scaled by 2^exp_q: < 2^40 each
    float q = __uint_as_float(sc->qmax_bits);
    if (!(q > 0.f)) return 0;
    int e;
    frexpf(q, &e);
    return 40 - e;
}

__device__ __forceinline__ int exp_s(const Scal* sc, int hb) {   // weights are scaled by 2^exp_s: sums < 2^62
    double w = __longlong_as_double((long long)sc->qwmax_bits);
    if (!(w > 0.0)) return 0;
    int e;
    frexp(w, &e);
    return 62 - hb - e;
}

__global__ void sc_zero_kernel(unsigned long long* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}

__global__ __launch_bounds__(256) void sc_qmax_kernel(ScoreArgs a) {
    const size_t n = (size_t)a.n_heads * a.nq * a.k;
    unsigned int m = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        m = max(m, __float_as_uint(fmaxf(a.qvals[i], 0.f)));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, (unsigned int)__shfl_xor((int)m, o));
    __shared__ unsigned int wmax[4];     // one atomic per block: they all hit the same word
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
        if (m) atomicMax(&a.sc->qmax_bits, m);
    }
}

__global__ __launch_bounds__(256) void sc_qacc_kernel(ScoreArgs a) {
    const size_t per_head = (size_t)a.nq * a.k, n = per_head * a.n_heads;
    const double scale = ldexp(1.0, exp_q(a.sc));
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        float v = fmaxf(a.qvals[i], 0.f);
        unsigned int f = (unsigned int)a.qids[i];
        if (v > 0.f && f < (unsigned int)a.n_feat) {
            size_t h = i / per_head;
            atomicAdd(&a.qacc[h * a.n_feat + f], (unsigned long long)llrint((double)v * scale));
        }
    }
}

// fixed-point sum -> query weight (double, stored in place); App. D.2 IDF with natural log.  For the LDS scatter the
// lists with a non-zero weight are also packed per head (in any order: the scores are exact integer sums).
// A block owns kQwPer * 256 consecutive (head, feature) entries: it packs its lists locally (prefix sum) and
// reserves their place in the head's array with one atomic, so a head's counter sees few updates.
constexpr int kQwPer = 16;

__global__ __launch_bounds__(256) void sc_qw_kernel(ScoreArgs a) {
    __shared__ int wsum[4];
    __shared__ int slot0;
    __shared__ unsigned long long wmax[4];
    const size_t n = (size_t)a.n_heads * a.n_feat;
    const size_t base = (size_t)blockIdx.x * (256 * kQwPer);
    const size_t end = base + 256 * kQwPer < n ? base + 256 * kQwPer : n;
    const double inv = ldexp(1.0, -exp_q(a.sc));
    const int tid = threadIdx.x;
    double w[kQwPer];
    int lb[kQwPer], le[kQwPer];
    double mx = 0.0;
#pragma unroll
    for (int j = 0; j < kQwPer; ++j) {
        const size_t i = base + (size_t)j * 256 + tid;
        w[j] = 0.0;
        lb[j] = le[j] = 0;
        if (i < n) {
            const unsigned long long s = a.qacc[i];
            if (s) {
                const size_t h = i / a.n_feat, f = i - h * a.n_feat;
                const int32_t* off = a.offsets + h * a.off_stride;
                lb[j] = off[f];
                le[j] = off[f + 1];
                const int freq = le[j] - lb[j];
                if (freq > 0 && !(a.max_freq > 0 && freq > a.max_freq))
                    w[j] = (double)s * inv / (log(1.0 + (double)freq) + 1.0);
            }
            a.qacc[i] = (unsigned long long)__double_as_longlong(w[j]);
            mx = fmax(mx, w[j]);
        }
    }
    if (a.npb) {
        const size_t h_last = (end - 1) / a.n_feat;
        for (size_t h = base / a.n_feat; h <= h_last; ++h) {      // the heads this block's entries belong to (mostly one)
            const size_t s0 = h * a.n_feat, s1 = s0 + a.n_feat;
            int c = 0;
#pragma unroll
            for (int j = 0; j < kQwPer; ++j) {
                const size_t i = base + (size_t)j * 256 + tid;
                c += (w[j] > 0.0 && i >= s0 && i < s1) ? 1 : 0;
            }
            int tot;
            const int ex = s3_block_excl_scan<256>(c, wsum, tot);
            if (tid == 0) slot0 = tot ? atomicAdd(&a.nact[h], tot) : 0;
            __syncthreads();
            int slot = slot0 + ex;
#pragma unroll
            for (int j = 0; j < kQwPer; ++j) {
                const size_t i = base + (size_t)j * 256 + tid;
                if (w[j] > 0.0 && i >= s0 && i < s1) a.act[s0 + slot++] = ActiveList{w[j], lb[j], le[j]};
            }
            __syncthreads();
        }
    }
    unsigned long long mb = (unsigned long long)__double_as_longlong(mx);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned int lo = (unsigned int)__shfl_xor((int)(unsigned int)mb, o);
        unsigned int hi = (unsigned int)__shfl_xor((int)(unsigned int)(mb >> 32), o);
        unsigned long long other = ((unsigned long long)hi << 32) | lo;
        mb = other > mb ? other : mb;
    }
    if ((tid & 63) == 0) wmax[tid >> 6] = mb;       // one atomic per block: they all hit the same word
    __syncthreads();
    if (tid == 0) {
        for (int q = 1; q < 4; ++q) mb = wmax[q] > mb ? wmax[q] : mb;
        if (mb) atomicMax(&a.sc->qwmax_bits, mb);
    }
}

// one wavefront per posting list with a non-zero weight
__global__ __launch_bounds__(256) void sc_scatter_kernel(ScoreArgs a) {
    const size_t wid = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= (size_t)a.n_heads * a.n_feat) return;
    const double w = __longlong_as_double((long long)a.qacc[wid]);
    if (!(w > 0.0)) return;
    const unsigned long long wf = (unsigned long long)llrint(w * ldexp(1.0, exp_s(a.sc, a.hb)));
    if (!wf) return;
    const size_t h = wid / a.n_feat, f = wid - h * a.n_feat;
    const int32_t* off = a.offsets + h * a.off_stride;
    const int32_t* pos = a.positions + h * a.pos_stride;
    const int b = off[f], e = off[f + 1];
    for (int i = b + (threadIdx.x & 63); i < e; i += 64) {
        unsigned int p = (unsigned int)pos[i];
        if (p < (unsigned long long)a.L) atomicAdd(&a.sfix[p], wf);
    }
}

// Postings gather with the scores of one block of positions held in LDS.
// Workgroup (b, g) owns positions [b * pb, (b + 1) * pb) and the heads of group g: it walks every posting list
// of those heads that has a non-zero weight and adds the postings that fall into its block with LDS atomics
// (64-bit fixed point, so the order of the additions does not matter), then stores the block: into S when there
// is one head group, else into that group's partial array (summed by sc_reduce_kernel).  No global atomics.
// The lists with a non-zero weight were packed per head by sc_qw_kernel.  A wavefront takes 64 of them at a time:
// lane l fetches weight and bounds of list l, then the lists are walked kWalk at a time (lanes over postings) so
// that kWalk independent loads are in flight.
// Lists are sorted by position when the index was fed increasing implicit positions; long lists are then
// narrowed to the block by a per-lane search first (lower_bound_pos).
constexpr int kScatterThreads = 1024;
constexpr int kWalk = 8;             // posting loads a wavefront keeps in flight
constexpr int kNarrowMin = 128;      // sorted lists longer than this are narrowed to the position block first
constexpr int kWalkRounds = 4;       // rounds in which kWalk lists advance together before the long rest is walked alone
constexpr int kMaxPB = 16384;
constexpr int kMaxBlocks = 64;       // longer contexts (> 1 Mi positions) use the global-atomic scatter

// First index in [b, e) whose position is >= key (e if none); pos[b .. e) ascending.  Eight-way search: the seven
// pivots of a step are independent loads, so a list of n postings costs about log8(n) memory latencies.
__device__ __forceinline__ int lower_bound_pos(const int32_t* pos, int b, int e, int64_t key) {
    while (e - b > 8) {
        const int step = (e - b) >> 3;
        int32_t v[7];
#pragma unroll
        for (int u = 0; u < 7; ++u) v[u] = pos[b + (u + 1) * step];
        int c = 0;
#pragma unroll
        for (int u = 0; u < 7; ++u) c += (int64_t)v[u] < key ? 1 : 0;
        const int nb = c ? b + c * step + 1 : b;          // everything up to the last pivot below the key is below it
        if (c < 7) e = b + (c + 1) * step;                // the first pivot at or above the key bounds the answer
        b = nb;
    }
    int32_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = b + u < e ? pos[b + u] : 0;
    int c = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) c += (b + u < e && (int64_t)v[u] < key) ? 1 : 0;
    return b + c;
}

__global__ __launch_bounds__(kScatterThreads) void sc_scatter_lds_kernel(ScoreArgs a) {
    extern __shared__ unsigned long long sblk[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t p0 = (int64_t)blockIdx.x * a.pb;
    const int64_t p1 = p0 + a.pb < a.L ? p0 + a.pb : a.L;
    const unsigned span = (unsigned)(p1 - p0);
    for (int i = tid; i < a.pb; i += kScatterThreads) sblk[i] = 0ull;
    __syncthreads();
    const double scale = ldexp(1.0, exp_s(a.sc, a.hb));
    const int h0 = blockIdx.y * a.heads_per, h1 = min(a.n_heads, h0 + a.heads_per);
    for (int h = h0; h < h1; ++h) {
        const int32_t* pos = a.positions + (size_t)h * a.pos_stride;
        const ActiveList* act = a.act + (size_t)h * a.n_feat;
        const int n_act = a.nact[h];
        for (int i0 = wave * 64; i0 < n_act; i0 += (kScatterThreads / 64) * 64) {
            unsigned long long wf = 0;
            int b = 0, e = 0;
            if (i0 + lane < n_act) {
                const uint4 raw = *reinterpret_cast<const uint4*>(act + i0 + lane);      // weight and bounds in one load
                const double lw = __longlong_as_double((long long)(((unsigned long long)raw.y << 32) | raw.x));
                wf = (unsigned long long)llrint(lw * scale);
                if (wf) {
                    b = (int)raw.z;
                    e = (int)raw.w;
                    if (a.sorted && a.npb > 1 && e - b > kNarrowMin) {      // the first and the last block need one search
                        if (blockIdx.x > 0) b = lower_bound_pos(pos, b, e, p0);
                        if ((int)blockIdx.x < a.npb - 1) e = lower_bound_pos(pos, b, e, p1);
                    }
                }
            }
            unsigned long long m = __ballot(e > b);
            while (m) {
                int bb[kWalk], ee[kWalk];
                unsigned long long ww[kWalk];
#pragma unroll
                for (int j = 0; j < kWalk; ++j) {
                    const int src = m ? (int)__builtin_ctzll(m) : -1;
                    if (m) m &= m - 1;
                    bb[j] = __builtin_amdgcn_readlane(b, src < 0 ? 0 : src);
                    ee[j] = src < 0 ? bb[j] : __builtin_amdgcn_readlane(e, src);
                    const unsigned lo = __builtin_amdgcn_readlane((unsigned)wf, src < 0 ? 0 : src);
                    const unsigned hi = __builtin_amdgcn_readlane((unsigned)(wf >> 32), src < 0 ? 0 : src);
                    ww[j] = ((unsigned long long)hi << 32) | lo;
                }
                // the kWalk lists side by side, 64 postings of each per round, for up to kWalkRounds rounds
                int longest = 0;
#pragma unroll
                for (int j = 0; j < kWalk; ++j) longest = max(longest, ee[j] - bb[j]);
                const int rounds = min((longest + 63) >> 6, kWalkRounds);
                for (int r = 0; r < rounds; ++r) {
                    int32_t pp[kWalk];
#pragma unroll
                    for (int j = 0; j < kWalk; ++j) {
                        const int q = bb[j] + r * 64 + lane;
                        pp[j] = q < ee[j] ? pos[q] : -1;
                    }
#pragma unroll
                    for (int j = 0; j < kWalk; ++j) {
                        const unsigned rr = (unsigned)((int64_t)pp[j] - p0);
                        if (pp[j] >= 0 && rr < span) atomicAdd(&sblk[rr], ww[j]);
                    }
                }
#pragma unroll
                for (int j = 0; j < kWalk; ++j)     // rest of a very long list, kWalk loads in flight per step
                    for (int q0 = bb[j] + 64 * kWalkRounds + lane; q0 - lane < ee[j]; q0 += 64 * kWalk) {
                        int32_t pq[kWalk];
#pragma unroll
                        for (int u = 0; u < kWalk; ++u) pq[u] = q0 + u * 64 < ee[j] ? pos[q0 + u * 64] : -1;
#pragma unroll
                        for (int u = 0; u < kWalk; ++u) {
                            const unsigned rr = (unsigned)((int64_t)pq[u] - p0);
                            if (pq[u] >= 0 && rr < span) atomicAdd(&sblk[rr], ww[j]);
                        }
                    }
            }
        }
    }
    __syncthreads();
    unsigned long long* dst = a.ngroup > 1 ? a.part + (size_t)blockIdx.y * a.L : a.sfix;
    for (int64_t i = tid; i < (int64_t)span; i += kScatterThreads) dst[p0 + i] = sblk[i];
}

__global__ __launch_bounds__(256) void sc_reduce_kernel(ScoreArgs a) {
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < a.L; t += (int64_t)gridDim.x * 256) {
        unsigned long long s = 0;
        for (int g = 0; g < a.ngroup; ++g) s += a.part[(size_t)g * a.L + t];
        a.sfix[t] = s;
    }
}

constexpr int kRun = 32;   // consecutive windows per thread (sliding sum, exact in integers)

__global__ __launch_bounds__(256) void sc_pool_kernel(ScoreArgs a) {
    const double inv = ldexp(1.0, -exp_s(a.sc, a.hb));
    if (a.scores_out)
        for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < a.L; t += (int64_t)gridDim.x * 256)
            a.scores_out[t] = (float)((double)a.sfix[t] * inv);
    for (int64_t s0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * kRun; s0 < a.nW; s0 += (int64_t)gridDim.x * 256 * kRun) {
        unsigned long long acc = 0;
        for (int t = 0; t < a.len; ++t) acc += a.sfix[s0 + t];
        a.wfix[s0] = (long long)acc;
        for (int j = 1; j < kRun && s0 + j < a.nW; ++j) {
            acc += a.sfix[s0 + j + a.len - 1] - a.sfix[s0 + j - 1];
            a.wfix[s0 + j] = (long long)acc;
        }
    }
}

// (value, index) argmax over the block: larger value wins, ties -> smaller index; value -1 = nothing
template <int NT>
__device__ __forceinline__ void block_argmax(long long& v, int& i, long long* sv, int* si) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned int lo = (unsigned int)__shfl_xor((int)(unsigned int)(unsigned long long)v, o);
        unsigned int hi = (unsigned int)__shfl_xor((int)(unsigned int)((unsigned long long)v >> 32), o);
        long long ov = (long long)(((unsigned long long)hi << 32) | lo);
        int oi = __shfl_xor(i, o);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sv[wave] = v; si[wave] = i; }
    __syncthreads();
    long long bv = sv[0];
    int bi = si[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) {
        long long ov = sv[w];
        int oi = si[w];
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    v = bv; i = bi;
}

__global__ __launch_bounds__(kTileW) void sc_tilemax_kernel(ScoreArgs a) {
    __shared__ long long sv[kTileW / 64];
    __shared__ int si[kTileW / 64];
    const int64_t s = (int64_t)blockIdx.x * kTileW + threadIdx.x;
    long long v = s < a.nW ? a.wfix[s] : -1;
    int i = s < a.nW ? (int)s : 0x7FFFFFFF;
    if (s < a.nW) a.dead[s] = 0;
    block_argmax<kTileW>(v, i, sv, si);
    if (threadIdx.x == 0) { a.tmaxv[blockIdx.x] = v; a.tmaxi[blockIdx.x] = i; }
}

__global__ __launch_bounds__(kTileW) void sc_topb_kernel(ScoreArgs a) {
    __shared__ long long sv[kTileW / 64];
    __shared__ int si[kTileW / 64];
    const int tid = threadIdx.x;
    const double inv = ldexp(1.0, -exp_s(a.sc, a.hb));
    int found = 0;
    for (int r = 0; r < a.top_b; ++r) {
        long long v = -1;
        int i = 0x7FFFFFFF;
        for (int t = tid; t < a.ntile; t += kTileW) {
            long long tv = a.tmaxv[t];
            int ti = a.tmaxi[t];
            if (tv > v || (tv == v && ti < i)) { v = tv; i = ti; }
        }
        block_argmax<kTileW>(v, i, sv, si);
        if (v < 0) break;
        if (tid == 0) {
            a.span_start[r] = i;
            a.span_score[r] = (float)((double)v * inv);
        }
        found = r + 1;
        const int64_t lo = a.nms ? max((int64_t)0, (int64_t)i - a.len + 1) : i;
        const int64_t hi = a.nms ? min(a.nW - 1, (int64_t)i + a.len - 1) : i;
        for (int64_t s = lo + tid; s <= hi; s += kTileW) a.dead[s] = 1;
        __syncthreads();
        for (int t = (int)(lo / kTileW); t <= (int)(hi / kTileW); ++t) {
            const int64_t s = (int64_t)t * kTileW + tid;
            long long tv = (s < a.nW && !a.dead[s]) ? a.wfix[s] : -1;
            int ti = tv >= 0 ? (int)s : 0x7FFFFFFF;
            block_argmax<kTileW>(tv, ti, sv, si);
            if (tid == 0) { a.tmaxv[t] = tv; a.tmaxi[t] = ti; }
        }
        __syncthreads();
    }
    for (int r = found + tid; r < a.top_b; r += kTileW) { a.span_start[r] = -1; a.span_score[r] = 0.f; }
    if (tid == 0) a.n_found[0] = found;
}

struct Layout {
    size_t sc, qacc, nact, sfix, wfix, dead, tmaxv, tmaxi, part, act, total;
    int pb, npb, heads_per, ngroup;   // LDS scatter geometry (npb == 0: the global-atomic scatter is used)
};

Layout layout(int n_heads, int n_feat, int64_t L) {
    Layout l;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += s3_align(bytes); return at; };
    const size_t ntile = (size_t)(L + kTileW - 1) / kTileW;
    l.sc = take(sizeof(Scal));
    l.sfix = take((size_t)L * 8);            // sc and sfix are adjacent: zeroed together with qacc
    l.qacc = take((size_t)n_heads * n_feat * 8);
    l.nact = take((size_t)n_heads * 4);     // zeroed with the three before it
    l.wfix = take((size_t)L * 8);
    l.dead = take((size_t)L);
    l.tmaxv = take(ntile * 8);
    l.tmaxi = take(ntile * 4);
    // position blocks of at most kMaxPB scores (128 KB of LDS); enough head groups for about one workgroup per compute unit
    l.pb = (int)(L < kMaxPB ? (L + 63) / 64 * 64 : kMaxPB);
    const int64_t npb = (L + l.pb - 1) / l.pb;
    l.npb = npb <= kMaxBlocks ? (int)npb : 0;
    l.heads_per = 1; l.ngroup = 1; l.part = o; l.act = o;
    if (l.npb) {
        int want = 256 / l.npb;
        int groups = n_heads < want ? n_heads : (want < 1 ? 1 : want);
        l.heads_per = (n_heads + groups - 1) / groups;
        l.ngroup = (n_heads + l.heads_per - 1) / l.heads_per;
        if (l.ngroup > 1) l.part = take((size_t)l.ngroup * L * 8);
        l.act = take((size_t)n_heads * n_feat * sizeof(ActiveList));
    }
    l.total = o;
    return l;
}

}  // namespace

extern "C" size_t s3_coactivate_score_workspace(const s3_index* idx, int64_t n_positions) {
    if (!idx || n_positions < 1) return 0;
    int n_heads, n_feat, k;
    int64_t tokens, os, ps;
    const int32_t *off, *pos;
    bool fin, sorted;
    s3_index_view(idx, &n_heads, &n_feat, &k, &tokens, &off, &os, &pos, &ps, &fin, &sorted);
    return layout(n_heads, n_feat, n_positions).total;
}

extern "C" int s3_coactivate_score(const s3_index* idx, const int32_t* qids, const float* qvals, int nq,
                                   int64_t n_positions, int span_len, int top_b, int32_t max_freq, int nms,
                                   float* scores_out, int32_t* span_start, float* span_score, int32_t* n_found,
                                   void* ws, size_t ws_bytes, void* stream) {
    if (!idx || !span_start || !span_score || !n_found || !ws) return s3_fail(S3_EINVAL, "s3_coactivate_score: null pointer");
    if (nq < 0 || (nq > 0 && (!qids || !qvals))) return s3_fail(S3_EINVAL, "s3_coactivate_score: bad query arrays");
    if (span_len < 1 || top_b < 1 || top_b > 1024)
        return s3_fail(S3_EINVAL, "s3_coactivate_score: span_len %d (>= 1) / top_b %d (1..1024) out of range", span_len, top_b);
    if (n_positions < 1 || n_positions >= (1LL << 31))
        return s3_fail(S3_EINVAL, "s3_coactivate_score: n_positions %lld out of range", (long long)n_positions);
    ScoreArgs a;
    int64_t tokens;
    bool fin, sorted;
    s3_index_view(idx, &a.n_heads, &a.n_feat, &a.k, &tokens, &a.offsets, &a.off_stride, &a.positions, &a.pos_stride, &fin,
                  &sorted);
    if (!fin) return s3_fail(S3_ESTATE, "s3_coactivate_score: index not finalized");
    if ((int64_t)nq * a.k > (1 << 20)) return s3_fail(S3_EINVAL, "s3_coactivate_score: nq * k %lld > 2^20", (long long)nq * a.k);
    const Layout l = layout(a.n_heads, a.n_feat, n_positions);
    if (ws_bytes < l.total) return s3_fail(S3_ECAPACITY, "s3_coactivate_score: workspace %zu < %zu bytes", ws_bytes, l.total);
    if ((uintptr_t)ws & 255) return s3_fail(S3_EINVAL, "s3_coactivate_score: workspace must be 256-byte aligned");

    char* base = (char*)ws;
    a.qids = qids; a.qvals = qvals; a.nq = nq;
    a.L = n_positions;
    a.len = (int)(span_len < n_positions ? span_len : n_positions);
    a.nW = n_positions - a.len + 1;
    a.top_b = top_b; a.nms = nms ? 1 : 0; a.max_freq = max_freq;
    // Headroom of the 64-bit fixed point: a position sums at most n_heads * k weights, a window at most span_len
    // positions; four more bits are spare.  Weights keep 62 - hb significant bits below the largest one.
    a.hb = s3_ceil_log2((unsigned)(a.n_heads * a.k)) + s3_ceil_log2((unsigned)a.len) + 4;
    if (a.hb > 40)
        return s3_fail(S3_EINVAL, "s3_coactivate_score: n_heads * k * span_len too large for the 64-bit fixed-point sums "
                                  "(log2 of it, rounded up per factor, must be <= 36)");
    a.sc = (Scal*)(base + l.sc);
    a.sfix = (unsigned long long*)(base + l.sfix);
    a.qacc = (unsigned long long*)(base + l.qacc);
    a.nact = (int*)(base + l.nact);
    a.act = (ActiveList*)(base + l.act);
    a.wfix = (long long*)(base + l.wfix);
    a.dead = (unsigned char*)(base + l.dead);
    a.tmaxv = (long long*)(base + l.tmaxv);
    a.tmaxi = (int*)(base + l.tmaxi);
    a.part = (unsigned long long*)(base + l.part);
    a.pb = l.pb; a.npb = l.npb; a.heads_per = l.heads_per; a.ngroup = l.ngroup; a.sorted = sorted ? 1 : 0;
    a.ntile = (int)((a.nW + kTileW - 1) / kTileW);
    a.scores_out = scores_out; a.span_start = span_start; a.span_score = span_score; a.n_found = n_found;

    hipStream_t st = (hipStream_t)stream;
    const size_t nzero = (l.wfix - l.sc) / 8;   // Scal + sfix + qacc + nact
    auto blocks = [](size_t n, size_t per) { size_t b = (n + per - 1) / per; return (unsigned)(b < 1 ? 1 : (b > 65536 ? 65536 : b)); };
    hipLaunchKernelGGL(sc_zero_kernel, dim3(blocks(nzero, 256)), dim3(256), 0, st, (unsigned long long*)(base + l.sc), nzero);
    const size_t npairs = (size_t)a.n_heads * nq * a.k;
    if (npairs) {
        hipLaunchKernelGGL(sc_qmax_kernel, dim3(blocks(npairs, 256 * 4) > 512 ? 512 : blocks(npairs, 256 * 4)), dim3(256), 0, st, a);
        hipLaunchKernelGGL(sc_qacc_kernel, dim3(blocks(npairs, 256)), dim3(256), 0, st, a);
        const size_t nhf = (size_t)a.n_heads * a.n_feat;
        hipLaunchKernelGGL(sc_qw_kernel, dim3((unsigned)((nhf + 256 * kQwPer - 1) / (256 * kQwPer))), dim3(256), 0, st, a);
        if (a.npb) {
            static S3LdsOnce once;
            if (int rc = s3_allow_lds(once, (const void*)sc_scatter_lds_kernel, kMaxPB * 8)) return rc;
            hipLaunchKernelGGL(sc_scatter_lds_kernel, dim3((unsigned)a.npb, (unsigned)a.ngroup), dim3(kScatterThreads),
                               (size_t)a.pb * 8, st, a);
            if (a.ngroup > 1) hipLaunchKernelGGL(sc_reduce_kernel, dim3(blocks((size_t)a.L, 256)), dim3(256), 0, st, a);
        } else {
            hipLaunchKernelGGL(sc_scatter_kernel, dim3((unsigned)((nhf + 3) / 4)), dim3(256), 0, st, a);
        }
    }
    hipLaunchKernelGGL(sc_pool_kernel, dim3(blocks((size_t)a.L, 256)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(sc_tilemax_kernel, dim3(a.ntile), dim3(kTileW), 0, st, a);
    hipLaunchKernelGGL(sc_topb_kernel, dim3(1), dim3(kTileW), 0, st, a);
    S3_HIP(hipGetLastError());
    return S3_OK;
}
