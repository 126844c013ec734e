// Generation-time co-activation scoring (Sec. 3.5 scoring equation; App. D.2 / App. E weights;
// Sec. 3.5 "Adaptive Granularity" read as box pooling + fixed-length spans with NMS).
//
//   1. query weights   qw[h][f] = IDF_h(f) * sum of the query activations that name f (summed per head in LDS)
//   2. postings gather S[t] += qw[h][f] for every t in I_h[f], all heads into one S: a workgroup keeps the scores
//      of one block of positions in LDS and reads, of every list, only the postings of its block (the index's
//      block table); no atomic ever reaches global memory, at any context length
//   3. span pooling    W[s] = S[s] + ... + S[s + len - 1], with the best window of every tile
//   4. Top-B           greedy best window, optional suppression of overlapping windows
//
// Every sum is carried in 64-bit fixed point (power-of-two scales derived on the device from a head's
// largest query activation / the largest weight), so additions commute exactly: the result does not
// depend on the order in which wavefronts reach a position, run-to-run output is bit-identical,
// and a window's score is exactly the sum of its members.  Values are rounded to fp32 once, on
// output.
#include "s3_common.h"

#include <math.h>

#include <type_traits>

namespace {

// A posting list with a non-zero query weight.
struct alignas(16) ActiveList {
    double w;
    int32_t f;
    int32_t pad;
};

struct ScoreArgs {
    const int32_t* qids;
    const float* qvals;
    const int32_t* offsets;
    const int32_t* positions;
    int64_t off_stride, pos_stride;
    const int32_t* btab;             // block table of the index (null: none or not usable)
    int nblk;                        // blocks the table covers
    // compact index (all null / 0 for the plain one): 16-bit block-relative postings in block-major order
    const uint16_t* delta;           // [n_heads] x delta_stride
    const int32_t* cstart;           // [n_heads] x cstart_stride: start of segment (block b, feature f) at b * n_feat + f
    const int32_t* cfreq;            // [n_heads][n_feat] list lengths (0: dropped)
    int64_t delta_stride, cstart_stride;
    int n_heads, n_feat, k, nq;
    int nr;                          // feature ranges per head (sc_prep_kernel)
    int64_t L, nW;
    int len, top_b, nms, hb;
    int32_t max_freq;
    unsigned long long* wmax;        // [n_heads * nr] bits (as double) of each range's largest weight; [n_heads * nr]: of all
    ActiveList* act;                 // [n_heads * n_feat] lists with a non-zero weight, packed per (head, range)
    int* nact;                       // [n_heads * nr] their number
    unsigned long long* sfix;        // [L]
    unsigned long long* part;        // [ngroup][L] partial sums of head groups (ngroup > 1)
    int pb, npb, heads_per, ngroup, sorted;   // position blocks / head groups of the gather
    long long* wfix;                 // [nW]
    long long* tmaxv;                // [ntile]
    int* tmaxi;                      // [ntile]
    int ntile;
    float* scores_out;
    int32_t* span_start;
    float* span_score;
    int32_t* n_found;
};

constexpr int kRange = 16384;        // features whose sums one workgroup of sc_prep_kernel holds in LDS
constexpr int kPrepThreads = 1024;
constexpr int kRun = 32;             // consecutive windows per thread (sliding sum, exact in integers)
constexpr int kTileW = 64 * kRun;    // windows per tile = per wavefront of the pooling kernel
constexpr int kTopThreads = 256;

__device__ __forceinline__ int exp_s(unsigned long long wmax_bits, int hb) {   // weights are scaled by 2^exp_s: sums < 2^62
    double w = __longlong_as_double((long long)wmax_bits);
    if (!(w > 0.0)) return 0;
    int e;
    frexp(w, &e);
    return 62 - hb - e;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned int lo = (unsigned int)__shfl_xor((int)(unsigned int)v, o);
        unsigned int hi = (unsigned int)__shfl_xor((int)(unsigned int)(v >> 32), o);
        unsigned long long other = ((unsigned long long)hi << 32) | lo;
        v = other > v ? other : v;
    }
    return v;
}

// Query weights of one (head, range of kRange features): the head's query pairs are summed per feature in LDS
// (64-bit fixed point, scaled by the head's largest activation, so the sum does not depend on the order), turned
// into weights qw[f] = IDF(f) * sum (App. D.2; natural log; lists longer than max_freq skipped, App. E), and the
// lists with a non-zero weight are packed for the gather.  One workgroup writes its own slice of every output:
// nothing has to be zeroed beforehand and no atomic leaves the workgroup.
__global__ __launch_bounds__(kPrepThreads) void sc_prep_kernel(ScoreArgs a) {
    extern __shared__ unsigned long long tbl[];
    __shared__ unsigned int amax[kPrepThreads / 64];
    __shared__ unsigned long long wmx[kPrepThreads / 64];
    __shared__ int wsum[kPrepThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.y, r = blockIdx.x;
    const int f0 = r * kRange, nf = min(kRange, a.n_feat - f0);
    for (int i = tid; i < nf; i += kPrepThreads) tbl[i] = 0ull;
    const size_t per_head = (size_t)a.nq * a.k;
    const float* qv = a.qvals + (size_t)h * per_head;
    const int32_t* qi = a.qids + (size_t)h * per_head;
    unsigned int m = 0;
    for (size_t i = tid; i < per_head; i += kPrepThreads) m = max(m, __float_as_uint(fmaxf(qv[i], 0.f)));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, (unsigned int)__shfl_xor((int)m, o));
    if (lane == 0) amax[wave] = m;
    __syncthreads();
    m = 0;
#pragma unroll
    for (int q = 0; q < kPrepThreads / 64; ++q) m = max(m, amax[q]);
    int eq = 0;                      // activations are scaled by 2^eq: each below 2^40, a sum of 2^20 of them below 2^60
    if (m) {
        int e;
        frexpf(__uint_as_float(m), &e);
        eq = 40 - e;
    }
    const double scale = ldexp(1.0, eq), inv = ldexp(1.0, -eq);
    for (size_t i = tid; i < per_head; i += kPrepThreads) {
        const float v = fmaxf(qv[i], 0.f);
        const unsigned int f = (unsigned int)(qi[i] - f0);
        if (v > 0.f && f < (unsigned int)nf) atomicAdd(&tbl[f], (unsigned long long)llrint((double)v * scale));
    }
    __syncthreads();
    constexpr int kPer = kRange / kPrepThreads;
    const int32_t* off = a.cfreq ? nullptr : a.offsets + (size_t)h * a.off_stride + f0;
    double w[kPer];
    int c = 0;
    double mx = 0.0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = j * kPrepThreads + tid;
        w[j] = 0.0;
        if (i < nf) {
            const unsigned long long sacc = tbl[i];
            if (sacc) {
                const int freq = a.cfreq ? a.cfreq[(size_t)h * a.n_feat + f0 + i] : off[i + 1] - off[i];
                if (freq > 0 && !(a.max_freq > 0 && freq > a.max_freq))
                    w[j] = (double)sacc * inv / ((double)logf(1.0f + (float)freq) + 1.0);
            }
        }
        c += w[j] > 0.0 ? 1 : 0;
        mx = fmax(mx, w[j]);
    }
    int tot;
    int slot = s3_block_excl_scan<kPrepThreads>(c, wsum, tot);
    ActiveList* out = a.act + (size_t)h * a.n_feat + f0;
#pragma unroll
    for (int j = 0; j < kPer; ++j)
        if (w[j] > 0.0) out[slot++] = ActiveList{w[j], f0 + j * kPrepThreads + tid, 0};
    const unsigned long long mb = wave_max_u64((unsigned long long)__double_as_longlong(mx));
    if (lane == 0) wmx[wave] = mb;
    __syncthreads();
    if (tid == 0) {
        unsigned long long best = 0;
        for (int q = 0; q < kPrepThreads / 64; ++q) best = wmx[q] > best ? wmx[q] : best;
        a.wmax[h * a.nr + r] = best;
        a.nact[h * a.nr + r] = tot;
    }
}

// Postings gather with the scores of one block of positions held in LDS.
// Workgroup (b, g) owns positions [b * pb, (b + 1) * pb) and the heads of group g: it walks every posting list
// of those heads that has a non-zero weight and adds the postings that fall into its block with LDS atomics
// (64-bit fixed point, so the order of the additions does not matter), then stores the block: into S when there
// is one head group, else into that group's partial array (summed by sc_reduce_kernel).  No global atomics.
// A wavefront takes 64 lists at a time: lane l fetches weight and feature of list l and the part of the list that
// lies in the block (its segment) -- from the index's block table when there is one; else, for lists sorted by
// position, by a search; else the whole list, every posting filtered.  Postings are read as aligned 16-byte vectors
// (what a wavefront keeps in flight bounds the rate: the gather is latency-bound).  Segments of more than 2 G
// vectors are walked one at a time by the whole wavefront, the others G lanes per segment (64 / G segments per load
// instruction); G is picked on the host from the mean segment length.
constexpr int kScatterThreads = 1024;
constexpr int kLong = 4;             // vector loads per lane in flight while a long segment is walked by the whole wavefront
constexpr int kShortSlots = 4;       // vector loads per lane in flight while short segments are walked by lane groups
constexpr int kNarrowMin = 128;      // sorted lists longer than this are narrowed to the position block by search
constexpr int kMaxPB = 1 << kS3PosBlockLog2;

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

// element j of a vector of four postings (int32: a 16-byte vector; uint16: an 8-byte one), as an unsigned position value
__device__ __forceinline__ unsigned vec_posting(const uint4& v, int j) {
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
    return w[j];
}
__device__ __forceinline__ unsigned vec_posting(const uint2& v, int j) {
    const unsigned w[2] = {v.x, v.y};
    return (w[j >> 1] >> ((j & 1) * 16)) & 0xFFFFu;
}

template <int G, bool CMP>
__global__ __launch_bounds__(kScatterThreads) void sc_scatter_lds_kernel(ScoreArgs a) {
    extern __shared__ unsigned long long sblk[];
    __shared__ unsigned long long wmx[kScatterThreads / 64];
    __shared__ int4 recs_all[kScatterThreads];           // per wavefront: (begin, length, weight) of the batch's segments
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int4* const recs = recs_all + wave * 64;
    const int blk = blockIdx.x;
    const int64_t p0 = (int64_t)blk * a.pb;
    const int64_t p1 = p0 + a.pb < a.L ? p0 + a.pb : a.L;
    const unsigned span = (unsigned)(p1 - p0);
    for (int i = tid; i < a.pb; i += kScatterThreads) sblk[i] = 0ull;
    // the largest weight over all heads fixes the fixed-point scale (every workgroup derives the same one)
    unsigned long long mb = 0;
    for (int i = tid; i < a.n_heads * a.nr; i += kScatterThreads) mb = a.wmax[i] > mb ? a.wmax[i] : mb;
    mb = wave_max_u64(mb);
    if (lane == 0) wmx[wave] = mb;
    __syncthreads();
    mb = 0;
#pragma unroll
    for (int q = 0; q < kScatterThreads / 64; ++q) mb = wmx[q] > mb ? wmx[q] : mb;
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) a.wmax[a.n_heads * a.nr] = mb;      // for the kernels that follow
    const double scale = ldexp(1.0, exp_s(mb, a.hb));
    const int nbk = a.nblk - 1;
    const int h0 = blockIdx.y * a.heads_per, h1 = min(a.n_heads, h0 + a.heads_per);
    for (int hr = h0 * a.nr; hr < h1 * a.nr; ++hr) {
        const int h = hr / a.nr, r = hr - h * a.nr;
        // compact index: 16-bit offsets from the block's start, the block's segments one after the other
        using Posting = typename std::conditional<CMP, uint16_t, int32_t>::type;
        const Posting* pos = CMP ? (const Posting*)(a.delta + (size_t)h * a.delta_stride)
                                 : (const Posting*)(a.positions + (size_t)h * a.pos_stride);
        const int32_t* off = CMP ? a.cstart + (size_t)h * a.cstart_stride + (size_t)blk * a.n_feat
                                 : a.offsets + (size_t)h * a.off_stride;
        const int32_t* tab = !CMP && a.btab ? a.btab + (size_t)h * a.n_feat * nbk : nullptr;
        const unsigned pbase = CMP ? 0u : (unsigned)p0;           // what a stored posting is relative to
        const bool cmp_empty = CMP && blk >= a.nblk;              // the compact index holds nothing beyond its blocks
        const ActiveList* act = a.act + (size_t)h * a.n_feat + (size_t)r * kRange;
        const int n_act = a.nact[hr];
        constexpr int kStep = (kScatterThreads / 64) * 64;
        uint4 raw_next = make_uint4(0, 0, 0, 0);
        if (wave * 64 + lane < n_act) raw_next = *reinterpret_cast<const uint4*>(act + wave * 64 + lane);
        for (int i0 = wave * 64; i0 < n_act; i0 += kStep) {
            unsigned long long wf = 0;
            int b = 0, e = 0;
            const uint4 raw = raw_next;                      // weight and feature in one load, fetched one batch ahead
            if (i0 + kStep + lane < n_act) raw_next = *reinterpret_cast<const uint4*>(act + i0 + kStep + lane);
            if (i0 + lane < n_act) {
                const double lw = __longlong_as_double((long long)(((unsigned long long)raw.y << 32) | raw.x));
                wf = (unsigned long long)llrint(lw * scale);
                if (wf) {
                    const int f = (int)raw.z;
                    if (CMP) {
                        if (!cmp_empty) {
                            b = off[f];
                            e = off[f + 1];
                        }
                    } else if (a.npb == 1) {
                        b = off[f];
                        e = off[f + 1];
                    } else if (tab) {         // blocks at or beyond the table's end hold nothing
                        const int lb = off[f], le = off[f + 1];
                        b = blk == 0 ? lb : (blk <= nbk ? tab[(size_t)f * nbk + blk - 1] : le);
                        e = blk < nbk ? tab[(size_t)f * nbk + blk] : le;
                        b = max(b, lb);       // whatever the table holds, nothing outside the list is read
                        e = min(e, le);
                    } else {
                        b = off[f];
                        e = off[f + 1];
                        if (a.sorted && e - b > kNarrowMin) {      // the first and the last block need one search
                            const int32_t* pl = a.positions + (size_t)h * a.pos_stride;
                            if (blk > 0) b = lower_bound_pos(pl, b, e, p0);
                            if (blk < a.npb - 1) e = lower_bound_pos(pl, b, e, p1);
                        }
                    }
                }
            }
            // this batch's segments (the part of each list that lies in the block) go to the wavefront's records
            const int n = wf ? max(e - b, 0) : 0;
            recs[lane] = make_int4(b, n, (int)(unsigned)wf, (int)(unsigned)(wf >> 32));
            // Every load is an aligned vector of four postings (16 bytes of int32, 8 bytes of uint16: as many loads in
            // flight per posting either way, half the bytes for the compact index): a segment is read from the vector
            // boundary at or before its first posting, and the elements in front of it and behind its end are masked
            // out (they lie in the same vector as a posting of the array, hence inside the array's allocation).
            constexpr int EPV = 4;
            constexpr int VB = EPV * (int)sizeof(Posting);
            using Vec = typename std::conditional<sizeof(Posting) == 4, uint4, uint2>::type;
            const int nv = n ? (int)(((((uintptr_t)(pos + b)) & (VB - 1)) / sizeof(Posting) + n + EPV - 1) / EPV) : 0;
            // long segments (more than 2 G vectors): one at a time, the whole wavefront, kLong vectors in flight per lane
            unsigned long long ml = __ballot(nv > 2 * G);
            while (ml) {
                const int src = (int)__builtin_ctzll(ml);
                ml &= ml - 1;
                const int sb = __builtin_amdgcn_readlane(b, src), sn = __builtin_amdgcn_readlane(n, src);
                const unsigned long long w = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(wf >> 32), src) << 32) |
                                             (unsigned)__builtin_amdgcn_readlane((int)(unsigned)wf, src);
                const uintptr_t addr = (uintptr_t)(pos + sb);                       // uniform
                const int shift = (int)((addr & (VB - 1)) / sizeof(Posting));
                const Vec* vp = (const Vec*)(addr & ~(uintptr_t)(VB - 1));
                const int total = shift + sn, nvec = (total + EPV - 1) / EPV;
                for (int v0 = 0; v0 < nvec; v0 += 64 * kLong) {
                    Vec raw[kLong];
#pragma unroll
                    for (int u = 0; u < kLong; ++u) {
                        const int vi = v0 + u * 64 + lane;
                        raw[u] = vi < nvec ? vp[vi] : Vec{};
                    }
#pragma unroll
                    for (int u = 0; u < kLong; ++u) {
                        const int el0 = (v0 + u * 64 + lane) * EPV;
#pragma unroll
                        for (int j = 0; j < EPV; ++j) {
                            const unsigned rr = vec_posting(raw[u], j) - pbase;
                            if (el0 + j >= shift && el0 + j < total && rr < span) atomicAdd(&sblk[rr], w);
                        }
                    }
                }
            }
            // short segments: G lanes per segment (one vector each, two rounds if needed), 64 / G segments per load
            // instruction, kShortSlots load instructions in flight
            constexpr int LPS = 64 / G;
            const int grp = lane / G, sub = lane % G;
            unsigned long long ms = __ballot(nv > 0 && nv <= 2 * G);
            while (ms) {
                int4 rc[kShortSlots];
                bool two = false;
#pragma unroll
                for (int u = 0; u < kShortSlots; ++u) {
                    int idx = -1;
#pragma unroll
                    for (int g = 0; g < LPS; ++g) {                        // the next LPS segments, one per lane group
                        const int sbit = ms ? (int)__builtin_ctzll(ms) : -1;
                        if (ms) ms &= ms - 1;
                        idx = grp == g ? sbit : idx;
                    }
                    rc[u] = idx >= 0 ? recs[idx] : make_int4(0, 0, 0, 0);
                }
                const Vec* vp[kShortSlots];
                int shift[kShortSlots], total[kShortSlots];
#pragma unroll
                for (int u = 0; u < kShortSlots; ++u) {
                    const uintptr_t addr = (uintptr_t)(pos + rc[u].x);
                    shift[u] = (int)((addr & (VB - 1)) / sizeof(Posting));
                    vp[u] = (const Vec*)(addr & ~(uintptr_t)(VB - 1));
                    total[u] = rc[u].y ? shift[u] + rc[u].y : 0;
                    two = two || total[u] > G * EPV;
                }
                const int chunks = __any(two) ? 2 : 1;
                for (int c = 0; c < chunks; ++c) {
                    Vec raw[kShortSlots];
#pragma unroll
                    for (int u = 0; u < kShortSlots; ++u)
                        raw[u] = (c * G + sub) * EPV < total[u] ? vp[u][c * G + sub] : Vec{};
#pragma unroll
                    for (int u = 0; u < kShortSlots; ++u) {
                        const unsigned long long w = ((unsigned long long)(unsigned)rc[u].w << 32) | (unsigned)rc[u].z;
                        const int el0 = (c * G + sub) * EPV;
#pragma unroll
                        for (int j = 0; j < EPV; ++j) {
                            const unsigned rr = vec_posting(raw[u], j) - pbase;
                            if (el0 + j >= shift[u] && el0 + j < total[u] && rr < span) atomicAdd(&sblk[rr], w);
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    unsigned long long* dst = a.ngroup > 1 ? a.part + (size_t)blockIdx.y * a.L : a.sfix;
    for (int64_t i = tid; i < (int64_t)span; i += kScatterThreads) dst[p0 + i] = sblk[i];
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

// S = sum of the head groups' partial arrays.  64 positions per workgroup, four threads per position (each takes
// every fourth group), so that a short context still fills the chip and every thread's loads are independent.
__global__ __launch_bounds__(256) void sc_reduce_kernel(ScoreArgs a) {
    __shared__ unsigned long long partial[4][64];
    const int p = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 64 + p;
    unsigned long long s0 = 0, s1 = 0;
    if (t < a.L) {
        int g = q;
        for (; g + 4 < a.ngroup; g += 8) {
            s0 += a.part[(size_t)g * a.L + t];
            s1 += a.part[(size_t)(g + 4) * a.L + t];
        }
        if (g < a.ngroup) s0 += a.part[(size_t)g * a.L + t];
    }
    partial[q][p] = s0 + s1;
    __syncthreads();
    if (q == 0 && t < a.L) a.sfix[t] = partial[0][p] + partial[1][p] + partial[2][p] + partial[3][p];
}

// Inclusive prefix sum of one 64-bit value per thread over the block (wrap-around arithmetic: exact differences).
template <int NT>
__device__ __forceinline__ unsigned long long block_incl_scan_u64(unsigned long long v, unsigned long long* wsum) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned int lo = (unsigned int)__shfl_up((int)(unsigned int)v, o);
        const unsigned int hi = (unsigned int)__shfl_up((int)(unsigned int)(v >> 32), o);
        if (lane >= o) v += ((unsigned long long)hi << 32) | lo;
    }
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    unsigned long long base = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) base += w < wave ? wsum[w] : 0ull;
    __syncthreads();
    return v + base;
}

// Span pooling, the fp32 scores, and the best window of every tile of kTileW windows (one workgroup per tile).
// The tile's positions are staged in LDS and turned into prefix sums there, so a window costs two LDS reads
// whatever its length: W[s] = P[s + len - 1] - P[s - 1], exact in 64-bit integers.  Larger value wins, ties ->
// smaller start.
constexpr int kPoolThreads = 256;
constexpr int kPoolMaxLen = 4096;      // longer windows take sc_pool_wide_kernel

__global__ __launch_bounds__(kPoolThreads) void sc_pool_kernel(ScoreArgs a) {
    extern __shared__ unsigned long long pre[];          // [kTileW + len - 1 (+ padding)] prefix sums
    __shared__ unsigned long long wsum[kPoolThreads / 64];
    __shared__ long long sv[kPoolThreads / 64];
    __shared__ int si[kPoolThreads / 64];
    const int tid = threadIdx.x;
    const double inv = ldexp(1.0, -exp_s(a.wmax[a.n_heads * a.nr], a.hb));
    const int64_t s0 = (int64_t)blockIdx.x * kTileW;
    const int64_t tend = (int)blockIdx.x == a.ntile - 1 ? a.L : s0 + kTileW;      // positions whose fp32 score this tile writes
    const int n_in = (int)(min(a.L, s0 + kTileW + a.len - 1) - s0);               // positions the tile's windows read
    constexpr int kPer = (kTileW + kPoolMaxLen + kPoolThreads - 1) / kPoolThreads;
    const int per = (n_in + kPoolThreads - 1) / kPoolThreads;                     // consecutive positions per thread (<= kPer)
    // each thread sums its own run, the block scans the run totals, the thread writes its run's prefixes
    unsigned long long run = 0;
    for (int j = 0; j < per; ++j) {
        const int i = tid * per + j;
        if (i < n_in) {
            const unsigned long long v = a.sfix[s0 + i];
            if (a.scores_out && s0 + i < tend) a.scores_out[s0 + i] = (float)((double)v * inv);
            run += v;
            pre[i] = run;
        }
    }
    (void)kPer;
    const unsigned long long incl = block_incl_scan_u64<kPoolThreads>(run, wsum);
    const unsigned long long base = incl - run;
    for (int j = 0; j < per; ++j) {
        const int i = tid * per + j;
        if (i < n_in) pre[i] += base;
    }
    __syncthreads();
    long long bv = -1;
    int bi = 0x7FFFFFFF;
    for (int q = tid; q < kTileW; q += kPoolThreads) {                            // ascending starts per thread
        const int64_t sw = s0 + q;
        if (sw < a.nW) {
            const long long w = (long long)(pre[q + a.len - 1] - (q ? pre[q - 1] : 0ull));
            a.wfix[sw] = w;
            if (w > bv) { bv = w; bi = (int)sw; }
        }
    }
    block_argmax<kPoolThreads>(bv, bi, sv, si);
    if (tid == 0) { a.tmaxv[blockIdx.x] = bv; a.tmaxi[blockIdx.x] = bi; }
}

// The same for windows longer than kPoolMaxLen: sliding sums from global memory, one wavefront per tile.
__global__ __launch_bounds__(256) void sc_pool_wide_kernel(ScoreArgs a) {
    const double inv = ldexp(1.0, -exp_s(a.wmax[a.n_heads * a.nr], a.hb));
    if (a.scores_out)
        for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < a.L; t += (int64_t)gridDim.x * 256)
            a.scores_out[t] = (float)((double)a.sfix[t] * inv);
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= a.ntile) return;
    const int64_t s0 = tile * kTileW + (int64_t)lane * kRun;
    long long bv = -1;
    int bi = 0x7FFFFFFF;
    if (s0 < a.nW) {
        unsigned long long acc = 0;
        for (int t = 0; t < a.len; ++t) acc += a.sfix[s0 + t];
        a.wfix[s0] = (long long)acc;
        bv = (long long)acc;
        bi = (int)s0;
        for (int j = 1; j < kRun && s0 + j < a.nW; ++j) {
            acc += a.sfix[s0 + j + a.len - 1] - a.sfix[s0 + j - 1];
            a.wfix[s0 + j] = (long long)acc;
            if ((long long)acc > bv) { bv = (long long)acc; bi = (int)(s0 + j); }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned int lo = (unsigned int)__shfl_xor((int)(unsigned int)(unsigned long long)bv, o);
        unsigned int hi = (unsigned int)__shfl_xor((int)(unsigned int)((unsigned long long)bv >> 32), o);
        long long ov = (long long)(((unsigned long long)hi << 32) | lo);
        int oi = __shfl_xor(bi, o);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { a.tmaxv[tile] = bv; a.tmaxi[tile] = bi; }
}

// Greedy Top-B with optional suppression of overlapping windows.  One small workgroup: the rounds depend on each
// other.  The tile maxima live in LDS (up to kTopCache tiles; in global memory beyond that); a round takes the best
// one, then searches the tiles again that the new span's suppression touches.  Whether a window is still alive
// follows from the spans chosen so far (kept in LDS): no flag array in memory, one global round trip per round.
constexpr int kTopCache = 4096;

__global__ __launch_bounds__(kTopThreads) void sc_topb_kernel(ScoreArgs a) {
    __shared__ long long sv[kTopThreads / 64];
    __shared__ int si[kTopThreads / 64];
    __shared__ long long cv[kTopCache];
    __shared__ int ci[kTopCache];
    __shared__ int sel[1024];
    const int tid = threadIdx.x;
    const bool cached = a.ntile <= kTopCache;
    const double inv = ldexp(1.0, -exp_s(a.wmax[a.n_heads * a.nr], a.hb));
    if (cached)
        for (int t = tid; t < a.ntile; t += kTopThreads) { cv[t] = a.tmaxv[t]; ci[t] = a.tmaxi[t]; }
    __syncthreads();
    int found = 0;
    for (int r = 0; r < a.top_b; ++r) {
        long long v = -1;
        int i = 0x7FFFFFFF;
        for (int t = tid; t < a.ntile; t += kTopThreads) {
            const long long tv = cached ? cv[t] : a.tmaxv[t];
            const int ti = cached ? ci[t] : a.tmaxi[t];
            if (tv > v || (tv == v && ti < i)) { v = tv; i = ti; }
        }
        block_argmax<kTopThreads>(v, i, sv, si);
        if (v < 0) break;
        if (tid == 0) {
            a.span_start[r] = i;
            a.span_score[r] = (float)((double)v * inv);
            sel[r] = i;
        }
        found = r + 1;
        __syncthreads();
        const int reach = a.nms ? a.len - 1 : 0;              // windows within `reach` of a chosen start are gone
        const int64_t lo = max((int64_t)0, (int64_t)i - reach), hi = min(a.nW - 1, (int64_t)i + reach);
        for (int t = (int)(lo / kTileW); t <= (int)(hi / kTileW); ++t) {
            const int64_t t0 = (int64_t)t * kTileW;
            long long w[kTileW / kTopThreads];
#pragma unroll
            for (int q = 0; q < kTileW / kTopThreads; ++q) {  // all loads first: one round trip
                const int64_t sw = t0 + q * kTopThreads + tid;
                w[q] = sw < a.nW ? a.wfix[sw] : -1;
            }
            for (int j = 0; j < found; ++j) {                 // chosen spans that reach into this tile
                const int64_t c = sel[j];
                if (c + reach < t0 || c - reach >= t0 + kTileW) continue;
#pragma unroll
                for (int q = 0; q < kTileW / kTopThreads; ++q) {
                    const int64_t sw = t0 + q * kTopThreads + tid;
                    if (sw >= c - reach && sw <= c + reach) w[q] = -1;
                }
            }
            long long tv = -1;
            int ti = 0x7FFFFFFF;
#pragma unroll
            for (int q = 0; q < kTileW / kTopThreads; ++q)    // ascending starts per thread: the first best one is kept
                if (w[q] > tv) { tv = w[q]; ti = (int)(t0 + q * kTopThreads + tid); }
            block_argmax<kTopThreads>(tv, ti, sv, si);
            if (tid == 0) {
                if (cached) { cv[t] = tv; ci[t] = ti; }
                else { a.tmaxv[t] = tv; a.tmaxi[t] = ti; }
            }
        }
        __syncthreads();
    }
    for (int r = found + tid; r < a.top_b; r += kTopThreads) { a.span_start[r] = -1; a.span_score[r] = 0.f; }
    if (tid == 0) a.n_found[0] = found;
}

struct Layout {
    size_t wmax, nact, sfix, wfix, tmaxv, tmaxi, part, act, total;
    int nr, pb, npb, heads_per, ngroup;   // feature ranges per head; position blocks and head groups of the gather
};

Layout layout(int n_heads, int n_feat, int64_t L) {
    Layout l;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += s3_align(bytes); return at; };
    const int64_t nW_max = L;
    const size_t ntile = (size_t)(nW_max + kTileW - 1) / kTileW;
    l.nr = (n_feat + kRange - 1) / kRange;
    l.wmax = take(((size_t)n_heads * l.nr + 1) * 8);
    l.nact = take((size_t)n_heads * l.nr * 4);
    l.sfix = take((size_t)L * 8);
    l.wfix = take((size_t)L * 8);
    l.tmaxv = take(ntile * 8);
    l.tmaxi = take(ntile * 4);
    // position blocks of at most kMaxPB scores (128 KB of LDS); enough head groups for about one workgroup per compute unit
    l.pb = (int)(L < kMaxPB ? (L + 63) / 64 * 64 : kMaxPB);
    l.npb = (int)((L + l.pb - 1) / l.pb);
    int want = 256 / l.npb;
    int groups = n_heads < want ? n_heads : (want < 1 ? 1 : want);
    l.heads_per = (n_heads + groups - 1) / groups;
    l.ngroup = (n_heads + l.heads_per - 1) / l.heads_per;
    l.part = o;
    if (l.ngroup > 1) l.part = take((size_t)l.ngroup * L * 8);
    l.act = take((size_t)n_heads * n_feat * sizeof(ActiveList));
    l.total = o;
    return l;
}

// What a scoring call reads from: the plain index (CSR + block table) or the compact one.
struct ScoreSource {
    int n_heads, n_feat, k;
    int64_t tokens;
    bool sorted;
    const int32_t* offsets = nullptr; const int32_t* positions = nullptr; int64_t off_stride = 0, pos_stride = 0;
    const int32_t* btab = nullptr; int nblk = 1;
    const uint16_t* delta = nullptr; const int32_t* cstart = nullptr; const int32_t* cfreq = nullptr;
    int64_t delta_stride = 0, cstart_stride = 0;
};

static int score_run(const char* who, const ScoreSource& v, const int32_t* qids, const float* qvals, int nq,
                     int64_t n_positions, int span_len, int top_b, int32_t max_freq, int nms, float* scores_out,
                     int32_t* span_start, float* span_score, int32_t* n_found, void* ws, size_t ws_bytes, void* stream) {
    if (!span_start || !span_score || !n_found || !ws) return s3_fail(S3_EINVAL, "%s: null pointer", who);
    if (nq < 0 || (nq > 0 && (!qids || !qvals))) return s3_fail(S3_EINVAL, "%s: bad query arrays", who);
    if (span_len < 1 || top_b < 1 || top_b > 1024)
        return s3_fail(S3_EINVAL, "%s: span_len %d (>= 1) / top_b %d (1..1024) out of range", who, span_len, top_b);
    if (n_positions < 1 || n_positions >= (1LL << 31))
        return s3_fail(S3_EINVAL, "%s: n_positions %lld out of range", who, (long long)n_positions);
    ScoreArgs a;
    a.n_heads = v.n_heads; a.n_feat = v.n_feat; a.k = v.k;
    a.offsets = v.offsets; a.off_stride = v.off_stride; a.positions = v.positions; a.pos_stride = v.pos_stride;
    a.btab = v.btab; a.nblk = v.nblk;
    a.delta = v.delta; a.cstart = v.cstart; a.cfreq = v.cfreq; a.delta_stride = v.delta_stride; a.cstart_stride = v.cstart_stride;
    if ((int64_t)nq * a.k > (1 << 20)) return s3_fail(S3_EINVAL, "%s: nq * k %lld > 2^20", who, (long long)nq * a.k);
    const Layout l = layout(a.n_heads, a.n_feat, n_positions);
    if (ws_bytes < l.total) return s3_fail(S3_ECAPACITY, "%s: workspace %zu < %zu bytes", who, ws_bytes, l.total);
    if ((uintptr_t)ws & 255) return s3_fail(S3_EINVAL, "%s: workspace must be 256-byte aligned", who);

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
        return s3_fail(S3_EINVAL, "%s: n_heads * k * span_len too large for the 64-bit fixed-point sums "
                                  "(log2 of it, rounded up per factor, must be <= 36)", who);
    a.nr = l.nr;
    a.wmax = (unsigned long long*)(base + l.wmax);
    a.nact = (int*)(base + l.nact);
    a.sfix = (unsigned long long*)(base + l.sfix);
    a.act = (ActiveList*)(base + l.act);
    a.wfix = (long long*)(base + l.wfix);
    a.tmaxv = (long long*)(base + l.tmaxv);
    a.tmaxi = (int*)(base + l.tmaxi);
    a.part = (unsigned long long*)(base + l.part);
    a.pb = l.pb; a.npb = l.npb; a.heads_per = l.heads_per; a.ngroup = l.ngroup; a.sorted = v.sorted ? 1 : 0;
    a.ntile = (int)((a.nW + kTileW - 1) / kTileW);
    a.scores_out = scores_out; a.span_start = span_start; a.span_score = span_score; a.n_found = n_found;

    hipStream_t st = (hipStream_t)stream;
    static S3LdsOnce once_prep, once_scatter[4];
    const int prep_lds = (a.n_feat < kRange ? a.n_feat : kRange) * 8;
    if (int rc = s3_allow_lds(once_prep, (const void*)sc_prep_kernel, kRange * 8)) return rc;
    // lanes per short segment: from the mean length of a list's part in one position block
    const double mean_seg = (double)v.tokens * a.k / ((double)a.n_feat * l.npb);
    const bool narrow = mean_seg <= 20.0, cmp = v.delta != nullptr;
    auto scatter = cmp ? (narrow ? sc_scatter_lds_kernel<8, true> : sc_scatter_lds_kernel<16, true>)
                       : (narrow ? sc_scatter_lds_kernel<8, false> : sc_scatter_lds_kernel<16, false>);
    if (int rc = s3_allow_lds(once_scatter[2 * cmp + narrow], (const void*)scatter, kMaxPB * 8)) return rc;
    // at most five launches: query weights, gather, sum of the head groups, pooling + tile maxima, Top-B
    hipLaunchKernelGGL(sc_prep_kernel, dim3((unsigned)a.nr, (unsigned)a.n_heads), dim3(kPrepThreads), (size_t)prep_lds, st, a);
    hipLaunchKernelGGL(scatter, dim3((unsigned)a.npb, (unsigned)a.ngroup), dim3(kScatterThreads), (size_t)a.pb * 8, st, a);
    if (a.ngroup > 1) hipLaunchKernelGGL(sc_reduce_kernel, dim3((unsigned)((a.L + 63) / 64)), dim3(256), 0, st, a);
    if (a.len <= kPoolMaxLen) {
        static S3LdsOnce once_pool;
        if (int rc = s3_allow_lds(once_pool, (const void*)sc_pool_kernel, (kTileW + kPoolMaxLen) * 8)) return rc;
        hipLaunchKernelGGL(sc_pool_kernel, dim3((unsigned)a.ntile), dim3(kPoolThreads), (size_t)(kTileW + a.len) * 8, st, a);
    } else {
        hipLaunchKernelGGL(sc_pool_wide_kernel, dim3((unsigned)((a.ntile + 3) / 4)), dim3(256), 0, st, a);
    }
    hipLaunchKernelGGL(sc_topb_kernel, dim3(1), dim3(kTopThreads), 0, st, a);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // namespace

extern "C" size_t s3_coactivate_score_workspace(const s3_index* idx, int64_t n_positions) {
    if (!idx || n_positions < 1) return 0;
    S3IndexView v;
    s3_index_view(idx, &v);
    return layout(v.n_heads, v.n_feat, n_positions).total;
}

extern "C" int s3_coactivate_score(const s3_index* idx, const int32_t* qids, const float* qvals, int nq,
                                   int64_t n_positions, int span_len, int top_b, int32_t max_freq, int nms,
                                   float* scores_out, int32_t* span_start, float* span_score, int32_t* n_found,
                                   void* ws, size_t ws_bytes, void* stream) {
    if (!idx) return s3_fail(S3_EINVAL, "s3_coactivate_score: null pointer");
    S3IndexView v;
    s3_index_view(idx, &v);
    if (!v.finalized) return s3_fail(S3_ESTATE, "s3_coactivate_score: index not finalized");
    ScoreSource src;
    src.n_heads = v.n_heads; src.n_feat = v.n_feat; src.k = v.k; src.tokens = v.tokens; src.sorted = v.sorted;
    src.offsets = v.offsets; src.off_stride = v.off_stride; src.positions = v.positions; src.pos_stride = v.pos_stride;
    src.btab = v.btab_valid ? v.btab : nullptr;
    src.nblk = v.btab_valid ? v.nblk : 1;
    return score_run("s3_coactivate_score", src, qids, qvals, nq, n_positions, span_len, top_b, max_freq, nms, scores_out,
                     span_start, span_score, n_found, ws, ws_bytes, stream);
}

extern "C" size_t s3_coactivate_score_compact_workspace(const s3_cindex* cidx, int64_t n_positions) {
    if (!cidx || n_positions < 1) return 0;
    S3CompactView c;
    s3_cindex_view(cidx, &c);
    return layout(c.n_heads, c.n_feat, n_positions).total;
}

extern "C" int s3_coactivate_score_compact(const s3_cindex* cidx, const int32_t* qids, const float* qvals, int nq,
                                           int64_t n_positions, int span_len, int top_b, int32_t max_freq, int nms,
                                           float* scores_out, int32_t* span_start, float* span_score, int32_t* n_found,
                                           void* ws, size_t ws_bytes, void* stream) {
    if (!cidx) return s3_fail(S3_EINVAL, "s3_coactivate_score_compact: null pointer");
    S3CompactView c;
    s3_cindex_view(cidx, &c);
    ScoreSource src;
    src.n_heads = c.n_heads; src.n_feat = c.n_feat; src.k = c.k; src.tokens = c.tokens; src.sorted = true;
    src.nblk = c.nblk;
    src.delta = c.delta; src.cstart = c.cstart; src.cfreq = c.cfreq; src.delta_stride = c.delta_stride;
    src.cstart_stride = c.cstart_stride;
    return score_run("s3_coactivate_score_compact", src, qids, qvals, nq, n_positions, span_len, top_b, max_freq, nms,
                     scores_out, span_start, span_score, n_found, ws, ws_bytes, stream);
}
