// The rest of Phase 2 and the set operations of Phase 3 (Sec. 3.5 "Adaptive Granularity", Sec. 3.6, Alg. 1):
//
//   s3_select_spans : S' = Conv1D(S) (the semantic density curve), density peaks by greedy non-maximum suppression
//                     (N centres), and a variable-length span around every peak: the positions where the density
//                     stays at or above a fraction of the peak's, up to a largest half length
//   s3_fuse_indices : Idx_final = spans U an index list supplied by the caller (the lexical retriever's) U the first
//                     and last positions (Lead/Tail), as a 0/1 mask and as the ascending list of selected positions
//
// The density is accumulated in fp64 in tap order from the fp32 scores and weights (each product of two fp32 values
// is exact in fp64, so the sum does not depend on whether the compiler fuses the multiply-add) and rounded to fp32
// once; every decision -- which position is a peak, where a span ends -- is taken on those fp32 values, with the
// threshold product formed in fp64.  A CPU reference that follows the same steps reaches the same integers.
#include "s3_common.h"

#include <math.h>

namespace {

constexpr int kConvThreads = 256;
constexpr int kConvPer = 4;
constexpr int kSelTile = kConvThreads * kConvPer;     // positions per tile (conv workgroup, peak search)
constexpr int kMaxTaps = 4096;
constexpr int kNmsThreads = 256;

struct SelArgs {
    const float* scores;
    const float* kernel;
    int64_t L;
    int K, n_centers, radius, max_half;
    float rel;
    float* dens;                 // [L]
    unsigned char* dead;         // [L]
    float* tmaxv;                // [ntile]
    int* tmaxi;                  // [ntile]
    int ntile;
    int32_t* center;
    float* center_density;
    int32_t* span_lo;
    int32_t* span_hi;
    int32_t* n_found;
};

// (value, index) argmax over the block: larger value wins, ties -> smaller index
template <int NT>
__device__ __forceinline__ void block_argmax_f(float& v, int& i, float* sv, int* si) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o);
        const int oi = __shfl_xor(i, o);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sv[wave] = v; si[wave] = i; }
    __syncthreads();
    float bv = sv[0];
    int bi = si[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) {
        const float ov = sv[w];
        const int oi = si[w];
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    v = bv; i = bi;
}

// D[t] = sum_j g[j] * S[t + j - floor(K / 2)] with zeros outside the context; one tile of positions per workgroup,
// its inputs and the weights staged in LDS; also clears the tile's suppression flags and records its best position.
__global__ __launch_bounds__(kConvThreads) void sel_conv_kernel(SelArgs a) {
    extern __shared__ float lds[];
    float* g = lds;                          // [K]
    float* s = lds + a.K;                    // [kSelTile + K - 1]
    __shared__ float sv[kConvThreads / 64];
    __shared__ int si[kConvThreads / 64];
    const int tid = threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.x * kSelTile;
    const int c = a.K / 2;
    for (int j = tid; j < a.K; j += kConvThreads) g[j] = a.kernel[j];
    for (int i = tid; i < kSelTile + a.K - 1; i += kConvThreads) {
        const int64_t u = t0 + i - c;
        s[i] = (u >= 0 && u < a.L) ? a.scores[u] : 0.f;
    }
    __syncthreads();
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
#pragma unroll
    for (int q = 0; q < kConvPer; ++q) {
        const int i = q * kConvThreads + tid;
        const int64_t t = t0 + i;
        if (t < a.L) {
            double acc = 0.0;
            for (int j = 0; j < a.K; ++j) acc += (double)g[j] * (double)s[i + j];
            const float dv = (float)acc;
            a.dens[t] = dv;
            a.dead[t] = 0;
            if (dv > bv) { bv = dv; bi = (int)t; }      // ascending t per thread: the first best one is kept
        }
    }
    block_argmax_f<kConvThreads>(bv, bi, sv, si);
    if (tid == 0) { a.tmaxv[blockIdx.x] = bv; a.tmaxi[blockIdx.x] = bi; }
}

// Greedy peak selection, then the span of every peak.  One workgroup: the rounds depend on each other.
__global__ __launch_bounds__(kNmsThreads) void sel_nms_kernel(SelArgs a) {
    __shared__ float sv[kNmsThreads / 64];
    __shared__ int si[kNmsThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int found = 0;
    for (int r = 0; r < a.n_centers; ++r) {
        float v = -INFINITY;
        int i = 0x7FFFFFFF;
        for (int t = tid; t < a.ntile; t += kNmsThreads) {
            const float tv = a.tmaxv[t];
            const int ti = a.tmaxi[t];
            if (tv > v || (tv == v && ti < i)) { v = tv; i = ti; }
        }
        block_argmax_f<kNmsThreads>(v, i, sv, si);
        if (!(v > 0.f)) break;                       // only positive density makes a centre
        if (tid == 0) {
            a.center[r] = i;
            a.center_density[r] = v;
        }
        found = r + 1;
        const int64_t lo = max((int64_t)0, (int64_t)i - a.radius), hi = min(a.L - 1, (int64_t)i + a.radius);
        for (int64_t t = lo + tid; t <= hi; t += kNmsThreads) a.dead[t] = 1;
        __syncthreads();
        for (int tl = (int)(lo / kSelTile); tl <= (int)(hi / kSelTile); ++tl) {
            float tv = -INFINITY;
            int ti = 0x7FFFFFFF;
            for (int q = tid; q < kSelTile; q += kNmsThreads) {
                const int64_t t = (int64_t)tl * kSelTile + q;
                if (t < a.L && !a.dead[t]) {
                    const float dv = a.dens[t];
                    if (dv > tv) { tv = dv; ti = (int)t; }
                }
            }
            block_argmax_f<kNmsThreads>(tv, ti, sv, si);
            if (tid == 0) { a.tmaxv[tl] = tv; a.tmaxi[tl] = ti; }
        }
        __syncthreads();
    }
    __syncthreads();
    // spans: a wavefront per centre walks outwards 64 positions at a time; the span ends before the first position
    // whose density is below rel * D[centre] or that is farther than max_half from the centre
    for (int r = wave; r < found; r += kNmsThreads / 64) {
        const int c = a.center[r];
        const double thr = (double)a.rel * (double)a.center_density[r];
        int ext[2];
#pragma unroll
        for (int side = 0; side < 2; ++side) {
            const int64_t room = side == 0 ? (int64_t)c : a.L - 1 - c;          // positions available on this side
            const int limit = (int)min((int64_t)a.max_half, room);
            int n = 0;                                                           // positions taken so far
            while (n < limit) {
                const int d = n + 1 + lane;                                      // distance from the centre
                bool ok = false;
                if (d <= limit) {
                    const int64_t t = side == 0 ? (int64_t)c - d : (int64_t)c + d;
                    ok = (double)a.dens[t] >= thr;
                }
                const unsigned long long m = __ballot(ok);
                const int run = m == ~0ull ? 64 : (int)__builtin_ctzll(~m);      // leading positions that pass
                n += run;
                if (run < 64) break;
            }
            ext[side] = min(n, limit);
        }
        if (lane == 0) {
            a.span_lo[r] = c - ext[0];
            a.span_hi[r] = c + ext[1];
        }
    }
    for (int r = found + tid; r < a.n_centers; r += kNmsThreads) {
        a.center[r] = -1; a.center_density[r] = 0.f; a.span_lo[r] = -1; a.span_hi[r] = -1;
    }
    if (tid == 0) a.n_found[0] = found;
}

// ---- Phase 3 set operations ----
constexpr int kFuseBlock = 4096;      // positions per workgroup in the count / compact passes
constexpr int kFuseThreads = 256;

__global__ void fuse_init_kernel(unsigned char* mask, int64_t L, int lead, int tail) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < L; t += (int64_t)gridDim.x * blockDim.x)
        mask[t] = (t < lead || t >= L - tail) ? 1 : 0;
}

// block x < max_spans: span x (if it exists); the other blocks: the caller's index list
__global__ void fuse_mark_kernel(unsigned char* mask, int64_t L, const int32_t* lo, const int32_t* hi, const int32_t* n_spans,
                                 int max_spans, const int32_t* extra, int64_t n_extra) {
    if ((int)blockIdx.x < max_spans) {
        const int ns = n_spans ? min(*n_spans, max_spans) : max_spans;
        if ((int)blockIdx.x >= ns) return;
        const int64_t a = max((int64_t)lo[blockIdx.x], (int64_t)0), b = min((int64_t)hi[blockIdx.x], L - 1);
        for (int64_t t = a + threadIdx.x; t <= b; t += blockDim.x) mask[t] = 1;
    } else {
        const int64_t i = ((int64_t)blockIdx.x - max_spans) * blockDim.x + threadIdx.x;
        if (i < n_extra) {
            const int32_t p = extra[i];
            if (p >= 0 && p < L) mask[p] = 1;
        }
    }
}

__global__ __launch_bounds__(kFuseThreads) void fuse_count_kernel(const unsigned char* mask, int64_t L, int* bsum) {
    __shared__ int wsum[kFuseThreads / 64];
    const int64_t t0 = (int64_t)blockIdx.x * kFuseBlock;
    int c = 0;
    for (int i = threadIdx.x; i < kFuseBlock; i += kFuseThreads) c += (t0 + i < L && mask[t0 + i]) ? 1 : 0;
    int tot;
    s3_block_excl_scan<kFuseThreads>(c, wsum, tot);
    if (threadIdx.x == 0) bsum[blockIdx.x] = tot;
}

// exclusive prefix of the block counts (one workgroup, in place); the total is the number of selected positions
__global__ __launch_bounds__(kFuseThreads) void fuse_scan_kernel(int* bsum, int nblocks, int32_t* n_out) {
    __shared__ int wsum[kFuseThreads / 64];
    int carry = 0;
    for (int b0 = 0; b0 < nblocks; b0 += kFuseThreads) {
        const int b = b0 + threadIdx.x;
        const int v = b < nblocks ? bsum[b] : 0;
        int tot;
        const int ex = s3_block_excl_scan<kFuseThreads>(v, wsum, tot);
        if (b < nblocks) bsum[b] = carry + ex;
        carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) n_out[0] = carry;
}

// thread i of a workgroup owns 16 consecutive positions, so that the output order is the position order
__global__ __launch_bounds__(kFuseThreads) void fuse_compact_kernel(const unsigned char* mask, int64_t L, const int* bsum,
                                                                     int32_t* idx) {
    __shared__ int wsum[kFuseThreads / 64];
    constexpr int kPer = kFuseBlock / kFuseThreads;
    const int64_t t0 = (int64_t)blockIdx.x * kFuseBlock + (int64_t)threadIdx.x * kPer;
    int c = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) c += (t0 + j < L && mask[t0 + j]) ? 1 : 0;
    int tot;
    int o = bsum[blockIdx.x] + s3_block_excl_scan<kFuseThreads>(c, wsum, tot);
#pragma unroll
    for (int j = 0; j < kPer; ++j)
        if (t0 + j < L && mask[t0 + j]) idx[o++] = (int32_t)(t0 + j);
}

struct SelLayout {
    size_t dens, dead, tmaxv, tmaxi, total;
};
SelLayout sel_layout(int64_t L) {
    SelLayout l;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += s3_align(bytes); return at; };
    const size_t ntile = (size_t)(L + kSelTile - 1) / kSelTile;
    l.dens = take((size_t)L * 4);
    l.dead = take((size_t)L);
    l.tmaxv = take(ntile * 4);
    l.tmaxi = take(ntile * 4);
    l.total = o;
    return l;
}

}  // namespace

extern "C" int s3_smoothing_kernel(int kind, int K, float* weights) {
    if (!weights) return s3_fail(S3_EINVAL, "s3_smoothing_kernel: null pointer");
    if (K < 1 || K > kMaxTaps || kind < S3_KERNEL_BOX || kind > S3_KERNEL_GAUSSIAN)
        return s3_fail(S3_EINVAL, "s3_smoothing_kernel: kind %d / K %d (1..%d) out of range", kind, K, kMaxTaps);
    auto shape = [&](int j) {
        if (kind == S3_KERNEL_TRIANGULAR) return (double)(j + 1 < K - j ? j + 1 : K - j);
        if (kind == S3_KERNEL_GAUSSIAN) {
            const double u = ((double)j - 0.5 * (K - 1)) / ((double)K / 6.0);
            return exp(-0.5 * u * u);
        }
        return 1.0;
    };
    double sum = 0.0;
    for (int j = 0; j < K; ++j) sum += shape(j);
    for (int j = 0; j < K; ++j) weights[j] = (float)(shape(j) / sum);
    return S3_OK;
}

extern "C" size_t s3_select_spans_workspace(int64_t n_positions) {
    if (n_positions < 1 || n_positions >= (1LL << 31)) return 0;
    return sel_layout(n_positions).total;
}

extern "C" int s3_select_spans(const float* scores, int64_t n_positions, const float* kernel, int K, int n_centers,
                               int nms_radius, float rel_threshold, int max_half_len, float* density_out,
                               int32_t* center, float* center_density, int32_t* span_lo, int32_t* span_hi,
                               int32_t* n_found, void* ws, size_t ws_bytes, void* stream) {
    if (!scores || !kernel || !center || !center_density || !span_lo || !span_hi || !n_found || !ws)
        return s3_fail(S3_EINVAL, "s3_select_spans: null pointer");
    if (n_positions < 1 || n_positions >= (1LL << 31))
        return s3_fail(S3_EINVAL, "s3_select_spans: n_positions %lld out of range", (long long)n_positions);
    if (K < 1 || K > kMaxTaps) return s3_fail(S3_EINVAL, "s3_select_spans: K %d not in [1, %d]", K, kMaxTaps);
    if (n_centers < 1 || n_centers > 4096 || nms_radius < 0 || max_half_len < 0)
        return s3_fail(S3_EINVAL, "s3_select_spans: n_centers %d (1..4096) / nms_radius %d / max_half_len %d out of range",
                       n_centers, nms_radius, max_half_len);
    if (!(rel_threshold >= 0.f && rel_threshold <= 1.f))
        return s3_fail(S3_EINVAL, "s3_select_spans: rel_threshold %g not in [0, 1]", (double)rel_threshold);
    const SelLayout l = sel_layout(n_positions);
    if (ws_bytes < l.total) return s3_fail(S3_ECAPACITY, "s3_select_spans: workspace %zu < %zu bytes", ws_bytes, l.total);
    if ((uintptr_t)ws & 255) return s3_fail(S3_EINVAL, "s3_select_spans: workspace must be 256-byte aligned");
    char* base = (char*)ws;
    SelArgs a;
    a.scores = scores; a.kernel = kernel; a.L = n_positions; a.K = K; a.n_centers = n_centers; a.radius = nms_radius;
    a.max_half = max_half_len; a.rel = rel_threshold;
    a.dens = density_out ? density_out : (float*)(base + l.dens);
    a.dead = (unsigned char*)(base + l.dead);
    a.tmaxv = (float*)(base + l.tmaxv);
    a.tmaxi = (int*)(base + l.tmaxi);
    a.ntile = (int)((n_positions + kSelTile - 1) / kSelTile);
    a.center = center; a.center_density = center_density; a.span_lo = span_lo; a.span_hi = span_hi; a.n_found = n_found;
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = (size_t)(2 * K - 1 + kSelTile) * 4;      // at most 36 KB: within the default limit
    hipLaunchKernelGGL(sel_conv_kernel, dim3((unsigned)a.ntile), dim3(kConvThreads), lds, st, a);
    hipLaunchKernelGGL(sel_nms_kernel, dim3(1), dim3(kNmsThreads), 0, st, a);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

extern "C" size_t s3_fuse_indices_workspace(int64_t n_positions) {
    if (n_positions < 1 || n_positions >= (1LL << 31)) return 0;
    return s3_align((size_t)((n_positions + kFuseBlock - 1) / kFuseBlock) * 4);
}

extern "C" int s3_fuse_indices(int64_t n_positions, const int32_t* span_lo, const int32_t* span_hi, const int32_t* n_spans,
                               int max_spans, const int32_t* extra, int64_t n_extra, int lead, int tail,
                               unsigned char* mask, int32_t* idx_out, int32_t* n_out, void* ws, size_t ws_bytes,
                               void* stream) {
    if (!mask || !idx_out || !n_out || !ws) return s3_fail(S3_EINVAL, "s3_fuse_indices: null pointer");
    if (n_positions < 1 || n_positions >= (1LL << 31))
        return s3_fail(S3_EINVAL, "s3_fuse_indices: n_positions %lld out of range", (long long)n_positions);
    if (max_spans < 0 || max_spans > 65535 || (max_spans > 0 && (!span_lo || !span_hi)))
        return s3_fail(S3_EINVAL, "s3_fuse_indices: bad span arrays (max_spans %d)", max_spans);
    if (n_extra < 0 || n_extra >= (1LL << 31) || (n_extra > 0 && !extra))
        return s3_fail(S3_EINVAL, "s3_fuse_indices: bad index list (n_extra %lld)", (long long)n_extra);
    if (lead < 0 || tail < 0) return s3_fail(S3_EINVAL, "s3_fuse_indices: lead %d / tail %d negative", lead, tail);
    const size_t need = s3_fuse_indices_workspace(n_positions);
    if (ws_bytes < need) return s3_fail(S3_ECAPACITY, "s3_fuse_indices: workspace %zu < %zu bytes", ws_bytes, need);
    if ((uintptr_t)ws & 255) return s3_fail(S3_EINVAL, "s3_fuse_indices: workspace must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    int* bsum = (int*)ws;
    const int nblocks = (int)((n_positions + kFuseBlock - 1) / kFuseBlock);
    const unsigned gi = (unsigned)((n_positions + 255) / 256 > 4096 ? 4096 : (n_positions + 255) / 256);
    hipLaunchKernelGGL(fuse_init_kernel, dim3(gi), dim3(256), 0, st, mask, n_positions, lead, tail);
    const unsigned gm = (unsigned)max_spans + (unsigned)((n_extra + 255) / 256);
    if (gm)
        hipLaunchKernelGGL(fuse_mark_kernel, dim3(gm), dim3(256), 0, st, mask, n_positions, span_lo, span_hi, n_spans,
                           max_spans, extra, n_extra);
    hipLaunchKernelGGL(fuse_count_kernel, dim3((unsigned)nblocks), dim3(kFuseThreads), 0, st, mask, n_positions, bsum);
    hipLaunchKernelGGL(fuse_scan_kernel, dim3(1), dim3(kFuseThreads), 0, st, bsum, nblocks, n_out);
    hipLaunchKernelGGL(fuse_compact_kernel, dim3((unsigned)nblocks), dim3(kFuseThreads), 0, st, mask, n_positions, bsum,
                       idx_out);
    S3_HIP(hipGetLastError());
    return S3_OK;
}
