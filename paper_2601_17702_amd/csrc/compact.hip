// Compact form of a finalized inverted index (Sec. 3.4 "CPU Index Size": contiguous integer arrays with delta
// encoding and optional stop-feature pruning), built for the way the scoring kernel reads postings:
//
//   - positions are cut into the scoring kernel's blocks of 2^14; a posting is stored as the 16-bit offset from the
//     start of its block (the delta against the block base): 2 bytes instead of 4, decodable by every lane on its own;
//   - the postings are ordered block by block, inside a block list by list (ascending feature id): everything a
//     scoring workgroup reads for its block is one contiguous run of memory instead of one short piece per list;
//   - cstart [nblk * n_feat + 1] says where the segment of (block b, feature f) starts (the skip table);
//     cfreq [n_feat] keeps each list's length for the IDF weight;
//   - a list longer than prune_freq (a stop feature) is dropped whole when prune_freq > 0.
//
// Built from the plain index's CSR and block table into a buffer the caller owns, so the plain index can be destroyed
// afterwards and its memory returned.
#include "s3_common.h"

#include <new>

struct s3_cindex {
    S3CompactView v;
};

void s3_cindex_view(const s3_cindex* cidx, S3CompactView* out) { *out = cidx->v; }

namespace {

constexpr int kScanChunk = 4096;      // entries per workgroup in the prefix-sum passes (256 threads x 16)
constexpr int kScanThreads = 256;

struct CmpArgs {
    const int32_t* offsets;
    const int32_t* positions;
    const int32_t* btab;          // null: one block
    int64_t off_stride, pos_stride;
    int n_heads, n_feat, nblk;
    int32_t prune_freq;
    int32_t* cstart;
    int32_t* cfreq;
    uint16_t* delta;
    int64_t cstart_stride, delta_stride;
    int32_t* bsum;                // [n_heads][nchunks + 1]
    int nchunks;
};

// where list f's part in block b begins and ends in the head's positions array
__device__ __forceinline__ void segment(const CmpArgs& a, const int32_t* off, const int32_t* tab, int f, int b, int& lo, int& hi) {
    const int nbk = a.nblk - 1, lb = off[f], le = off[f + 1];
    lo = b == 0 ? lb : tab[(size_t)f * nbk + b - 1];
    hi = b < nbk ? tab[(size_t)f * nbk + b] : le;
    lo = min(max(lo, lb), le);    // whatever the table holds, nothing outside the list is read
    hi = min(max(hi, lo), le);
}

// cstart[b * n_feat + f] = length of segment (b, f), 0 for a dropped list; cfreq[f] = length of the kept list
__global__ __launch_bounds__(256) void cmp_count_kernel(CmpArgs a) {
    const int h = blockIdx.z, b = blockIdx.y, f = blockIdx.x * 256 + threadIdx.x;
    if (f >= a.n_feat) return;
    const int32_t* off = a.offsets + (size_t)h * a.off_stride;
    const int32_t* tab = a.btab ? a.btab + (size_t)h * a.n_feat * (a.nblk - 1) : nullptr;
    const int len = off[f + 1] - off[f];
    const bool keep = !(a.prune_freq > 0 && len > a.prune_freq);
    int lo, hi;
    segment(a, off, tab, f, b, lo, hi);
    a.cstart[(size_t)h * a.cstart_stride + (size_t)b * a.n_feat + f] = keep ? hi - lo : 0;
    if (b == 0) a.cfreq[(size_t)h * a.n_feat + f] = keep ? len : 0;
}

// exclusive prefix sum of the nblk * n_feat counts of every head, in place, total behind the last one: chunk sums,
// scan of the chunk sums (one workgroup per head), chunk-local scan plus the chunk's base
__global__ __launch_bounds__(kScanThreads) void cmp_chunk_sum_kernel(CmpArgs a) {
    __shared__ int wsum[kScanThreads / 64];
    const int h = blockIdx.y;
    const int64_t n = (int64_t)a.nblk * a.n_feat, i0 = (int64_t)blockIdx.x * kScanChunk;
    const int32_t* c = a.cstart + (size_t)h * a.cstart_stride;
    int s = 0;
    for (int i = threadIdx.x; i < kScanChunk; i += kScanThreads) s += i0 + i < n ? c[i0 + i] : 0;
    int tot;
    s3_block_excl_scan<kScanThreads>(s, wsum, tot);
    if (threadIdx.x == 0) a.bsum[(size_t)h * (a.nchunks + 1) + blockIdx.x] = tot;
}

__global__ __launch_bounds__(kScanThreads) void cmp_scan_sums_kernel(CmpArgs a) {
    __shared__ int wsum[kScanThreads / 64];
    int32_t* bs = a.bsum + (size_t)blockIdx.x * (a.nchunks + 1);
    int carry = 0;
    for (int b0 = 0; b0 < a.nchunks; b0 += kScanThreads) {
        const int b = b0 + threadIdx.x;
        const int v = b < a.nchunks ? bs[b] : 0;
        int tot;
        const int ex = s3_block_excl_scan<kScanThreads>(v, wsum, tot);
        if (b < a.nchunks) bs[b] = carry + ex;
        carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        bs[a.nchunks] = carry;
        a.cstart[(size_t)blockIdx.x * a.cstart_stride + (size_t)a.nblk * a.n_feat] = carry;      // end of the last segment
    }
}

__global__ __launch_bounds__(kScanThreads) void cmp_chunk_scan_kernel(CmpArgs a) {
    __shared__ int wsum[kScanThreads / 64];
    constexpr int kPer = kScanChunk / kScanThreads;
    const int h = blockIdx.y;
    const int64_t n = (int64_t)a.nblk * a.n_feat, i0 = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kPer;
    int32_t* c = a.cstart + (size_t)h * a.cstart_stride;
    int v[kPer], s = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        v[j] = i0 + j < n ? c[i0 + j] : 0;
        s += v[j];
    }
    int tot;
    int run = a.bsum[(size_t)h * (a.nchunks + 1) + blockIdx.x] + s3_block_excl_scan<kScanThreads>(s, wsum, tot);
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        if (i0 + j < n) c[i0 + j] = run;
        run += v[j];
    }
}

// Copies the segments of (head, block, 256 consecutive features): a wavefront takes 64 features, finds each one's
// source and destination, and copies one segment after the other, lanes over postings.
__global__ __launch_bounds__(256) void cmp_copy_kernel(CmpArgs a) {
    const int h = blockIdx.z, b = blockIdx.y, lane = threadIdx.x & 63;
    const int f = blockIdx.x * 256 + threadIdx.x;
    const int32_t* off = a.offsets + (size_t)h * a.off_stride;
    const int32_t* tab = a.btab ? a.btab + (size_t)h * a.n_feat * (a.nblk - 1) : nullptr;
    const int32_t* pos = a.positions + (size_t)h * a.pos_stride;
    const int32_t* cs = a.cstart + (size_t)h * a.cstart_stride + (size_t)b * a.n_feat;
    uint16_t* out = a.delta + (size_t)h * a.delta_stride;
    int src = 0, dst = 0, n = 0;
    if (f < a.n_feat) {
        dst = cs[f];
        n = cs[f + 1] - dst;                   // 0 for a dropped list
        if (n > 0) {
            int hi;
            segment(a, off, tab, f, b, src, hi);
            n = min(n, hi - src);
        }
    }
    const int base = b << kS3PosBlockLog2;
    unsigned long long m = __ballot(n > 0);
    while (m) {
        const int l = (int)__builtin_ctzll(m);
        m &= m - 1;
        const int ssrc = __builtin_amdgcn_readlane(src, l), sdst = __builtin_amdgcn_readlane(dst, l);
        const int sn = __builtin_amdgcn_readlane(n, l);
        for (int q = lane; q < sn; q += 64) out[sdst + q] = (uint16_t)(pos[ssrc + q] - base);
    }
}

}  // namespace

extern "C" {

size_t s3_index_compact_bytes(const s3_index* idx) {
    if (!idx) return 0;
    S3IndexView v;
    s3_index_view(idx, &v);
    const int nblk = v.nblk ? v.nblk : 1;
    const int64_t cs = (int64_t)nblk * v.n_feat + 1;
    const int nchunks = (int)((cs - 1 + kScanChunk - 1) / kScanChunk);
    return s3_align((size_t)v.n_heads * cs * 4) + s3_align((size_t)v.n_heads * v.n_feat * 4) +
           s3_align((size_t)v.n_heads * (size_t)(v.tokens * v.k) * 2) + s3_align((size_t)v.n_heads * (nchunks + 1) * 4);
}

int s3_index_compact(const s3_index* idx, int32_t prune_freq, void* buf, size_t buf_bytes, s3_cindex** out, void* stream) {
    if (!idx || !out || !buf) return s3_fail(S3_EINVAL, "s3_index_compact: null pointer");
    if (prune_freq < 0) return s3_fail(S3_EINVAL, "s3_index_compact: prune_freq %d negative", (int)prune_freq);
    if ((uintptr_t)buf & 255) return s3_fail(S3_EINVAL, "s3_index_compact: buffer must be 256-byte aligned");
    S3IndexView v;
    s3_index_view(idx, &v);
    if (!v.finalized) return s3_fail(S3_ESTATE, "s3_index_compact: index not finalized");
    // one block needs no table; more blocks need the block table, which holds for lists that ascend in position
    // (implicit, increasing positions) and lie inside the blocks the index was created for
    const bool one_block = v.sorted && v.max_pos < (1LL << kS3PosBlockLog2);
    if (!one_block && !v.btab_valid)
        return s3_fail(S3_ESTATE, "s3_index_compact: needs implicit increasing positions below %lld (%d blocks of %d)",
                       (long long)kS3MaxTableBlocks << kS3PosBlockLog2, kS3MaxTableBlocks, 1 << kS3PosBlockLog2);
    const size_t need = s3_index_compact_bytes(idx);
    if (buf_bytes < need) return s3_fail(S3_ECAPACITY, "s3_index_compact: buffer %zu < %zu bytes", buf_bytes, need);
    s3_cindex* c = new (std::nothrow) s3_cindex();
    if (!c) return s3_fail(S3_EHIP, "s3_index_compact: out of host memory");
    CmpArgs a;
    a.offsets = v.offsets; a.positions = v.positions; a.off_stride = v.off_stride; a.pos_stride = v.pos_stride;
    a.nblk = one_block ? 1 : v.nblk;
    a.btab = one_block ? nullptr : v.btab;
    a.n_heads = v.n_heads; a.n_feat = v.n_feat; a.prune_freq = prune_freq;
    const int64_t cs = (int64_t)(v.nblk ? v.nblk : 1) * v.n_feat + 1;      // stride as sized by s3_index_compact_bytes
    const int64_t used = (int64_t)a.nblk * v.n_feat;
    a.nchunks = (int)((used + kScanChunk - 1) / kScanChunk);
    char* base = (char*)buf;
    size_t o = 0;
    auto take = [&](size_t bytes) { char* at = base + o; o += s3_align(bytes); return at; };
    a.cstart = (int32_t*)take((size_t)v.n_heads * cs * 4);
    a.cfreq = (int32_t*)take((size_t)v.n_heads * v.n_feat * 4);
    a.delta = (uint16_t*)take((size_t)v.n_heads * (size_t)(v.tokens * v.k) * 2);
    a.bsum = (int32_t*)take((size_t)v.n_heads * (a.nchunks + 1) * 4);
    a.cstart_stride = cs; a.delta_stride = v.tokens * v.k;
    hipStream_t st = (hipStream_t)stream;
    const dim3 gf((unsigned)((v.n_feat + 255) / 256), (unsigned)a.nblk, (unsigned)v.n_heads);
    hipLaunchKernelGGL(cmp_count_kernel, gf, dim3(256), 0, st, a);
    hipLaunchKernelGGL(cmp_chunk_sum_kernel, dim3((unsigned)a.nchunks, (unsigned)v.n_heads), dim3(kScanThreads), 0, st, a);
    hipLaunchKernelGGL(cmp_scan_sums_kernel, dim3((unsigned)v.n_heads), dim3(kScanThreads), 0, st, a);
    hipLaunchKernelGGL(cmp_chunk_scan_kernel, dim3((unsigned)a.nchunks, (unsigned)v.n_heads), dim3(kScanThreads), 0, st, a);
    hipLaunchKernelGGL(cmp_copy_kernel, gf, dim3(256), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        delete c;
        return s3_fail(S3_EHIP, "s3_index_compact: launch failed: %s", hipGetErrorString(e));
    }
    c->v.n_heads = v.n_heads; c->v.n_feat = v.n_feat; c->v.k = v.k; c->v.nblk = a.nblk; c->v.tokens = v.tokens;
    c->v.cstart = a.cstart; c->v.delta = a.delta; c->v.cfreq = a.cfreq;
    c->v.cstart_stride = a.cstart_stride; c->v.delta_stride = a.delta_stride;
    *out = c;
    return S3_OK;
}

void s3_cindex_destroy(s3_cindex* cidx) { delete cidx; }

int s3_cindex_info(const s3_cindex* cidx, int* n_blocks, int64_t* max_postings) {
    if (!cidx || !n_blocks || !max_postings) return s3_fail(S3_EINVAL, "s3_cindex_info: null pointer");
    *n_blocks = cidx->v.nblk;
    *max_postings = cidx->v.delta_stride;
    return S3_OK;
}

int s3_cindex_export(const s3_cindex* cidx, int head, int32_t* cstart_out, uint16_t* delta_out, int32_t* cfreq_out,
                     void* stream) {
    if (!cidx) return s3_fail(S3_EINVAL, "s3_cindex_export: null pointer");
    const S3CompactView& v = cidx->v;
    if (head < 0 || head >= v.n_heads) return s3_fail(S3_EINVAL, "s3_cindex_export: head %d out of range", head);
    hipStream_t st = (hipStream_t)stream;
    if (cstart_out)
        S3_HIP(hipMemcpyAsync(cstart_out, v.cstart + (size_t)head * v.cstart_stride, ((size_t)v.nblk * v.n_feat + 1) * 4,
                              hipMemcpyDeviceToDevice, st));
    if (delta_out && v.delta_stride)
        S3_HIP(hipMemcpyAsync(delta_out, v.delta + (size_t)head * v.delta_stride, (size_t)v.delta_stride * 2,
                              hipMemcpyDeviceToDevice, st));
    if (cfreq_out)
        S3_HIP(hipMemcpyAsync(cfreq_out, v.cfreq + (size_t)head * v.n_feat, (size_t)v.n_feat * 4, hipMemcpyDeviceToDevice, st));
    return S3_OK;
}

}  // extern "C"
