// Inverted index build on the GPU (Sec. 3.4: I[f] <- I[f] U {t}; contiguous CSR layout of
// Sec. 3.4 "CPU Index Size").
//
// A direct counting-sort scatter of (feature -> position) writes 4 bytes to one of n_feat
// places per posting: nothing coalesces.  The build is therefore a two-level (most-significant
// digit first) stable counting sort whose every global write is a contiguous run:
//
//   append   : each tile of <= 8192 postings (<= 8192/k tokens of one head) is split in LDS by
//              the feature's coarse bucket (f >> S, at most 256 buckets) and written out as one
//              contiguous tile of packed (row << S | f & mask) words, plus a small table of
//              (offset, count) per (bucket, tile).  The order inside a bucket stays the append
//              order (stable), so positions inside a posting list come out ascending.
//   finalize : per (head, bucket) the pieces of all tiles are gathered in tile order, split in
//              LDS by the low feature bits (stable again) and written to their final place in the
//              CSR; the per-feature counts of the bucket give offsets[].
//
// The bucket pass is one pass of a ballot-based multi-way split: the lanes of a wavefront that hold the same
// digit find each other with one ballot per digit bit, per-wavefront counters and one block-wide prefix sum
// give every entry its rank.  The append pass ranks with one returning LDS add per token row instead (a token's
// ids are distinct, so the entries of one feature are always in different rows and keep their order); for very
// small k it uses the ballots too.
//
// The order of the entries of ONE feature is fixed by prefix sums over lane, row and wavefront orders: the CSR is
// bit-identical from run to run and independent of how the stream was chunked.  (Inside a tile of the intermediate
// array, entries of different features that share a bucket and a token may come in either order.)
#include "s3_common.h"

#include <new>

namespace {

constexpr int kTilePost = 8192;       // postings per partition tile (upper bound)
constexpr int kSortCap = 8192;        // entries split per round in the bucket pass

struct IdxDev {
    uint32_t* inter;      // [n_heads][max_tiles * tile_post] packed (row << S | f_lo), bucket-sorted per tile
    uint32_t* piece;      // [n_heads][NB][max_tiles]  (offset_in_tile << 16 | count)
    int32_t* total;       // [n_heads][NB]
    int32_t* bbase;       // [n_heads][NB + 1]
    int32_t* offsets;     // [n_heads][n_feat + 1]  (stride off_stride)
    int32_t* positions;   // [n_heads][pos_stride]
    const int32_t* pos_log;   // [max_tokens] absolute position of each appended row (read unless pos_affine)
    int32_t* btab;            // [n_heads][n_feat][nblk - 1] block table for scoring, or null
    int64_t inter_stride, piece_stride, off_stride, pos_stride;
    int n_feat, k, S, NB, nbB, ptok, tile_post, max_tiles;
    int w16;                  // intermediate entries are 16 bits: (row inside the tile) << S | f & mask (else 32 bits, row of the stream)
    int nblk;                 // position blocks the table covers
    int pos_affine;           // position of row r is pos0 + r (every append used contiguous implicit positions)
    int32_t pos0;
    uint32_t kinv;        // ceil(2^32 / k) for k > 1: i / k == umulhi(i, kinv) for every posting index of a tile
};

// Stable multi-way split of up to kSplitWaves * kSplitRounds * 64 keyed entries by a digit of at most 8 bits.
// Wavefront w owns the entries [w seg, (w + 1) seg) in rounds of 64 (lane order = entry order).
//   count   : split_round() per round: the lanes that share a digit find each other with one ballot per digit bit;
//             the first of them adds their number to the wavefront's own counter row (one writer per counter and
//             instruction, so nothing depends on an ordering of atomics), every lane reads the counter back and so
//             knows its rank among the wavefront's entries of that digit, this round and the earlier ones
//   scan    : split_scan(): exclusive prefix over (digit major, wavefront minor) turns the counters into bases
//   rank    : split_rank(): base of (wavefront, digit) + rank inside the wavefront
constexpr int kSplitThreads = 1024;
constexpr int kSplitWaves = kSplitThreads / 64;
constexpr int kSplitRounds = 8;          // 16 wavefronts x 8 rounds x 64 lanes = 8192 entries per pass
constexpr int kSplitOcc = 8;             // wavefronts per SIMD the kernels are built for: two workgroups per compute unit
constexpr unsigned kSplitValid = 1u << 31;
constexpr int kRowAtomicMinK = 8;        // Top-k sizes from which the append ranks a round row by row (at most 9 rows)

// One round for this lane's entry with digit `dg` (low NBITS bits, the rest 0; 0 on an invalid lane).  Returns
// dg | rank inside the wavefront << 8 | kSplitValid, or 0 for an invalid lane.
template <int NBITS>
__device__ __forceinline__ unsigned split_round(int* cnt_row, unsigned dg, bool valid) {
    const unsigned long long v = __ballot(valid);
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
#pragma unroll
    for (int bit = 0; bit < NBITS; ++bit) {
        int m = (int)(dg << (31 - bit)) >> 31;                  // all ones when the bit is set
        asm volatile("" : "+v"(m));                             // one bit-field extract serves the ballot and the select
        const unsigned long long b = __ballot(m != 0);
        // keep the lanes whose bit equals mine: x & ~(b ^ m) as one three-input bit operation (table 0x90)
        lo = __builtin_amdgcn_bitop3_b32(lo, (unsigned)b, (unsigned)m, 0x90);
        hi = __builtin_amdgcn_bitop3_b32(hi, (unsigned)(b >> 32), (unsigned)m, 0x90);
    }
    const unsigned before = __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));   // equal digits in lower lanes
    const unsigned total = (unsigned)(__popc(lo) + __popc(hi));                                  // equal digits in the round
    unsigned res = 0u;
    if (valid) {
        if (before == 0) atomicAdd(&cnt_row[dg], (int)total);
        // the wavefront's LDS accesses execute in program order: this read sees the group's add
        const unsigned after = (unsigned)cnt_row[dg];
        res = dg | ((after - total + before) << 8) | kSplitValid;
    }
    return res;
}

__device__ __forceinline__ int split_rank(const int* cnt_row, unsigned m) {
    return cnt_row[m & 0xFFu] + (int)((m >> 8) & 0x3FFFu);
}

// cnt: [kSplitWaves][nd] counts -> running bases; dstart[d] / dcount[d]: first rank and number of entries of digit d
__device__ __forceinline__ void split_scan(int* cnt, int nd, int* dstart, int* dcount, int* wsum) {
    const int tid = threadIdx.x;
    constexpr int per = kSplitWaves * 256 / kSplitThreads;     // 4 entries per thread when nd = 256
    // entry e = d * kSplitWaves + w; thread t owns e = per t .. per t + per - 1 (one digit: per divides kSplitWaves)
    const int d = tid * per / kSplitWaves, w0 = tid * per % kSplitWaves;
    int v[per], s = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {
        v[j] = d < nd ? cnt[(w0 + j) * nd + d] : 0;
        s += v[j];
    }
    int tot;
    int ex = s3_block_excl_scan<kSplitThreads>(s, wsum, tot);
    if (d < nd) {
        int run = ex;
#pragma unroll
        for (int j = 0; j < per; ++j) {
            cnt[(w0 + j) * nd + d] = run;
            run += v[j];
        }
    }
    // the kSplitWaves / per threads of a digit are adjacent lanes: their sum is the digit's count
    static_assert(kSplitWaves / per == 2 || kSplitWaves / per == 4, "a digit's threads are an aligned group of 2 or 4 lanes");
    int dc = s;
    dc += __builtin_amdgcn_update_dpp(0, dc, 0xB1, 0xf, 0xf, false);     // lanes 1 0 3 2 of each group of four
    if (kSplitWaves / per == 4) dc += __builtin_amdgcn_update_dpp(0, dc, 0x4E, 0xf, 0xf, false);     // lanes 2 3 0 1
    if (d < nd && w0 == 0) { dstart[d] = ex; dcount[d] = dc; }
    __syncthreads();
}

// One tile of <= tile_post postings of one head: split by bucket, write the tile and its piece table.
// `src` is the first row of tile `tile0` (row stride k, head stride head_stride elements).
__global__ __launch_bounds__(kSplitThreads, kSplitOcc) void idx_partition_kernel(const int32_t* src, int64_t head_stride,
                                                                         int rows_avail, int tile0, IdxDev d) {
    __shared__ int cnt[kSplitWaves * 256];
    __shared__ uint32_t stage[kTilePost];
    __shared__ int wsum[kSplitWaves];
    __shared__ int bstart[256], bcount[256];

    const int tid = threadIdx.x, lane = tid & 63, head = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = tile0 + blockIdx.x;
    const int nrows = min(d.ptok, rows_avail - (int)blockIdx.x * d.ptok);
    const int n = nrows * d.k;
    const int32_t* s = src + (size_t)head * head_stride + (size_t)blockIdx.x * d.ptok * d.k;
    const uint32_t mask = (1u << d.S) - 1u;
    const uint32_t row0 = (uint32_t)tile * (uint32_t)d.ptok;
    const int nd = 1 << d.nbB;

    int* row = cnt + wave * nd;
    uint32_t word[kSplitRounds];
    unsigned meta[kSplitRounds];       // split_round()
    const int i0 = wave * (kSplitRounds * 64) + lane;
    if (i0 - lane + kSplitRounds * 64 <= n) {      // uniform: the wavefront's whole share exists
#pragma unroll
        for (int r = 0; r < kSplitRounds; ++r) word[r] = (uint32_t)s[i0 + r * 64];
    } else {                                       // ragged tail: read a clamped index, drop it below
#pragma unroll
        for (int r = 0; r < kSplitRounds; ++r) word[r] = (uint32_t)s[min(i0 + r * 64, n - 1)];
    }
    for (int i = tid; i < kSplitWaves * nd; i += kSplitThreads) cnt[i] = 0;      // while the loads are in flight
    __syncthreads();
    const uint32_t k_is_1 = d.k == 1;
#pragma unroll
    for (int r = 0; r < kSplitRounds; ++r) {
        const uint32_t i = (uint32_t)(i0 + r * 64);
        const bool valid = (int)i < n;
        const uint32_t id = valid ? word[r] : 0u;
        const uint32_t dg = min(id >> d.S, (uint32_t)(nd - 1));   // ids are < n_feat by contract; never index past the counters
        const uint32_t trow = __umulhi(i, d.kinv) + i * k_is_1;   // i / k (kinv is 0 when k == 1)
        word[r] = (((d.w16 ? 0u : row0) + trow) << d.S) | (id & mask);
        if (d.k >= kRowAtomicMinK) {
            // A token's ids are distinct, so entries of one feature never share a row: one returning LDS add per row
            // of the round (in row order; a wavefront's LDS operations execute in program order) ranks every entry
            // behind the earlier entries of its bucket in this wavefront.  Entries of different features in one
            // row get their ranks in any order, which no posting list can see.
            const uint32_t first = __builtin_amdgcn_readfirstlane(__umulhi(i - lane, d.kinv));
            const uint32_t last = __builtin_amdgcn_readfirstlane(__umulhi(i - lane + 63u, d.kinv));
            unsigned res = 0u;
            for (uint32_t rr = first; rr <= last; ++rr)
                if (valid && trow == rr) res = dg | ((unsigned)atomicAdd(&row[dg], 1) << 8) | kSplitValid;
            meta[r] = res;
        } else {
            meta[r] = split_round<8>(row, dg, valid);
        }
    }
    __syncthreads();
    split_scan(cnt, nd, bstart, bcount, wsum);
#pragma unroll
    for (int r = 0; r < kSplitRounds; ++r) {
        if (meta[r] & kSplitValid) stage[split_rank(row, meta[r])] = word[r];
    }
    __syncthreads();
    const size_t at = (size_t)head * d.inter_stride + (size_t)tile * d.tile_post;
    if (d.w16) {
        uint16_t* out = (uint16_t*)d.inter + at;
        for (int i = tid; i < n; i += kSplitThreads) out[i] = (uint16_t)stage[i];
    } else {
        uint32_t* out = d.inter + at;
        for (int i = tid; i < n; i += kSplitThreads) out[i] = stage[i];
    }
    uint32_t* pc = d.piece + (size_t)head * d.piece_stride;
    for (int b = tid; b < d.NB; b += kSplitThreads)
        pc[(size_t)b * d.max_tiles + tile] = ((uint32_t)bstart[b] << 16) | (uint32_t)bcount[b];
}

__global__ __launch_bounds__(256) void idx_totals_kernel(IdxDev d, int n_tiles) {
    __shared__ int wsum[4];
    const int b = blockIdx.x, head = blockIdx.y;
    const uint32_t* pc = d.piece + (size_t)head * d.piece_stride + (size_t)b * d.max_tiles;
    int acc = 0;
    for (int t = threadIdx.x; t < n_tiles; t += 256) acc += (int)(pc[t] & 0xFFFFu);
    int tot;
    s3_block_excl_scan<256>(acc, wsum, tot);
    if (threadIdx.x == 0) d.total[(size_t)head * d.NB + b] = tot;
}

__global__ __launch_bounds__(256) void idx_bucket_scan_kernel(IdxDev d) {
    __shared__ int wsum[4];
    const int head = blockIdx.x, b = threadIdx.x;
    int v = b < d.NB ? d.total[(size_t)head * d.NB + b] : 0;
    int tot;
    int ex = s3_block_excl_scan<256>(v, wsum, tot);
    int32_t* bb = d.bbase + (size_t)head * (d.NB + 1);
    if (b < d.NB) bb[b] = ex;
    if (b == 0) {
        bb[d.NB] = tot;
        d.offsets[(size_t)head * d.off_stride + d.n_feat] = tot;
    }
}

// One (head, bucket): gather its pieces in tile order, split by the low feature bits, write the CSR.
// A bucket of at most kSortCap postings (the usual case) is done in one round: its sorted positions are
// staged in LDS and written as one contiguous run.  A larger bucket (a very frequent feature) is counted
// first and then taken in rounds of whole pieces, each round writing behind per-feature cursors.
template <int NBITS>
__global__ __launch_bounds__(kSplitThreads, kSplitOcc) void idx_bucket_sort_kernel(IdxDev d, int n_tiles) {
    extern __shared__ __align__(16) uint32_t dyn[];
    uint32_t* bufa = dyn;                          // [kSortCap] gathered entries of the round; once every wavefront
    int32_t* bufb = (int32_t*)dyn;                 // holds its entries in registers: the sorted positions (same memory)
    int* pref = (int*)(dyn + kSortCap);            // [kSplitThreads + 1]
    uint32_t* pinfo = (uint32_t*)(pref + kSplitThreads + 1);   // [kSplitThreads] piece words of the round
    int* wsum = (int*)(pinfo + kSplitThreads);     // [16]
    int* hist = wsum + 16;                         // [256] whole-bucket counts (before the first round only)
    int* rcount = hist;                            //       per-round counts afterwards
    int* cursor = hist + 256;                      // [256]
    int* rstart = cursor + 256;                    // [256]
    int* lstart = rstart + 256;                    // [256] where each list starts in the head's positions array
    int* nextj = lstart + 256;                     // [256] first block whose start in the list is not known yet
    int* cnt = nextj + 256;                        // [kSplitWaves << S]

    const int tid = threadIdx.x, lane = tid & 63, head = blockIdx.y;
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  The pieces of adjacent buckets are
    // adjacent in memory and share cache lines, so adjacent buckets go to the SAME XCD one after the other: the
    // second touch of a line then hits that L2 (it halves the bytes fetched; the time does not change).
    const int b = (d.NB & 7) == 0 ? (int)(blockIdx.x & 7) * (d.NB >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the first round's piece words are requested together with the bucket's totals: one memory latency, not two
    const uint32_t* pc = d.piece + (size_t)head * d.piece_stride + (size_t)b * d.max_tiles;
    uint32_t p_next = tid < n_tiles ? pc[tid] : 0u;
    const int n_b = d.total[(size_t)head * d.NB + b];
    const int out_base = d.bbase[(size_t)head * (d.NB + 1) + b];
    const int nd = 1 << d.S;
    const int nfl = min(nd, d.n_feat - (b << d.S));
    const uint32_t mask = (1u << d.S) - 1u;
    int32_t* offs = d.offsets + (size_t)head * d.off_stride + ((size_t)b << d.S);
    const int nbk = d.btab ? d.nblk - 1 : 0;      // block-table entries per list
    int32_t* tab = d.btab ? d.btab + ((size_t)head * d.n_feat + ((size_t)b << d.S)) * nbk : nullptr;
    if (n_b == 0) {
        if (tid < nfl) {
            offs[tid] = out_base;
            for (int j = 0; j < nbk; ++j) tab[tid * nbk + j] = out_base;
        }
        return;
    }
    // entry i of the head's intermediate array (16-bit entries carry the row inside their tile: the caller adds the tile's first row)
    const uint16_t* inter16 = (const uint16_t*)d.inter + (size_t)head * d.inter_stride;
    int32_t* posout = d.positions + (size_t)head * d.pos_stride;
    const bool multi = n_b > kSortCap || n_tiles > kSplitThreads;   // more than one round of pieces

    if (tid < 256) nextj[tid] = 1;
    if (multi) {   // count the whole bucket first: the CSR offsets are needed before the first round is written
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int t = wave; t < n_tiles; t += kSplitWaves) {
            uint32_t p = pc[t];
            int c = (int)(p & 0xFFFFu);
            const size_t e0 = (size_t)t * d.tile_post + (p >> 16);
            if (d.w16) {
                for (int i = lane; i < c; i += 64) atomicAdd(&hist[inter16[e0 + i] & mask], 1);
            } else {
                for (int i = lane; i < c; i += 64) atomicAdd(&hist[d.inter[(size_t)head * d.inter_stride + e0 + i] & mask], 1);
            }
        }
        __syncthreads();
        int tot;
        int ex = s3_block_excl_scan<kSplitThreads>(tid < nd ? hist[tid] : 0, wsum, tot);
        if (tid < nd) cursor[tid] = lstart[tid] = out_base + ex;
        if (tid < nfl) offs[tid] = out_base + ex;
        __syncthreads();
    }

    for (int tp = 0; tp < n_tiles;) {
        // take as many whole pieces (in tile order) as fit in one round; thread t looks at piece tp + t
        const uint32_t p = p_next;
        const int c = (int)(p & 0xFFFFu);
        int tot;
        const int ex = s3_block_excl_scan<kSplitThreads>(c, wsum, tot);
        pref[tid] = ex;
        pinfo[tid] = p;
        if (tid == kSplitThreads - 1) pref[kSplitThreads] = tot;
        int m = __syncthreads_count(ex + c <= kSortCap);    // prefix property: the first m threads qualify
        m = min(m, n_tiles - tp);
        const int n_r = pref[m];
        // gather: a half wavefront copies one piece, four pieces per step
        {
            const int hw = tid >> 5, l0 = tid & 31;
            for (int j0 = hw; j0 < m; j0 += 4 * (kSplitThreads / 32)) {
                size_t sp[4];                      // first entry of the piece in the head's intermediate array
                int dst[4], cc[4];
                uint32_t v[4], v2[4], add[4];      // add: what turns a 16-bit entry into the 32-bit form (its tile's first row)
                const uint32_t* in32 = d.inter + (size_t)head * d.inter_stride;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = j0 + q * (kSplitThreads / 32);
                    const uint32_t pj = j < m ? pinfo[j] : 0u;
                    const int tile = tp + (j < m ? j : 0);
                    cc[q] = (int)(pj & 0xFFFFu);
                    dst[q] = j < m ? pref[j] : 0;
                    sp[q] = (size_t)tile * d.tile_post + (pj >> 16);
                    add[q] = d.w16 ? ((uint32_t)tile * (uint32_t)d.ptok) << d.S : 0u;
                }
                if (d.w16) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {  // the first 64 entries of each piece: eight loads in flight
                        v[q] = l0 < cc[q] ? inter16[sp[q] + l0] : 0u;
                        v2[q] = l0 + 32 < cc[q] ? inter16[sp[q] + l0 + 32] : 0u;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        v[q] = l0 < cc[q] ? in32[sp[q] + l0] : 0u;
                        v2[q] = l0 + 32 < cc[q] ? in32[sp[q] + l0 + 32] : 0u;
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (l0 < cc[q]) bufa[dst[q] + l0] = v[q] + add[q];
                    if (l0 + 32 < cc[q]) bufa[dst[q] + l0 + 32] = v2[q] + add[q];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    for (int l = l0 + 64; l < cc[q]; l += 32)
                        bufa[dst[q] + l] = (d.w16 ? (uint32_t)inter16[sp[q] + l] : in32[sp[q] + l]) + add[q];
            }
        }
        for (int i = tid; i < kSplitWaves * nd; i += kSplitThreads) cnt[i] = 0;
        __syncthreads();

        int* row = cnt + wave * nd;
        const int seg = ((n_r + kSplitWaves - 1) / kSplitWaves + 63) & ~63;      // entries per wavefront (<= 64 kSplitRounds)
        int32_t pos[kSplitRounds];
        unsigned meta[kSplitRounds];       // split_round()
#pragma unroll
        for (int r = 0; r < kSplitRounds; ++r) {
            if (r * 64 >= seg) {          // uniform: this round is past the wavefront's share
                meta[r] = 0u;
                pos[r] = 0;
                continue;
            }
            const int i = wave * seg + r * 64 + lane;
            const uint32_t e = i < n_r ? bufa[i] : 0u;
            meta[r] = e;
            // all loads in flight at once; used only after the scan (row 0 if idle)
            pos[r] = d.pos_affine ? d.pos0 + (int32_t)(e >> d.S) : d.pos_log[e >> d.S];
        }
#pragma unroll
        for (int r = 0; r < kSplitRounds; ++r) {
            if (r * 64 >= seg) {          // uniform: this round is past the wavefront's share
                meta[r] = 0u;
                continue;
            }
            const bool valid = wave * seg + r * 64 + lane < n_r;
            meta[r] = split_round<NBITS>(row, meta[r] & mask, valid);
        }
        __syncthreads();
        split_scan(cnt, nd, rstart, rcount, wsum);
        if (!multi && tid < nfl) offs[tid] = out_base + rstart[tid];
        if (multi) {
#pragma unroll
            for (int r = 0; r < kSplitRounds; ++r)
                if (r * 64 < seg && (meta[r] & kSplitValid)) {
                    const unsigned fl = meta[r] & 0xFFu;
                    const int i = split_rank(row, meta[r]);
                    posout[cursor[fl] + (i - rstart[fl])] = pos[r];
                    if (nbk) bufb[i] = pos[r];
                }
        } else {
            if (tid < nd) lstart[tid] = out_base + rstart[tid];
#pragma unroll
            for (int r = 0; r < kSplitRounds; ++r)
                if (r * 64 < seg && (meta[r] & kSplitValid)) bufb[split_rank(row, meta[r])] = pos[r];
        }
        __syncthreads();
        if (nbk && tid < nfl && rcount[tid] > 0) {
            // Block table, one thread per list: the round's part of the list is sorted in bufb; every block that
            // starts at or before its last entry and whose start is not known yet starts at the first entry of the
            // part that lies in it or beyond (binary search).  Rounds come in position order.
            const int32_t* seg = bufb + rstart[tid];
            const int n = rcount[tid];
            const int last = seg[n - 1];
            const int gbase = multi ? cursor[tid] : lstart[tid];
            int j = nextj[tid];
            while (j <= nbk && last >= (j << kS3PosBlockLog2)) {
                const int key = j << kS3PosBlockLog2;
                int lo = 0, hi = n;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (seg[mid] < key) lo = mid + 1; else hi = mid;
                }
                tab[tid * nbk + j - 1] = gbase + lo;
                ++j;
            }
            nextj[tid] = j;
        }
        if (multi) {
            if (tid < nd) cursor[tid] += rcount[tid];
        } else {
            if (tid < nd) cursor[tid] = lstart[tid] + rcount[tid];
            for (int i = tid; i < n_r; i += kSplitThreads) posout[out_base + i] = bufb[i];
        }
        tp += m;
        if (tp < n_tiles) p_next = tp + tid < n_tiles ? pc[tp + tid] : 0u;
        __syncthreads();
    }
    if (nbk && tid < nfl) {      // the blocks after a list's last entry start at its end; an empty list's all do
        const int end = cursor[tid];
        for (int j = nextj[tid]; j <= nbk; ++j) tab[tid * nbk + j - 1] = end;
    }
}

__global__ void idx_fill_positions_kernel(int32_t* dst, int n, int32_t base) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = base + i;
}

size_t bucket_sort_lds(int S) {
    return (size_t)kSortCap * 4 + (kSplitThreads + 1) * 4 + kSplitThreads * 4 + 16 * 4 + 5 * 256 * 4 +
           ((size_t)kSplitWaves << S) * 4;
}

struct Geometry {
    int S, NB, nbB, ptok, tile_post, w16;
};

bool geometry(int n_feat, int k, Geometry& g) {
    if (n_feat < 1 || n_feat > S3_MAX_FEAT || k < 1 || k > S3_MAX_K) return false;
    int bits = s3_ceil_log2((unsigned)n_feat);
    g.S = bits > 8 ? bits - 8 : 0;
    g.NB = (n_feat + (1 << g.S) - 1) >> g.S;
    g.nbB = s3_ceil_log2((unsigned)g.NB);
    g.ptok = kTilePost / k;
    g.tile_post = g.ptok * k;
    g.w16 = g.S + s3_ceil_log2((unsigned)g.ptok) <= 16;      // (row inside the tile, low feature bits) fit 16 bits
    return true;
}

int run_partition(const int32_t* src, int64_t head_stride, int rows, int tile0, int n_heads, const IdxDev& d,
                  hipStream_t st) {
    if (rows <= 0) return S3_OK;
    int ntiles = (rows + d.ptok - 1) / d.ptok;
    hipLaunchKernelGGL(idx_partition_kernel, dim3(ntiles, n_heads), dim3(kSplitThreads), 0, st, src, head_stride, rows,
                       tile0, d);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

int run_finalize(const IdxDev& d, int n_heads, int n_tiles, hipStream_t st) {
    hipLaunchKernelGGL(idx_totals_kernel, dim3(d.NB, n_heads), dim3(256), 0, st, d, n_tiles);
    hipLaunchKernelGGL(idx_bucket_scan_kernel, dim3(n_heads), dim3(256), 0, st, d);
    // one ballot per low feature bit: the widths that the supported SAE sizes use most get their own build
    const dim3 grid(d.NB, n_heads), block(kSplitThreads);
    const size_t lds = bucket_sort_lds(d.S);       // < 64 KB: two workgroups per compute unit
    if (d.S <= 6) hipLaunchKernelGGL(idx_bucket_sort_kernel<6>, grid, block, lds, st, d, n_tiles);
    else if (d.S == 7) hipLaunchKernelGGL(idx_bucket_sort_kernel<7>, grid, block, lds, st, d, n_tiles);
    else hipLaunchKernelGGL(idx_bucket_sort_kernel<8>, grid, block, lds, st, d, n_tiles);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // namespace

struct s3_index {
    int n_heads, n_feat, k;
    int64_t max_tokens, tokens;
    bool finalized;
    bool sorted;          // every posting list is in increasing position order (implicit, increasing positions only)
    int64_t last_pos;     // position of the last appended row (implicit positions)
    int64_t max_pos;      // largest position appended so far (implicit positions; meaningless once !sorted)
    bool affine;          // every append so far used implicit positions continuing the first one's: row r is at pos0 + r
    int32_t pos0;
    int nblk;             // position blocks covered by the block table (0: no table)
    int32_t* btab;
    Geometry g;
    IdxDev d;
    int32_t* pos_log;
    int32_t* pending;     // [n_heads][ptok][k]: rows of the tile that is not complete yet
    void* block;          // the one device allocation everything above lives in
};

// Internal view for the scoring translation unit.
void s3_index_view(const s3_index* idx, S3IndexView* v) {
    v->n_heads = idx->n_heads; v->n_feat = idx->n_feat; v->k = idx->k; v->tokens = idx->tokens;
    v->offsets = idx->d.offsets; v->off_stride = idx->d.off_stride;
    v->positions = idx->d.positions; v->pos_stride = idx->d.pos_stride;
    v->finalized = idx->finalized; v->sorted = idx->sorted; v->max_pos = idx->max_pos;
    v->btab = idx->btab; v->nblk = idx->nblk;
    v->btab_valid = idx->btab && idx->sorted && idx->max_pos < ((int64_t)idx->nblk << kS3PosBlockLog2);
}

// Workspace of the one-shot build: inter | piece | total | bbase | pos_log
static size_t build_layout(int T, int k, int n_feat, const Geometry& g, size_t off[5]) {
    int max_tiles = (T + g.ptok - 1) / g.ptok;
    if (max_tiles < 1) max_tiles = 1;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += s3_align(bytes); return at; };
    off[0] = take((size_t)max_tiles * g.tile_post * 4);
    off[1] = take((size_t)g.NB * max_tiles * 4);
    off[2] = take((size_t)g.NB * 4);
    off[3] = take((size_t)(g.NB + 1) * 4);
    off[4] = take((size_t)(T > 0 ? T : 1) * 4);
    return o;
}

__global__ void idx_fill_kernel(int32_t* dst, int n, int32_t v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

static int index_build_impl(const char* who, const int32_t* ids, const int32_t* positions, int T, int k, int n_feat,
                            int32_t* offsets, int32_t* out_positions, void* ws, size_t ws_bytes, void* stream) {
    Geometry g;
    if (T < 0 || !geometry(n_feat, k, g)) return s3_fail(S3_EINVAL, "%s: T %d, n_feat %d, k %d out of range", who, T, n_feat, k);
    if (!offsets || (T > 0 && (!ids || !out_positions || !ws))) return s3_fail(S3_EINVAL, "%s: null pointer", who);
    if (T > (1 << 24) || (int64_t)T * k >= (1LL << 31)) return s3_fail(S3_EINVAL, "%s: T %d too large", who, T);
    size_t off[5];
    size_t need = build_layout(T, k, n_feat, g, off);
    if (T > 0 && ws_bytes < need) return s3_fail(S3_ECAPACITY, "%s: workspace %zu < %zu bytes", who, ws_bytes, need);
    if (T > 0 && ((uintptr_t)ws & 255)) return s3_fail(S3_EINVAL, "%s: workspace must be 256-byte aligned", who);
    hipStream_t st = (hipStream_t)stream;
    if (T == 0) {      // an empty index: every list is empty (a fill kernel, so that a caller may capture the call in a graph)
        hipLaunchKernelGGL(idx_fill_kernel, dim3((n_feat + 1 + 255) / 256), dim3(256), 0, st, offsets, n_feat + 1, 0);
        S3_HIP(hipGetLastError());
        return S3_OK;
    }
    char* base = (char*)ws;
    IdxDev d;
    d.n_feat = n_feat; d.k = k; d.S = g.S; d.NB = g.NB; d.nbB = g.nbB; d.ptok = g.ptok; d.tile_post = g.tile_post; d.w16 = g.w16;
    d.kinv = k > 1 ? (uint32_t)(((1ull << 32) + (uint32_t)k - 1) / (uint32_t)k) : 0u;
    d.max_tiles = (T + g.ptok - 1) / g.ptok;
    d.inter = (uint32_t*)(base + off[0]); d.piece = (uint32_t*)(base + off[1]);
    d.total = (int32_t*)(base + off[2]); d.bbase = (int32_t*)(base + off[3]);
    int32_t* plog = (int32_t*)(base + off[4]);
    d.pos_log = plog; d.offsets = offsets; d.positions = out_positions;
    d.inter_stride = 0; d.piece_stride = 0; d.off_stride = 0; d.pos_stride = 0;
    d.btab = nullptr; d.nblk = 0; d.pos_affine = positions ? 0 : 1; d.pos0 = 0;
    if (positions) S3_HIP(hipMemcpyAsync(plog, positions, (size_t)T * 4, hipMemcpyDeviceToDevice, st));
    int rc = run_partition(ids, 0, T, 0, 1, d, st);
    if (rc) return rc;
    return run_finalize(d, 1, d.max_tiles, st);
}

// Scratch of s3_index_build_static: one array per GPU the library runs on, held until the process ends.  The name
// below is a host-side stand-in; the array's device address is looked up once per device and used from then on.
static __device__ __align__(256) unsigned char scratch[S3_STATIC_SCRATCH_BYTES];

static int static_scratch(void** out) {
    static std::mutex mu;
    static void* ptr[kS3MaxDevices] = {};
    int dev = 0;
    S3_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kS3MaxDevices) return s3_fail(S3_EINVAL, "s3_index_build_static: device %d not supported", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        S3_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return s3_fail(S3_EHIP, "s3_index_build_static: hipGetSymbolAddress returned a null address");
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return S3_OK;
}

extern "C" {

int s3_index_create(int n_heads, int n_feat, int k, int64_t max_tokens, s3_index** out) {
    if (!out) return s3_fail(S3_EINVAL, "s3_index_create: null out");
    Geometry g;
    if (n_heads < 1 || !geometry(n_feat, k, g))
        return s3_fail(S3_EINVAL, "s3_index_create: n_heads %d, n_feat %d (<= %d), k %d (<= %d) out of range", n_heads,
                       n_feat, S3_MAX_FEAT, k, S3_MAX_K);
    if (max_tokens < 1 || max_tokens > (1 << 24) || max_tokens * k >= (1LL << 31))
        return s3_fail(S3_EINVAL, "s3_index_create: max_tokens %lld out of range (<= 2^24 and max_tokens * k < 2^31)",
                       (long long)max_tokens);
    s3_index* ix = new (std::nothrow) s3_index();
    if (!ix) return s3_fail(S3_EHIP, "s3_index_create: out of host memory");
    ix->n_heads = n_heads; ix->n_feat = n_feat; ix->k = k; ix->max_tokens = max_tokens; ix->tokens = 0;
    ix->finalized = false; ix->sorted = true; ix->last_pos = -1; ix->max_pos = -1; ix->affine = true; ix->pos0 = 0; ix->g = g;
    const int64_t nb = (max_tokens + (1 << kS3PosBlockLog2) - 1) >> kS3PosBlockLog2;
    ix->nblk = nb >= 2 && nb <= kS3MaxTableBlocks ? (int)nb : 0;
    IdxDev& d = ix->d;
    d.n_feat = n_feat; d.k = k; d.S = g.S; d.NB = g.NB; d.nbB = g.nbB; d.ptok = g.ptok; d.tile_post = g.tile_post; d.w16 = g.w16;
    d.kinv = k > 1 ? (uint32_t)(((1ull << 32) + (uint32_t)k - 1) / (uint32_t)k) : 0u;
    d.max_tiles = (int)((max_tokens + g.ptok - 1) / g.ptok);
    d.inter_stride = (int64_t)d.max_tiles * g.tile_post;
    d.piece_stride = (int64_t)g.NB * d.max_tiles;
    d.off_stride = n_feat + 1;
    d.pos_stride = max_tokens * k;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += s3_align(bytes); return at; };
    size_t o_inter = take((size_t)n_heads * d.inter_stride * 4);
    size_t o_piece = take((size_t)n_heads * d.piece_stride * 4);
    size_t o_total = take((size_t)n_heads * g.NB * 4);
    size_t o_bbase = take((size_t)n_heads * (g.NB + 1) * 4);
    size_t o_offs = take((size_t)n_heads * d.off_stride * 4);
    size_t o_pos = take((size_t)n_heads * d.pos_stride * 4);
    size_t o_plog = take((size_t)max_tokens * 4);
    size_t o_pend = take((size_t)n_heads * g.tile_post * 4);
    size_t o_btab = take(ix->nblk ? (size_t)n_heads * n_feat * (ix->nblk - 1) * 4 : 0);
    hipError_t e = hipMalloc(&ix->block, o);
    if (e != hipSuccess) {
        delete ix;
        return s3_fail(S3_EHIP, "s3_index_create: hipMalloc of %zu bytes failed: %s", o, hipGetErrorString(e));
    }
    char* base = (char*)ix->block;
    d.inter = (uint32_t*)(base + o_inter); d.piece = (uint32_t*)(base + o_piece);
    d.total = (int32_t*)(base + o_total); d.bbase = (int32_t*)(base + o_bbase);
    d.offsets = (int32_t*)(base + o_offs); d.positions = (int32_t*)(base + o_pos);
    ix->pos_log = (int32_t*)(base + o_plog); d.pos_log = ix->pos_log;
    ix->pending = (int32_t*)(base + o_pend);
    ix->btab = ix->nblk ? (int32_t*)(base + o_btab) : nullptr;
    d.btab = ix->btab; d.nblk = ix->nblk; d.pos_affine = 0; d.pos0 = 0;
    *out = ix;
    return S3_OK;
}

void s3_index_destroy(s3_index* idx) {
    if (!idx) return;
    if (idx->block) (void)hipFree(idx->block);
    delete idx;
}

int64_t s3_index_tokens(const s3_index* idx) { return idx ? idx->tokens : 0; }

int s3_index_reset(s3_index* idx) {
    if (!idx) return s3_fail(S3_EINVAL, "s3_index_reset: null index");
    idx->tokens = 0;
    idx->finalized = false;
    idx->sorted = true;
    idx->last_pos = -1;
    idx->max_pos = -1;
    idx->affine = true;
    idx->pos0 = 0;
    return S3_OK;
}

int s3_index_append(s3_index* idx, const int32_t* ids, int T, const int32_t* positions, int32_t base_pos,
                    void* stream) {
    if (!idx || (!ids && T > 0)) return s3_fail(S3_EINVAL, "s3_index_append: null pointer");
    if (T < 0) return s3_fail(S3_EINVAL, "s3_index_append: T %d < 0", T);
    if (idx->finalized) return s3_fail(S3_ESTATE, "s3_index_append: index already finalized");
    if (idx->tokens + T > idx->max_tokens)
        return s3_fail(S3_ECAPACITY, "s3_index_append: %lld + %d tokens exceed max_tokens %lld", (long long)idx->tokens,
                       T, (long long)idx->max_tokens);
    if (T == 0) return S3_OK;
    hipStream_t st = (hipStream_t)stream;
    const IdxDev& d = idx->d;
    const int k = idx->k, ptok = d.ptok, H = idx->n_heads;
    const int64_t r0 = idx->tokens;
    // While every append continues the first one's implicit positions, row r is at pos0 + r and no position is
    // stored.  The first append that breaks the pattern writes the positions of the rows before it, and from
    // then on every append stores its own.
    const bool continues = !positions && (r0 == 0 || (idx->affine && (int64_t)base_pos == (int64_t)idx->pos0 + r0));
    if (idx->affine && !continues && r0 > 0)
        hipLaunchKernelGGL(idx_fill_positions_kernel, dim3((unsigned)((r0 + 255) / 256)), dim3(256), 0, st, idx->pos_log,
                           (int)r0, idx->pos0);
    if (r0 == 0 && !positions) idx->pos0 = base_pos;
    idx->affine = idx->affine && continues;
    if (positions) {
        idx->sorted = false;          // caller-given positions: order unknown to the host
        S3_HIP(hipMemcpyAsync(idx->pos_log + r0, positions, (size_t)T * 4, hipMemcpyDeviceToDevice, st));
    } else {
        if ((int64_t)base_pos <= idx->last_pos) idx->sorted = false;
        idx->last_pos = (int64_t)base_pos + T - 1;
        if (idx->last_pos > idx->max_pos) idx->max_pos = idx->last_pos;
        if (!idx->affine)
            hipLaunchKernelGGL(idx_fill_positions_kernel, dim3((T + 255) / 256), dim3(256), 0, st, idx->pos_log + r0, T,
                               base_pos);
    }
    int done = 0;
    const int in_tile = (int)(r0 % ptok);
    if (in_tile) {   // complete the tile left open by the previous append
        int fill = T < ptok - in_tile ? T : ptok - in_tile;
        S3_HIP(hipMemcpy2DAsync(idx->pending + (size_t)in_tile * k, (size_t)d.tile_post * 4, ids, (size_t)T * k * 4,
                                (size_t)fill * k * 4, H, hipMemcpyDeviceToDevice, st));
        done = fill;
        if (in_tile + fill == ptok) {
            int rc = run_partition(idx->pending, d.tile_post, ptok, (int)(r0 / ptok), H, d, st);
            if (rc) return rc;
        }
    }
    const int full = (T - done) / ptok * ptok;
    if (full) {
        int rc = run_partition(ids + (size_t)done * k, (int64_t)T * k, full, (int)((r0 + done) / ptok), H, d, st);
        if (rc) return rc;
        done += full;
    }
    if (done < T)   // rows of a tile that is not complete yet
        S3_HIP(hipMemcpy2DAsync(idx->pending, (size_t)d.tile_post * 4, ids + (size_t)done * k, (size_t)T * k * 4,
                                (size_t)(T - done) * k * 4, H, hipMemcpyDeviceToDevice, st));
    idx->tokens += T;
    return S3_OK;
}

int s3_index_finalize(s3_index* idx, void* stream) {
    if (!idx) return s3_fail(S3_EINVAL, "s3_index_finalize: null index");
    if (idx->finalized) return s3_fail(S3_ESTATE, "s3_index_finalize: already finalized");
    hipStream_t st = (hipStream_t)stream;
    const IdxDev& d = idx->d;
    const int rem = (int)(idx->tokens % d.ptok);
    if (rem) {
        int rc = run_partition(idx->pending, d.tile_post, rem, (int)(idx->tokens / d.ptok), idx->n_heads, d, st);
        if (rc) return rc;
    }
    const int n_tiles = (int)((idx->tokens + d.ptok - 1) / d.ptok);
    IdxDev df = d;
    df.pos_affine = idx->affine ? 1 : 0;
    df.pos0 = idx->pos0;
    int rc = run_finalize(df, idx->n_heads, n_tiles, st);
    if (rc) return rc;
    idx->finalized = true;
    return S3_OK;
}

int s3_index_csr(const s3_index* idx, int head, const int32_t** offsets, const int32_t** positions,
                 int64_t* n_postings) {
    if (!idx || !offsets || !positions || !n_postings) return s3_fail(S3_EINVAL, "s3_index_csr: null pointer");
    if (head < 0 || head >= idx->n_heads) return s3_fail(S3_EINVAL, "s3_index_csr: head %d out of range", head);
    if (!idx->finalized) return s3_fail(S3_ESTATE, "s3_index_csr: index not finalized");
    *offsets = idx->d.offsets + (size_t)head * idx->d.off_stride;
    *positions = idx->d.positions + (size_t)head * idx->d.pos_stride;
    *n_postings = idx->tokens * idx->k;
    return S3_OK;
}

int s3_index_export(const s3_index* idx, int head, int32_t* offsets_out, int32_t* positions_out, void* stream) {
    const int32_t *o, *p;
    int64_t n;
    int rc = s3_index_csr(idx, head, &o, &p, &n);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (offsets_out)
        S3_HIP(hipMemcpyAsync(offsets_out, o, (size_t)(idx->n_feat + 1) * 4, hipMemcpyDeviceToDevice, st));
    if (positions_out && n)
        S3_HIP(hipMemcpyAsync(positions_out, p, (size_t)n * 4, hipMemcpyDeviceToDevice, st));
    return S3_OK;
}

size_t s3_index_build_workspace(int T, int k, int n_feat) {
    Geometry g;
    if (T < 0 || !geometry(n_feat, k, g)) return 0;
    size_t off[5];
    return build_layout(T, k, n_feat, g, off);
}

int s3_index_build(const int32_t* ids, const int32_t* positions, int T, int k, int n_feat, int32_t* offsets,
                   int32_t* out_positions, void* ws, size_t ws_bytes, void* stream) {
    return index_build_impl("s3_index_build", ids, positions, T, k, n_feat, offsets, out_positions, ws, ws_bytes, stream);
}

int s3_index_build_static(const int32_t* ids, const int32_t* positions, int T, int k, int n_feat, int32_t* offsets,
                          int32_t* out_positions, void* stream) {
    Geometry g;
    if (T < 0 || !geometry(n_feat, k, g))
        return s3_fail(S3_EINVAL, "s3_index_build_static: T %d, n_feat %d, k %d out of range", T, n_feat, k);
    size_t off[5];
    const size_t need = build_layout(T, k, n_feat, g, off);
    if (need > S3_STATIC_SCRATCH_BYTES)
        return s3_fail(S3_ECAPACITY, "s3_index_build_static: T %d x k %d needs %zu bytes of scratch, the built-in buffer has %zu",
                       T, k, need, (size_t)S3_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return index_build_impl("s3_index_build_static", ids, positions, T, k, n_feat, offsets, out_positions, ws,
                            S3_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"
