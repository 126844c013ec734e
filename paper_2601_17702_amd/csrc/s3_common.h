// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

// The library is built with -fvisibility=hidden: only what the public header declares is exported.
#pragma GCC visibility push(default)
#include "../../include/s3attn.h"
#pragma GCC visibility pop

int s3_fail(int code, const char* fmt, ...);   // records the thread-local message, returns code

#define S3_HIP(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess)                                                            \
            return s3_fail(S3_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));      \
    } while (0)

// Raises a kernel's dynamic-LDS limit once per device (thread-safe).  One S3LdsOnce object per kernel.
constexpr int kS3MaxDevices = 64;
struct S3LdsOnce {
    std::once_flag flag[kS3MaxDevices];
    hipError_t err[kS3MaxDevices];
};
int s3_allow_lds(S3LdsOnce& once, const void* kernel, int bytes);

static inline size_t s3_align(size_t n, size_t a = 256) { return (n + a - 1) / a * a; }
static inline int s3_ceil_log2(unsigned v) {
    int b = 0;
    while ((1u << b) < v) ++b;
    return b;
}

// Scoring keeps the scores of one block of 2^kS3PosBlockLog2 positions in LDS at a time; finalize records, per
// posting list, where each block starts (the block table), so that scoring reads no posting outside its block.
constexpr int kS3PosBlockLog2 = 14;
constexpr int kS3MaxTableBlocks = 64;      // no table for indexes of more blocks (longer lists are searched instead)

// Read-only view of an index for the scoring translation unit (defined in index.hip).
struct S3IndexView {
    int n_heads, n_feat, k;
    int64_t tokens;
    const int32_t* offsets;      // [n_heads] x off_stride
    const int32_t* positions;    // [n_heads] x pos_stride
    int64_t off_stride, pos_stride;
    bool finalized;
    bool sorted;                 // every list ascends in position (implicit, increasing positions only)
    int64_t max_pos;             // largest position appended (meaningful while sorted)
    // block table: btab[(h * n_feat + f) * (nblk - 1) + j - 1] = index, in head h's positions array, of the first
    // posting of list f whose position is >= j << kS3PosBlockLog2, j = 1 .. nblk - 1.  Null when there is none;
    // valid only for sorted lists whose positions are all below nblk << kS3PosBlockLog2 (btab_valid).
    const int32_t* btab;
    int nblk;
    bool btab_valid;
};
void s3_index_view(const s3_index* idx, S3IndexView* out);

// Read-only view of a compact index for the scoring translation unit (defined in compact.hip).
struct S3CompactView {
    int n_heads, n_feat, k, nblk;
    int64_t tokens;
    const int32_t* cstart;       // [n_heads] x cstart_stride (nblk * n_feat + 1 entries used)
    const uint16_t* delta;       // [n_heads] x delta_stride
    const int32_t* cfreq;        // [n_heads][n_feat]
    int64_t cstart_stride, delta_stride;
};
void s3_cindex_view(const s3_cindex* cidx, S3CompactView* out);

// ---- prefix sums shared by the index and the scoring kernels ----
// Inclusive prefix sums over the lanes of a wavefront / over each row of 16 lanes, by data-parallel-primitive
// lane shifts: row_shr 1, 2, 4, 8 inside the rows, then lane 15 of a row into the next row, lane 31 into rows 2, 3.
__device__ __forceinline__ int s3_row_incl_scan(int x) {
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);
    return x;
}
__device__ __forceinline__ int s3_wave_incl_scan(int x) {
    x = s3_row_incl_scan(x);
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);
    return x;
}

// Exclusive prefix sum of one int per thread over the block, in thread order.  wsum: one int per wavefront.
template <int NT>
__device__ __forceinline__ int s3_block_excl_scan(int v, int* wsum, int& total) {
    constexpr int NW = NT / 64;
    static_assert(NW == 4 || NW == 8 || NW == 16, "wavefront sums are scanned inside one row of 16 lanes");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int x = s3_wave_incl_scan(v);
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    const int s = s3_row_incl_scan(wsum[lane & (NW - 1)]);     // lanes 0 .. NW-1: sums of wavefronts 0 .. lane
    __syncthreads();
    total = __builtin_amdgcn_readlane(s, NW - 1);
    const int base = wave ? __builtin_amdgcn_readlane(s, wave - 1) : 0;
    return base + x - v;
}

// ---- encoder internals shared by the generic and the fast kernel ----
struct EncParams {
    const char* x;
    const char* w;
    const float* b;
    int32_t* ids;
    float* vals;
    int T, n_feat, k, n_heads, capt, tiles_per_head;
    int headroom;  // generic kernel: free list slots per token required before a run of appends (32, or 16 for k > 64)
    int ablate;    // tuning builds (-DS3_TUNING) only: parts of the kernel compiled out; always 0 in the product
    int soft;      // fast path: list length per lane that asks for a workgroup-wide refresh (0: off)
    int fsplit;    // fast path, plain calls: 1, or F > 1 = the call's heads are F feature ranges of each real head (head h reads
                   // the tokens of head h / F, its feature ids start at (h % F) * n_feat, values leave without the ReLU)
    // streamed calls (threshold carried from the previous chunk), fast path only
    float margin;              // relative margin below the carried bound
    int mode;                  // 0 plain, 1 start from the carried bound, 2 redo the tokens listed in redo_list,
                               // 3 pilot: first token tile of the heads that carry no bound yet, from -inf
    const float* hint_in;      // [n_heads][2]: lower bounds of tau / |x| and of tau seen in the previous call
    const float* boot_in;      // [n_heads][2]: the bounds the caller carried in (both -inf: the pilot covers tile 0)
    unsigned* hint_out;        // [n_heads][2]: ordered keys of this call's minima (atomicMin)
    float* hint_sum;           // [n_heads][3]: sums of tau, |x| and the token count over this call
    int32_t* redo_list;        // [n_heads][T] tokens whose carried bound was too high
    int32_t* redo_cnt;         // [n_heads]
};

#ifdef S3_TUNING
int env_int(const char* name, int dflt);      // tuning knobs are read from the environment in tuning builds only
#endif
bool s3_encode_fast_ok(int dtype, int d_head, int n_feat, int k);   // shapes the fast kernel is built for
int s3_encode_fast_launch(EncParams p, hipStream_t st);
// The same result by two launches' worth of workgroups: every head's features in two halves, each half's Top-k into
// part_ids / part_vals ([2 n_heads][T][k] each), then merged.  For calls with too few token tiles to fill the chip.
bool s3_encode_fast_split_pays(int n_heads, int T, int n_feat, int k);
int s3_encode_fast_split(EncParams p, int32_t* part_ids, float* part_vals, hipStream_t st);
size_t s3_encode_fast_stream_workspace(int n_heads, int T);
int s3_encode_fast_stream(EncParams p, float* hint, void* ws, hipStream_t st);   // hint [n_heads][2] device, in/out

// Workgroup -> (head, token tile).  Workgroups are dealt round-robin to the 8 XCDs (each with its own
// L2), so consecutive tiles of one head are placed on the SAME XCD: they stream the same W_enc rows at
// about the same time and share them in that L2.  Heads beyond the last multiple of 8 map linearly.
__device__ __forceinline__ void s3_block_to_tile(unsigned bid, int n_heads, int tiles_per_head, int& head, int& tt) {
    const unsigned full = (unsigned)(n_heads / 8) * 8u * (unsigned)tiles_per_head;
    if (bid < full) {
        unsigned xcd = bid & 7u, slot = bid >> 3;
        head = (int)(slot / tiles_per_head) * 8 + (int)xcd;
        tt = (int)(slot % tiles_per_head);
    } else {
        unsigned r = bid - full;
        head = (n_heads / 8) * 8 + (int)(r / tiles_per_head);
        tt = (int)(r % tiles_per_head);
    }
}
