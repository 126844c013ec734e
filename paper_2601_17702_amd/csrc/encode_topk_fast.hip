// Fast path of the fused SAE encoder + Top-k (Sec. 3.3; k = 128 is the sparsity of App. B.3): bf16, d_head = 128,
// k <= 128, n_feat a multiple of 128.  The kernel body lives in encode_topk_fast_impl.inc and is built three times:
// 8 wavefronts with 40 list slots per lane for k <= 32, 4 wavefronts with 80 slots per lane for k <= 64, 2 wavefronts
// with 140 slots per lane for k <= 128.
//
// Same method as the generic kernel (features on the MFMA M axis, per-token threshold tau,
// candidate lists in LDS, exact selection), laid out for two wavefronts per SIMD:
//
//   - workgroup = 8 (k <= 32) or 4 (k <= 64) wavefronts of 32 tokens.  W_enc streams through a ring of four 32-feature
//     stages in LDS.  Each wavefront copies 4 rows of a stage per step straight from global memory
//     into LDS (no registers in between); the copies of a pair of stages are started one pair
//     (64 features) ahead of their MFMAs; one barrier per pair;
//   - rows are 256 bytes, unpadded; the sixteen 16-byte pieces of row r are stored at piece index
//     (c xor (r & 15)), which makes the 16-byte fragment reads of 16 consecutive rows conflict-free;
//   - b_enc is copied the same way (fp32) and read as the accumulator's initial value (the first
//     MFMA's C operand), so the bias costs no vector-ALU instruction;
//   - the epilogue of a stage is lane-parallel and runs between the MFMAs of the next stage: every lane
//     packs the 16 signs of (tau - accumulator) into a hit mask, picks its first hit with a 16-to-1
//     select tree and appends it under the mask of lanes that have one (no branch per accumulator; the
//     MFMA chain is spelled out in assembly so that it keeps this interleaving).  A lane with a second
//     hit in the same stage takes it in a short loop after the chain (one stage in eight has one).
//     Each lane owns a fixed list of CAPL slots, so "list full" is one compare on its write pointer;
//   - threshold refreshes are voted per workgroup at the pair barrier, so that all wavefronts
//     refresh at the same point instead of stalling each other one after the other; the refresh
//     loads the lane's candidates into registers once and narrows tau there;
//   - the final k candidates of a token are sorted with a 32-lane bitonic network (two tokens per
//     wavefront step) and written coalesced.
//
// LDS accesses inside the stage loop (fragment reads, list appends, votes) are written as inline
// assembly: the compiler orders every LDS access it knows of behind ALL outstanding global->LDS
// copies (it cannot tell which bytes a copy writes), which would drain the copy pipeline in every step.
// The waits that the ring really needs are the explicit s_waitcnt before each barrier.
#include "s3_common.h"

#include <float.h>
#include <math.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kFT = 32;          // features per stage (one 32x32 MFMA tile per wavefront)
constexpr int kRing = 4;         // stages in the LDS ring
constexpr int DH = 128;
constexpr int NS = DH / 16;      // MFMA K steps per stage
constexpr int RB = DH * 2;       // bytes of one W row
constexpr int kStageB = kFT * RB;
constexpr int kBiasB = 256;      // the 64 fp32 biases of a pair of stages (one wavefront-wide copy)
constexpr int kGuard = 4;        // free slots that a refresh leaves in every list at least
constexpr float kHintMargin = 0.04f;   // streamed calls start 4 % below the carried bound
constexpr float kRedoMargin = 0.05f;   // bounds of a head that needed the redo pass are lowered by this much more
constexpr float kPilotMargin = 0.03f;  // bounds taken from the pilot's single tile are lowered by this much more
constexpr int kOffBias = kRing * kStageB;
constexpr int kOffVote = kOffBias + (kRing / 2) * kBiasB;
constexpr int kOffVal = kOffVote + 16;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(1))) const void glb_cvoid;

// compile-time ablation masks: the product library instantiates the kernels with 0 only; builds with -DS3_TUNING
// (measurement tooling, never shipped) also instantiate kernels without appends and with per-phase cycle counters
constexpr int kNoHits = 1, kProfile = 16;
constexpr int kFillWGs = 256;      // workgroups that give every compute unit one

#ifdef S3_TUNING
// kProfile build: cycles per phase, summed over the steps of wavefronts 0 and 4 of workgroup 0
__device__ unsigned long long s3_prof[32];
#endif

__device__ __forceinline__ void lds_store_u32(unsigned addr, unsigned v) {
    asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}

// Waits until at most N of this wavefront's global->LDS copies are in flight and all its LDS accesses are
// done, then joins the workgroup barrier.
template <int N>
__device__ __forceinline__ void stage_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

__device__ __forceinline__ unsigned ordered_key(float v) {
    unsigned u = __float_as_uint(v);
    return u ^ ((unsigned)((int)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_value(unsigned k) {
    return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// x of this lane combined with x of the token's other lane (lane ^ 32): one cross-half swap, no LDS
__device__ __forceinline__ int pair_sum(int x) {
    auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return (int)(r[0] + r[1]);
}
__device__ __forceinline__ float pair_fsum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float pair_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_min(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

struct Refreshed {
    int cnt;
    float tau;
    int passes;   // search passes taken (read by the profiling build only)
    unsigned t[4];   // profiling build: cycles of load / bracket / search / compaction
};

// Streamed calls: counters and this call's minima start empty; afterwards the minima become the carried bounds.
__global__ void enc_stream_prep_kernel(int32_t* redo_cnt, unsigned* hint_out, float* hint_sum, int n_heads) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_heads) redo_cnt[i] = 0;
    if (i < 2 * n_heads) hint_out[i] = 0xFFFFFFFFu;
    if (i < 3 * n_heads) hint_sum[i] = 0.f;
}
// Two candidate bounds per head: (smallest tau / |x|) * |x_t| and the smallest tau.  Which one predicts a token's
// threshold better depends on the data (pre-activations dominated by W x scale with |x|, those dominated by the
// bias do not); using both at once would fail whenever either overshoots.  The one that was tighter on average
// over this call's tokens is carried, the other one is set to -inf.
// `boot`: null for the bounds carried out of the call.  Else (after the pilot launch) the bounds the caller carried
// in: heads that had one keep it for the main launch, the others start from the pilot's tile, lowered by `extra`
// because the minimum over one tile of tokens is a weaker bound than the minimum over a whole chunk.
// `redo_cnt` (bounds carried out of the call only): a head whose carried bound was too high for some token of this
// call hands on a bound that is lower by kRedoMargin more, so that a drifting stream does not pay a redo pass in
// every call.
__global__ void enc_stream_post_kernel(const unsigned* hint_out, const float* hint_sum, float* hint, int n_heads,
                                       const float* boot, float extra, const int32_t* redo_cnt) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= n_heads) return;
    if (redo_cnt && redo_cnt[h] > 0) extra += kRedoMargin;
    if (boot && !(boot[2 * h] == -INFINITY && boot[2 * h + 1] == -INFINITY)) {
        hint[2 * h] = boot[2 * h];
        hint[2 * h + 1] = boot[2 * h + 1];
        return;
    }
    const float r = hint_out[2 * h] == 0xFFFFFFFFu ? -INFINITY : key_value(hint_out[2 * h]);
    const float a = hint_out[2 * h + 1] == 0xFFFFFFFFu ? -INFINITY : key_value(hint_out[2 * h + 1]);
    const float s_tau = hint_sum[3 * h], s_x = hint_sum[3 * h + 1], s_n = hint_sum[3 * h + 2];
    const float waste_r = r > -INFINITY ? s_tau - r * s_x : INFINITY;
    const float waste_a = a > -INFINITY ? s_tau - a * s_n : INFINITY;
    const bool use_r = waste_r <= waste_a;
    hint[2 * h] = use_r ? r - extra * fabsf(r) : -INFINITY;
    hint[2 * h + 1] = use_r ? -INFINITY : a - extra * fabsf(a);
}

// One build of the kernel per list geometry: 8 wavefronts x 40 slots per lane for k <= 32, 4 wavefronts x 80 slots
// per lane for k <= 64 (same LDS footprint), 2 wavefronts x 140 slots per lane for k <= 128 (a lane must be able to
// hold all k survivors of its token: they may all fall into its half of the features).
namespace k32 {
#define S3_CFG_WAVES 8
#define S3_CFG_CAPL 40
#define S3_CFG_KMAX 32
#include "encode_topk_fast_impl.inc"
#undef S3_CFG_WAVES
#undef S3_CFG_CAPL
#undef S3_CFG_KMAX
}  // namespace k32
namespace k64 {
#define S3_CFG_WAVES 4
#define S3_CFG_CAPL 80
#define S3_CFG_KMAX 64
#include "encode_topk_fast_impl.inc"
#undef S3_CFG_WAVES
#undef S3_CFG_CAPL
#undef S3_CFG_KMAX
}  // namespace k64
namespace k128 {
#define S3_CFG_WAVES 2
#define S3_CFG_CAPL 140
#define S3_CFG_KMAX 128
#include "encode_topk_fast_impl.inc"
#undef S3_CFG_WAVES
#undef S3_CFG_CAPL
#undef S3_CFG_KMAX
}  // namespace k128
namespace k128n {      // the same lists in workgroups of one wavefront: twice the workgroups when a call has few tokens
#define S3_CFG_WAVES 1
#define S3_CFG_CAPL 140
#define S3_CFG_KMAX 128
#include "encode_topk_fast_impl.inc"
#undef S3_CFG_WAVES
#undef S3_CFG_CAPL
#undef S3_CFG_KMAX
}  // namespace k128n

}  // namespace

bool s3_encode_fast_ok(int dtype, int d_head, int n_feat, int k) {
    return dtype == S3_BF16 && d_head == DH && k <= k128::kMaxK && n_feat % (4 * kFT) == 0;
}

static int fast_dispatch(EncParams p, hipStream_t st);

int s3_encode_fast_launch(EncParams p, hipStream_t st) {
    p.mode = 0;
    p.hint_in = nullptr; p.boot_in = nullptr; p.hint_out = nullptr; p.hint_sum = nullptr; p.redo_list = nullptr; p.redo_cnt = nullptr;
    return fast_dispatch(p, st);
}

// Merge of the two halves' Top-k of one token (each sorted by pre-activation descending, feature id ascending; no key
// occurs twice): an entry's place is its place in its own list plus the number of entries of the other list in front
// of it, found by bisection.  One wavefront per (head, token), two entries of each list per lane (k <= 128).
__global__ __launch_bounds__(256) void enc_merge2_kernel(const int32_t* __restrict__ part_ids, const float* __restrict__ part_vals,
                                                         int n_heads, int T, int k, int32_t* __restrict__ ids,
                                                         float* __restrict__ vals) {
    __shared__ unsigned skey[4][2][128];
    __shared__ int sid[4][2][128];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long long row = (long long)blockIdx.x * 4 + w;           // head * T + token
    const bool live = row < (long long)n_heads * T;
    const int head = live ? (int)(row / T) : 0, tok = live ? (int)(row % T) : 0;
    for (int l = 0; l < 2; ++l) {
        const size_t src = (((size_t)(2 * head + l)) * T + tok) * k;
        for (int e = lane; e < k; e += 64) {
            skey[w][l][e] = live ? ordered_key(part_vals[src + e]) : 0u;
            sid[w][l][e] = live ? part_ids[src + e] : 0;
        }
    }
    __syncthreads();
    if (!live) return;
    const size_t dst = (size_t)row * k;
    for (int l = 0; l < 2; ++l) {
        const unsigned* okey = skey[w][l ^ 1];
        const int* oid = sid[w][l ^ 1];
        for (int e = lane; e < k; e += 64) {
            const unsigned kv = skey[w][l][e];
            const int id = sid[w][l][e];
            int lo = 0, hi = k;                                    // entries of the other list in front of this one
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                const bool before = okey[mid] > kv || (okey[mid] == kv && oid[mid] < id);
                if (before) lo = mid + 1; else hi = mid;
            }
            const int rank = e + lo;
            if (rank < k) {
                ids[dst + rank] = id;
                vals[dst + rank] = fmaxf(key_value(kv), 0.f);
            }
        }
    }
}

bool s3_encode_fast_split_pays(int n_heads, int T, int n_feat, int k) {
    if (k <= k64::kMaxK || k > k128::kMaxK || n_feat % 256 != 0 || n_feat / 2 < k) return false;   // built for the k <= 128 lists only
    const long long tiles = (long long)n_heads * ((T + k128n::kTokWG - 1) / k128n::kTokWG);
    return 2 * tiles <= kFillWGs;
}

int s3_encode_fast_split(EncParams p, int32_t* part_ids, float* part_vals, hipStream_t st) {
    int32_t* ids = p.ids;
    float* vals = p.vals;
    const int n_heads = p.n_heads;
    p.ids = part_ids; p.vals = part_vals;
    p.n_heads = 2 * n_heads; p.n_feat /= 2; p.fsplit = 2;
    if (int rc = s3_encode_fast_launch(p, st)) return rc;
    const long long rows = (long long)n_heads * p.T;
    hipLaunchKernelGGL(enc_merge2_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, (const int32_t*)part_ids,
                       (const float*)part_vals, n_heads, p.T, p.k, ids, vals);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

size_t s3_encode_fast_stream_workspace(int n_heads, int T) {
    return s3_align((size_t)n_heads * 4) + 2 * s3_align((size_t)n_heads * 8) + s3_align((size_t)n_heads * 12) +
           s3_align((size_t)n_heads * T * 4);
}

// Pilot (heads without a carried bound: their first token tile, from -inf), main pass from the carried or the
// pilot's bounds, redo pass (from -inf) for the tokens whose bound was too high; then this call's minima become
// the bounds for the next call.  All on `st`; nothing is read back.
int s3_encode_fast_stream(EncParams p, float* hint, void* ws, hipStream_t st) {
    char* base = (char*)ws;
    size_t o = 0;
    auto take = [&](size_t bytes) { char* at = base + o; o += s3_align(bytes); return at; };
    p.redo_cnt = (int32_t*)take((size_t)p.n_heads * 4);
    p.hint_out = (unsigned*)take((size_t)p.n_heads * 8);
    float* hint_mid = (float*)take((size_t)p.n_heads * 8);
    p.hint_sum = (float*)take((size_t)p.n_heads * 12);
    p.redo_list = (int32_t*)take((size_t)p.n_heads * p.T * 4);
    const int nb = (3 * p.n_heads + 255) / 256;
    hipLaunchKernelGGL(enc_stream_prep_kernel, dim3(nb), dim3(256), 0, st, p.redo_cnt, p.hint_out, p.hint_sum, p.n_heads);
    p.margin = kHintMargin;
    float extra = kPilotMargin;
#ifdef S3_TUNING
    p.margin = (float)env_int("S3_ENC_MARGIN", (int)(kHintMargin * 1000.f + 0.5f)) * 1e-3f;   // per mille
    extra = (float)env_int("S3_ENC_PILOT_MARGIN", (int)(kPilotMargin * 1000.f + 0.5f)) * 1e-3f;
#endif
    p.boot_in = hint;
    p.hint_in = nullptr;
    p.mode = 3;
    int rc = fast_dispatch(p, st);
    if (rc) return rc;
    hipLaunchKernelGGL(enc_stream_post_kernel, dim3(nb), dim3(256), 0, st, p.hint_out, p.hint_sum, hint_mid, p.n_heads,
                       (const float*)hint, extra, (const int32_t*)nullptr);
    p.hint_in = hint_mid;
    p.mode = 1;
    rc = fast_dispatch(p, st);
    if (rc) return rc;
    p.mode = 2;
    rc = fast_dispatch(p, st);
    if (rc) return rc;
    hipLaunchKernelGGL(enc_stream_post_kernel, dim3(nb), dim3(256), 0, st, p.hint_out, p.hint_sum, hint, p.n_heads,
                       (const float*)nullptr, 0.f, (const int32_t*)p.redo_cnt);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

static int fast_dispatch(EncParams p, hipStream_t st) {
    const bool small_k = p.k <= k32::kMaxK, large_k = p.k > k64::kMaxK;
    p.soft = small_k ? k32::kSoftDefault : (large_k ? k128::kSoftDefault : k64::kSoftDefault);      // list length that asks for a voted refresh
#ifdef S3_TUNING
    const int capl = small_k ? k32::CAPL : (large_k ? k128::CAPL : k64::CAPL);
    p.soft = env_int("S3_ENC_SOFT", p.soft);                       // 0 = no voted refreshes
    if (p.soft < 0 || p.soft > capl - kGuard) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: bad S3_ENC_SOFT");
    if (large_k) {
        if (p.ablate) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: S3_ENC_ABLATE %d is not built for k > 64", p.ablate);
    } else if (small_k) {
        switch (p.ablate) {       // parts of the kernel compiled out (results are then meaningless)
            case 0: break;
            case 1: return k32::launch_fast<kNoHits>(p, st);
            case 16: return k32::launch_fast<kProfile>(p, st);
            case 17: return k32::launch_fast<kProfile | kNoHits>(p, st);
            default: return s3_fail(S3_EINVAL, "s3_sae_encode_topk: S3_ENC_ABLATE %d is not built", p.ablate);
        }
    } else {
        switch (p.ablate) {
            case 0: break;
            case 1: return k64::launch_fast<kNoHits>(p, st);
            default: return s3_fail(S3_EINVAL, "s3_sae_encode_topk: S3_ENC_ABLATE %d is not built", p.ablate);
        }
    }
#endif
    if (large_k) {
        // A call whose token tiles would leave most compute units without a workgroup (an SAE training batch: one
        // head, a few thousand tokens) runs in one-wavefront workgroups instead.
        const long long tiles = (long long)p.n_heads * ((p.T + k128::kTokWG - 1) / k128::kTokWG);
        return tiles < kFillWGs ? k128n::launch_fast<0>(p, st) : k128::launch_fast<0>(p, st);
    }
    return small_k ? k32::launch_fast<0>(p, st) : k64::launch_fast<0>(p, st);
}

#ifdef S3_TUNING
// Measurement aid of the tuning build: phase cycle sums of the last S3_ENC_ABLATE=16/17 launch.
extern "C" __attribute__((visibility("default"))) int s3_debug_profile(unsigned long long* out32) {
    S3_HIP(hipDeviceSynchronize());
    S3_HIP(hipMemcpyFromSymbol(out32, HIP_SYMBOL(s3_prof), sizeof(unsigned long long) * 32));
    return S3_OK;
}
#endif
