// Fast path of the fused SAE encoder + Top-k (Sec. 3.3): bf16, d_head = 128, k <= 32,
// n_feat a multiple of 128.
//
// Same method as the generic kernel (features on the MFMA M axis, per-token threshold tau,
// candidate lists in LDS, exact selection), laid out for two wavefronts per SIMD:
//
//   - workgroup = 8 wavefronts = 256 tokens.  W_enc streams through a ring of four 32-feature
//     stages in LDS.  Each wavefront copies 4 rows of a stage per step straight from global memory
//     into LDS (no registers in between); the copies of a pair of stages are started one pair
//     (64 features) ahead of their MFMAs; one barrier per pair;
//   - rows are 256 bytes, unpadded; the sixteen 16-byte pieces of row r are stored at piece index
//     (c xor (r & 15)), which makes the 16-byte fragment reads of 16 consecutive rows conflict-free;
//   - b_enc is copied the same way (fp32) and read as the accumulator's initial value (the first
//     MFMA's C operand), so the bias costs no vector-ALU instruction;
//   - the epilogue of a stage takes the 16 hit masks (accumulator > tau, one scalar mask each) back
//     to back, then walks them with scalar branches; an accumulator with a survivor somewhere in the
//     wavefront runs a short append block under that mask.  Each lane owns a fixed list of CAPL slots,
//     so "list nearly full" is one compare on the lane's write pointer;
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

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kTokWG = 256;
constexpr int kFT = 32;          // features per stage (one 32x32 MFMA tile per wavefront)
constexpr int kRing = 4;         // stages in the LDS ring
constexpr int DH = 128;
constexpr int NS = DH / 16;      // MFMA K steps per stage
constexpr int RB = DH * 2;       // bytes of one W row
constexpr int kStageB = kFT * RB;
constexpr int kBiasB = 256;      // the 64 fp32 biases of a pair of stages (one wavefront-wide copy)
constexpr int CAPL = 40;         // list slots per lane (a token has two lanes)
constexpr int kGuard = 4;        // appends possible between two fullness checks
constexpr float kHintMargin = 0.03f;   // streamed calls start 3 % below the carried bound
constexpr int kOffBias = kRing * kStageB;
constexpr int kOffVote = kOffBias + (kRing / 2) * kBiasB;
constexpr int kOffVal = kOffVote + 16;
constexpr int kOffId = kOffVal + kWaves * 2 * CAPL * 32 * 4;
constexpr int kLdsBytes = kOffId + kWaves * 2 * CAPL * 32 * 2;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(1))) const void glb_cvoid;

// compile-time ablation masks of the tuning builds (0 in the product kernel)
constexpr int kNoHits = 1, kProfile = 16;

// kProfile build: cycles per phase, summed over the steps of wavefronts 0 and 4 of workgroup 0
__device__ unsigned long long s3_prof[32];

__device__ __forceinline__ void lds_store_f32(unsigned addr, float v) {
    asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_store_u16(unsigned addr, unsigned v) {
    asm volatile("ds_write_b16 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_store_u32(unsigned addr, unsigned v) {
    asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ unsigned lds_load_u32(unsigned addr) {
    unsigned v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(addr) : "memory");
    return v;
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

// Number of this token's candidates >= m (both lanes).  Ten compares into ten scalar masks, then ten
// add-with-carry on two alternating counters: written out so that no instruction waits for the one before it.
__device__ __forceinline__ int count_ge_regs(const float (&r)[CAPL], float m) {
    static_assert(CAPL % 10 == 0, "count_ge_regs works in blocks of ten");
    int c0 = 0, c1 = 0;
#pragma unroll
    for (int b = 0; b < CAPL; b += 10) {
        unsigned long long m0, m1, m2, m3, m4, m5, m6, m7, m8, m9;
        asm("v_cmp_ge_f32_e64 %2, %12, %22\n\t"
            "v_cmp_ge_f32_e64 %3, %13, %22\n\t"
            "v_cmp_ge_f32_e64 %4, %14, %22\n\t"
            "v_cmp_ge_f32_e64 %5, %15, %22\n\t"
            "v_cmp_ge_f32_e64 %6, %16, %22\n\t"
            "v_cmp_ge_f32_e64 %7, %17, %22\n\t"
            "v_cmp_ge_f32_e64 %8, %18, %22\n\t"
            "v_cmp_ge_f32_e64 %9, %19, %22\n\t"
            "v_cmp_ge_f32_e64 %10, %20, %22\n\t"
            "v_cmp_ge_f32_e64 %11, %21, %22\n\t"
            "v_addc_co_u32_e64 %0, vcc, 0, %0, %2\n\t"
            "v_addc_co_u32_e64 %1, vcc, 0, %1, %3\n\t"
            "v_addc_co_u32_e64 %0, vcc, 0, %0, %4\n\t"
            "v_addc_co_u32_e64 %1, vcc, 0, %1, %5\n\t"
            "v_addc_co_u32_e64 %0, vcc, 0, %0, %6\n\t"
            "v_addc_co_u32_e64 %1, vcc, 0, %1, %7\n\t"
            "v_addc_co_u32_e64 %0, vcc, 0, %0, %8\n\t"
            "v_addc_co_u32_e64 %1, vcc, 0, %1, %9\n\t"
            "v_addc_co_u32_e64 %0, vcc, 0, %0, %10\n\t"
            "v_addc_co_u32_e64 %1, vcc, 0, %1, %11"
            : "+v"(c0), "+v"(c1), "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6), "=&s"(m7),
              "=&s"(m8), "=&s"(m9)
            : "v"(r[b + 0]), "v"(r[b + 1]), "v"(r[b + 2]), "v"(r[b + 3]), "v"(r[b + 4]), "v"(r[b + 5]), "v"(r[b + 6]),
              "v"(r[b + 7]), "v"(r[b + 8]), "v"(r[b + 9]), "v"(m)
            : "vcc");
    }
    return pair_sum(c0 + c1);
}

struct Refreshed {
    int cnt;
    float tau;
    int passes;   // search passes taken (read by the profiling build only)
    unsigned t[4];   // profiling build: cycles of load / bracket / search / compaction
};

// Tighten tau of every token of the wavefront and compact the lists (slot i of this lane's list lives
// at cv[32 i] / ci[32 i]).  A token with >= k candidates ends with between k and `target` of them
// (exactly k when target == k), all >= the new tau; every dropped candidate is below k kept ones
// (ties: higher feature id).  Counts are over both lanes of the token.  Empty slots are held as -inf, which
// no candidate equals (pre-activations are finite).  The search for tau brackets the k-th largest value
// between lo (count >= k) and hi (count < k); it alternates interpolation on the logarithm of the counts
// (the upper tail of the candidates is close to exponential) with plain halving.  The compaction writes
// every element to the current end of the kept prefix and advances the end only past kept elements, so it
// has no branches.
template <bool PROF>
__device__ __attribute__((noinline)) Refreshed refresh_fast(lds_f32* cv, lds_u16* ci, int k, int target, int cnt, float tau) {
    Refreshed out;
    unsigned tp = PROF ? (unsigned)clock64() : 0u;
#define S3_RT(I) if (PROF) { const unsigned now_ = (unsigned)clock64(); out.t[I] = now_ - tp; tp = now_; }
    const int total = pair_sum(cnt);
    const bool active = total >= k;
    float r[CAPL];
    uint16_t ids[CAPL];
#pragma unroll
    for (int i = 0; i < CAPL; ++i) {
        float v = cv[32 * i];
        ids[i] = ci[32 * i];
        r[i] = i < cnt ? v : -INFINITY;
    }
    if (PROF) asm volatile("" ::"v"(r[CAPL - 1]), "v"(ids[CAPL - 1]));
    S3_RT(0)
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) mx = fmaxf(mx, r[i]);
    mx = pair_max(mx);
    float lo = tau;
    if (__any(active && !(tau > -INFINITY))) {    // no finite threshold yet: start from the smallest candidate
        float mn = INFINITY;
#pragma unroll
        for (int i = 0; i < CAPL; ++i) mn = fminf(mn, r[i] > -INFINITY ? r[i] : INFINITY);
        mn = pair_min(mn);
        if (!(tau > -INFINITY)) lo = mn;
    }
    float hi = nextafterf(mx, INFINITY);          // exclusive upper end of the bracket: no candidate is >= hi
    int clo = total, chi = 0;
    bool done = !active || clo <= target;
    bool split_failed = false;
    S3_RT(1)
    const float lwant = __log2f(0.5f * (float)(k + target));
    bool interp = true;
    int passes = 0;
    while (__any(!done)) {
        ++passes;
        const float llo = __log2f((float)clo), lhi = __log2f((float)max(chi, 1));
        const float t = fminf(fmaxf((llo - lwant) / (llo - lhi), 0.0625f), 0.9375f);
        float mid = lo + (hi - lo) * t;
        if (!interp || !(mid > lo && mid < hi)) mid = 0.5f * lo + 0.5f * hi;
        const bool can = (mid > lo) && (mid < hi);
        const int cm = count_ge_regs(r, mid);
        if (!done) {
            if (!can) { done = true; split_failed = true; }      // lo and hi are neighbouring floats
            else if (cm >= k) { lo = mid; clo = cm; if (clo <= target) done = true; }
            else { hi = mid; chi = cm; }
        }
        interp = !interp;
    }
    S3_RT(2)
    const bool tie = active && split_failed && clo > target;
    lds_f32* wv_ = cv;
    lds_u16* wi_ = ci;
    if (!__any(tie)) {
        const float cut = fmaxf(lo, -FLT_MAX);                   // empty slots never pass
#pragma unroll
        for (int i = 0; i < CAPL; ++i) {
            const bool keep = r[i] >= cut;
            *wv_ = r[i];
            *wi_ = ids[i];
            wv_ += keep ? 32 : 0;
            wi_ += keep ? 32 : 0;
        }
    } else {      // some token: every candidate in [lo, hi) equals lo; keep its tied ones with the lowest ids (rare)
        int cgt = 0;
#pragma unroll
        for (int i = 0; i < CAPL; ++i) cgt += (r[i] > lo) ? 1 : 0;
        cgt = pair_sum(cgt);
        const int need = k - cgt;
        int ilo = -1, ihi = 0xFFFF;
        for (int it = 0; it < 16; ++it) {
            const int mid = (ilo + ihi) >> 1;
            int ce = 0;
#pragma unroll
            for (int i = 0; i < CAPL; ++i) ce += (r[i] == lo && (int)ids[i] <= mid) ? 1 : 0;
            ce = pair_sum(ce);
            if (ce >= need) ihi = mid; else ilo = mid;
        }
        const int idcut = tie ? ihi : 0xFFFF;
        const float cut = fmaxf(lo, -FLT_MAX);
#pragma unroll
        for (int i = 0; i < CAPL; ++i) {
            const bool keep = r[i] >= cut && !(r[i] == lo && (int)ids[i] > idcut);
            *wv_ = r[i];
            *wi_ = ids[i];
            wv_ += keep ? 32 : 0;
            wi_ += keep ? 32 : 0;
        }
    }
    S3_RT(3)
#undef S3_RT
    out.cnt = (int)(wv_ - cv) >> 5;
    out.tau = active ? lo : tau;
    out.passes = passes;
    return out;
}

template <int ABL>
__global__ __launch_bounds__(kThreads) void sae_encode_topk_fast_kernel(EncParams p) {
    extern __shared__ __align__(16) char smem[];
    lds_char* const sm = (lds_char*)smem;                  // ring [kRing][32 rows][256 B] at 0, pieces xor-swizzled
    const unsigned sm_a = (unsigned)(uintptr_t)sm;
    const unsigned vote_a = sm_a + kOffVote;   // [4] refresh votes, slot = step & 3

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront index as a scalar: branches on it are uniform
    const int n = lane & 31, half = lane >> 5;
    int head, tt;
    s3_block_to_tile(blockIdx.x, p.n_heads, p.tiles_per_head, head, tt);
    int tok = tt * kTokWG + wv * 32 + n;
    bool tok_ok = tok < p.T;
    if (p.mode == 2) {      // redo pass: this workgroup's tokens come from the head's list (uniform early exit)
        const int rc = p.redo_cnt[head];
        if (tt * kTokWG >= rc) return;
        tok_ok = tok < rc;
        tok = tok_ok ? p.redo_list[(size_t)head * p.T + tok] : 0;
    }

    bf16x8 bfr[NS];
    {
        const char* row = p.x + ((size_t)head * p.T + (tok_ok ? tok : 0)) * RB;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint4 u = tok_ok ? *(const uint4*)(row + (16 * s + 8 * half) * 2) : make_uint4(0, 0, 0, 0);
            bfr[s] = __builtin_bit_cast(bf16x8, u);
        }
    }

    // this lane's list: slot i of the values at pv0 + 32 i floats, of the ids at pi0 + 32 i
    lds_f32* const pv0 = (lds_f32*)(sm + kOffVal) + (wv * 2 + half) * CAPL * 32 + n;
    lds_u16* const pi0 = (lds_u16*)(sm + kOffId) + (wv * 2 + half) * CAPL * 32 + n;
    const unsigned pv0a = (unsigned)(uintptr_t)pv0, pi0a = (unsigned)(uintptr_t)pi0;
    unsigned pv = pv0a, pi = pi0a;                                 // write pointers (LDS byte addresses)
    const unsigned pv_full = pv0a + (CAPL - kGuard) * 128;         // above this a group of 4 may not fit
    const unsigned pv_soft = pv0a + (p.soft > 0 ? p.soft : CAPL) * 128;                  // above this the lane asks for a voted refresh
    float tau = (ABL & kNoHits) ? INFINITY : -INFINITY;
    // |x| of the lane's token: the k-th largest pre-activation of a token scales with it, which makes the
    // previous chunk's smallest tau / |x| a useful starting threshold for this chunk's tokens
    float xnorm;
    {
        float ss = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const u32x4 u = __builtin_bit_cast(u32x4, bfr[s]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float lo = __uint_as_float(u[j] << 16), hi = __uint_as_float(u[j] & 0xFFFF0000u);
                ss += lo * lo + hi * hi;
            }
        }
        xnorm = sqrtf(pair_fsum(ss));
    }
    if (p.mode == 1 && !(ABL & kNoHits)) {
        // carried bounds, lowered by a margin (a bound that is still too high only costs a redo of that token)
        const float hr = p.hint_in[2 * head], ha = p.hint_in[2 * head + 1];
        const float tr = hr > -INFINITY ? hr * xnorm : -INFINITY;
        const float t0 = fmaxf(tr, ha);             // one of the two is -inf (see enc_stream_post_kernel)
        tau = t0 > -INFINITY ? t0 - p.margin * fabsf(t0) : -INFINITY;
    }
    if (!tok_ok) tau = INFINITY;      // lanes without a token (ragged last tile, short redo list) collect nothing
    const bool wave_active = __any(tok_ok);      // a wavefront without tokens only takes part in copies and barriers
    const int k = p.k;
    const int loose = min(k + (k >> 3) + 2, CAPL - kGuard);
    const int nst = p.n_feat / kFT;                                // a multiple of 4

    // ---- global -> LDS copy of one stage: wavefront w copies rows 4w .. 4w+3 (16 lanes per row); lane l
    // writes piece l of the wavefront's 1 KB, which must hold column piece (l & 15) xor (row & 15) of its row.
    // Every wavefront also copies the 64 biases of a pair of stages to the same place: the copies carry
    // identical bytes, and each wavefront only has to wait for its own.
    // A pair past the end is clamped to the last pair: the copy then lands in ring slots that are not read any more.
    const int crow = wv * 4 + (lane >> 4);
    const char* const wsrc = p.w + (size_t)head * p.n_feat * RB;
    const float* const bsrc = p.b + (size_t)head * p.n_feat;
    const unsigned wlane = (unsigned)(crow * RB + (((lane & 15) ^ (crow & 15)) << 4));
    const unsigned blane = (unsigned)(lane * 4);
    // stages J, J + 1 -> ring slots 2 Q, 2 Q + 1 and bias slot Q
#define S3_LOAD_PAIR(J, Q)                                                                                   \
    do {                                                                                                     \
        const int js_ = min((J), nst - 2);                                                                   \
        const char* ws_ = wsrc + (size_t)js_ * kStageB + wlane;                                              \
        __builtin_amdgcn_global_load_lds((glb_cvoid*)ws_, (lds_void*)(sm + (2 * (Q)) * kStageB + wv * 1024), 16, 0, 0); \
        __builtin_amdgcn_global_load_lds((glb_cvoid*)(ws_ + kStageB),                                        \
                                         (lds_void*)(sm + (2 * (Q) + 1) * kStageB + wv * 1024), 16, 0, 0);   \
        __builtin_amdgcn_global_load_lds((glb_cvoid*)((const char*)(bsrc + js_ * kFT) + blane),              \
                                         (lds_void*)(sm + kOffBias + (Q) * kBiasB), 4, 0, 0);                \
    } while (0)

    // ---- fragment addresses: lane (row n, half h) reads column piece 2s + h of its row in K step s;
    // its 16 accumulators are features q*8 + h*4 + 0..3 (q = 0..3) of the stage
    unsigned xo[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) xo[s] = sm_a + (unsigned)(n * RB + (((2 * s + half) ^ (n & 15)) << 4));
    const unsigned ba = sm_a + (unsigned)(kOffBias + half * 16);

    f32x16 acc0 = {}, acc1 = {};     // ping-pong: one is written by the MFMAs while the other one is compared
    unsigned long long hm[16];       // hit masks of the stage whose epilogue comes next
    // All LDS reads of a step in one statement that also waits for them: 4 x 16 B of biases, 8 x 16 B of W
    // fragments of ring slot BUF, and the vote slot of the previous step.  Declares the step's fragment
    // variables; S3_MFMAS consumes them (the bias vector is the first MFMA's C operand).
#define S3_BIAS_OFF(BUF) (((BUF) >> 1) * kBiasB + ((BUF) & 1) * 128)
#define S3_READS(BUF)                                                                                        \
    f32x4 c0_, c1_, c2_, c3_;                                                                                \
    u32x4 f0_, f1_, f2_, f3_, f4_, f5_, f6_, f7_;                                                            \
    unsigned vt_;                                                                                            \
    asm volatile(                                                                                            \
        "ds_read_b128 %0, %13 offset:%23\n\t"                                                                \
        "ds_read_b128 %1, %13 offset:%24\n\t"                                                                \
        "ds_read_b128 %2, %13 offset:%25\n\t"                                                                \
        "ds_read_b128 %3, %13 offset:%26\n\t"                                                                \
        "ds_read_b128 %4, %14 offset:%27\n\t"                                                                \
        "ds_read_b128 %5, %15 offset:%27\n\t"                                                                \
        "ds_read_b128 %6, %16 offset:%27\n\t"                                                                \
        "ds_read_b128 %7, %17 offset:%27\n\t"                                                                \
        "ds_read_b128 %8, %18 offset:%27\n\t"                                                                \
        "ds_read_b128 %9, %19 offset:%27\n\t"                                                                \
        "ds_read_b128 %10, %20 offset:%27\n\t"                                                               \
        "ds_read_b128 %11, %21 offset:%27\n\t"                                                               \
        "ds_read_b32 %12, %22 offset:%28\n\t"                                                                \
        "s_waitcnt lgkmcnt(0)"                                                                               \
        : "=&v"(c0_), "=&v"(c1_), "=&v"(c2_), "=&v"(c3_), "=&v"(f0_), "=&v"(f1_), "=&v"(f2_), "=&v"(f3_),    \
          "=&v"(f4_), "=&v"(f5_), "=&v"(f6_), "=&v"(f7_), "=&v"(vt_)                                         \
        : "v"(ba), "v"(xo[0]), "v"(xo[1]), "v"(xo[2]), "v"(xo[3]), "v"(xo[4]), "v"(xo[5]), "v"(xo[6]),       \
          "v"(xo[7]), "v"(vote_a), "n"(S3_BIAS_OFF(BUF)), "n"(S3_BIAS_OFF(BUF) + 32), "n"(S3_BIAS_OFF(BUF) + 64), \
          "n"(S3_BIAS_OFF(BUF) + 96), "n"((BUF) * kStageB), "n"(((((BUF) >> 1) ^ 1) & 1) * 4)                \
        : "memory");                                                                                         \
    S3_T(1)
    // MFMAs of a stage into ACC; the 16 compares of the previous stage's accumulators (PREV) sit between them:
    // they need no MFMA result of this chain, so they run while the wavefront would otherwise wait for it.
#define S3_MFMAS(ACC, PREV)                                                                                  \
    {                                                                                                        \
        f32x16 ci_ = __builtin_shufflevector(__builtin_shufflevector(c0_, c1_, 0, 1, 2, 3, 4, 5, 6, 7),      \
                                             __builtin_shufflevector(c2_, c3_, 0, 1, 2, 3, 4, 5, 6, 7),      \
                                             0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);          \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f0_), bfr[0], ci_, 0, 0, 0); \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f1_), bfr[1], ACC, 0, 0, 0); \
        S3_MASKS8(PREV, 0, "");                                                                              \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f2_), bfr[2], ACC, 0, 0, 0); \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f3_), bfr[3], ACC, 0, 0, 0); \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f4_), bfr[4], ACC, 0, 0, 0); \
        S3_MASKS8(PREV, 8, "");                                                                              \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f5_), bfr[5], ACC, 0, 0, 0); \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f6_), bfr[6], ACC, 0, 0, 0); \
        ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f7_), bfr[7], ACC, 0, 0, 0); \
    }

#define S3_REFRESH(TARGET)                                                                                   \
    do {                                                                                                     \
        const unsigned t0_ = (ABL & kProfile) ? (unsigned)clock64() : 0u;                                    \
        if (ABL & kProfile) napp += (pv - pv0a) >> 7;                                                        \
        Refreshed r_ = refresh_fast<(ABL & kProfile) != 0>(pv0, pi0, k, (TARGET), (int)(pv - pv0a) >> 7, tau);                      \
        if (ABL & kProfile) {                                                                                \
            napp -= r_.cnt;                                                                                  \
            prof[6] += (unsigned)clock64() - t0_;                                                            \
            prof[7] += 1 + (r_.passes << 16);                                                                \
            for (int i_ = 0; i_ < 4; ++i_) rprof[i_] += r_.t[i_];                                            \
        }                                                                                                    \
        tau = r_.tau;                                                                                        \
        pv = pv0a + r_.cnt * 128;                                                                            \
        pi = pi0a + r_.cnt * 64;                                                                             \
    } while (0)
    // The compiler does not see that the compares below read MFMA results: the wait states that an 8-pass
    // MFMA needs before a vector instruction may read its destination are spelled out.
#define S3_MFMA_NOPS "s_nop 7\n\ts_nop 4\n\t"
    // Hit masks of accumulators B0 .. B0+7 (one scalar 64-lane mask each), computed back to back so that the
    // branches below wait for no vector compare.
#define S3_MASKS8(ACC, B0, NOPS)                                                                                \
    asm volatile(NOPS "v_cmp_gt_f32_e64 %0, %8, %16\n\t"                                                                 \
        "v_cmp_gt_f32_e64 %1, %9, %16\n\t"                                                                   \
        "v_cmp_gt_f32_e64 %2, %10, %16\n\t"                                                                  \
        "v_cmp_gt_f32_e64 %3, %11, %16\n\t"                                                                  \
        "v_cmp_gt_f32_e64 %4, %12, %16\n\t"                                                                  \
        "v_cmp_gt_f32_e64 %5, %13, %16\n\t"                                                                  \
        "v_cmp_gt_f32_e64 %6, %14, %16\n\t"                                                                  \
        "v_cmp_gt_f32_e64 %7, %15, %16"                                                                      \
        : "=s"(hm[(B0) + 0]), "=s"(hm[(B0) + 1]), "=s"(hm[(B0) + 2]), "=s"(hm[(B0) + 3]), "=s"(hm[(B0) + 4]), \
          "=s"(hm[(B0) + 5]), "=s"(hm[(B0) + 6]), "=s"(hm[(B0) + 7])                                         \
        : "v"(ACC[(B0) + 0]), "v"(ACC[(B0) + 1]), "v"(ACC[(B0) + 2]), "v"(ACC[(B0) + 3]), "v"(ACC[(B0) + 4]), \
          "v"(ACC[(B0) + 5]), "v"(ACC[(B0) + 6]), "v"(ACC[(B0) + 7]), "v"(tau))
    // Accumulator R (feature fb + 8 (R / 4) + R % 4): skipped by a scalar branch when no lane of the wavefront
    // has a survivor; otherwise the lanes of its mask append (value, id), advance their write pointers and
    // record in `full` whether a list got too long.  The workgroup runs with all lanes enabled here.
#define S3_HIT(ACC, R)                                                                                       \
    if (__builtin_expect(hm[R] != 0, 0)) {                                                                   \
        unsigned t_;                                                                                         \
        asm volatile("s_mov_b64 exec, %[m]\n\t"                                                              \
                     "v_add_u32 %[t], %[c], %[fb]\n\t"                                                       \
                     "ds_write_b32 %[pv], %[a]\n\t"                                                          \
                     "ds_write_b16 %[pi], %[t]\n\t"                                                          \
                     "v_add_u32 %[pv], 0x80, %[pv]\n\t"                                                      \
                     "v_add_u32 %[pi], 64, %[pi]\n\t"                                                        \
                     "v_cmp_gt_u32 vcc, %[pv], %[lim]\n\t"                                                   \
                     "s_mov_b64 exec, -1\n\t"                                                                \
                     "s_or_b64 %[full], %[full], vcc"                                                        \
                     : [pv] "+v"(pv), [pi] "+v"(pi), [full] "+s"(full), [t] "=&v"(t_)                        \
                     : [m] "s"(hm[R]), [a] "v"(ACC[R]), [fb] "v"(fb), [c] "n"(8 * ((R) / 4) + (R) % 4),      \
                       [lim] "v"(pv_full)                                                                    \
                     : "vcc", "memory");                                                                     \
    }
    // Every lane has >= kGuard free slots at the start of a group of 4 accumulators.  The masks of later
    // groups were taken with the threshold before a refresh: they may name candidates below the new one,
    // which the next refresh drops.
#define S3_GROUP(ACC, G)                                                                                     \
    S3_HIT(ACC, 4 * (G) + 0) S3_HIT(ACC, 4 * (G) + 1) S3_HIT(ACC, 4 * (G) + 2) S3_HIT(ACC, 4 * (G) + 3)      \
    if (__builtin_expect(full != 0, 0)) {                                                                    \
        S3_REFRESH(loose);                                                                                   \
        full = 0;                                                                                            \
    }
    // Epilogue of stage ST in step JJ: refresh first if the workgroup voted for it in the previous step
    // (the vote slot then holds this step's number), and cast a vote for the next step if a list is long.
#define S3_VOTED_REFRESH(VT, PP)                                                                             \
    if (__builtin_expect(__builtin_amdgcn_readfirstlane((int)(VT)) == (PP), 0)) S3_REFRESH(loose);
#define S3_VOTE_CAST(PP)                                                                                     \
    if (__builtin_expect(__any(pv > pv_soft), 0)) lds_store_u32(vote_a + ((PP) & 1) * 4, (unsigned)((PP) + 1));
    // Appends of stage ST, whose accumulators are ACC and whose hit masks are in hm.
#define S3_HITS(ACC, ST)                                                                                     \
    do {                                                                                                     \
        S3_T(9)                                                                                              \
        const unsigned fb = (unsigned)((ST) * kFT + half * 4);                                               \
        S3_GROUP(ACC, 0) S3_GROUP(ACC, 1) S3_GROUP(ACC, 2) S3_GROUP(ACC, 3)                                  \
        S3_T(10)                                                                                             \
    } while (0)
    unsigned long long full = 0;
#define S3_T(I)                                                                                              \
    if (ABL & kProfile) {                                                                                    \
        const unsigned now_ = (unsigned)clock64();                                                           \
        prof[I] += now_ - tprev;                                                                             \
        tprev = now_;                                                                                        \
    }
    unsigned prof[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    unsigned rprof[4] = {0, 0, 0, 0};
    unsigned napp = 0;     // candidates this lane appended and later dropped
    unsigned tprev = (ABL & kProfile) ? (unsigned)clock64() : 0u;

    if (tid < 4) lds_store_u32(vote_a + tid * 4, 0xFFFFFFFFu);
    S3_LOAD_PAIR(0, 0);
    stage_barrier<0>();

    // Pair step P (stages 2P, 2P+1 in ring slots 2Q, 2Q+1 with Q = P & 1) starts the copy of the next pair into
    // the other two slots, runs MFMAs and epilogue of its two stages, waits for its copies and joins the barrier:
    // one barrier per 64 features, and a copy has a whole pair step to arrive.  A vote cast in pair step P
    // (slot P & 1 holds P + 1) makes every wavefront refresh at the start of pair step P + 1.
#define S3_PSTEP(Q)                                                                                          \
    {                                                                                                        \
        const int pp_ = (j >> 1) + (Q);                                                                      \
        S3_LOAD_PAIR(2 * pp_ + 2, (Q) ^ 1);                                                                  \
        S3_T(0)                                                                                              \
        if (wave_active) {                                                                                   \
            S3_READS(2 * (Q))                                                                                \
            S3_MFMAS(acc0, acc1)                                                                             \
            S3_T(2)                                                                                          \
            S3_VOTED_REFRESH(vt_, pp_)                                                                       \
            S3_T(8)                                                                                          \
            if ((Q) != 0 || j > 0) S3_HITS(acc1, 2 * pp_ - 1);                                               \
        }                                                                                                    \
        if (wave_active) {                                                                                   \
            S3_READS(2 * (Q) + 1)                                                                            \
            S3_MFMAS(acc1, acc0)                                                                             \
            S3_T(2)                                                                                          \
            S3_HITS(acc0, 2 * pp_);                                                                          \
            S3_VOTE_CAST(pp_)                                                                                \
        }                                                                                                    \
        S3_T(3)                                                                                              \
        stage_barrier<0>();                                                                                  \
        S3_T(4)                                                                                              \
    }
    for (int j = 0; j < nst; j += 4) { S3_PSTEP(0) S3_PSTEP(1) }
#undef S3_PSTEP
    S3_MASKS8(acc1, 0, S3_MFMA_NOPS);
    S3_MASKS8(acc1, 8, "");
    S3_HITS(acc1, nst - 1);
    stage_barrier<0>();          // no copy may be in flight when the workgroup ends; lists are complete
    S3_REFRESH(k);
    S3_T(5)
    if (ABL & kProfile) {
        napp += (pv - pv0a) >> 7;
        for (int d = 32; d > 0; d >>= 1) napp += __shfl_xor((int)napp, d);
        prof[5] = napp;    // appends of the whole wavefront (32 tokens)
    }
    if ((ABL & kProfile) && blockIdx.x == 0 && lane == 0 && (wv & 3) == 0) {
        for (int i = 0; i < 12; ++i) s3_prof[(wv >> 2) * 12 + i] = prof[i];
        if (wv == 0) for (int i = 0; i < 4; ++i) s3_prof[24 + i] = rprof[i];
    }

    const int cnt = (int)(pv - pv0a) >> 7;
    // A token that started from a carried bound and ends with fewer than k candidates is queued for the redo
    // pass (its rows are written there).  Every other token reports its final threshold: the minima over the
    // call (of tau / |x| and of tau) are the bounds carried to the next chunk.
    const bool failed = tok_ok && pair_sum(cnt) < k;
    if (p.mode != 0) {
        if (failed && half == 0) p.redo_list[(size_t)head * p.T + atomicAdd(&p.redo_cnt[head], 1)] = tok;
        float r = tok_ok && !failed && xnorm > 0.f ? tau / xnorm : INFINITY;
        float a = tok_ok && !failed ? tau : INFINITY;
#pragma unroll
        for (int d = 16; d > 0; d >>= 1) {
            r = fminf(r, __shfl_xor(r, d));
            a = fminf(a, __shfl_xor(a, d));
        }
        // sums of tau, |x| and the token count: they tell which of the two bounds was the tighter one on this call
        float s_tau = tok_ok && !failed && half == 0 ? tau : 0.f;
        float s_x = tok_ok && !failed && half == 0 ? xnorm : 0.f;
        float s_n = tok_ok && !failed && half == 0 ? 1.f : 0.f;
#pragma unroll
        for (int d = 16; d > 0; d >>= 1) {
            s_tau += __shfl_xor(s_tau, d);
            s_x += __shfl_xor(s_x, d);
            s_n += __shfl_xor(s_n, d);
        }
        if (lane == 0) {
            if (r < INFINITY) atomicMin(&p.hint_out[2 * head], ordered_key(r));
            if (a < INFINITY) atomicMin(&p.hint_out[2 * head + 1], ordered_key(a));
            if (s_n > 0.f) {
                atomicAdd(&p.hint_sum[3 * head], s_tau);
                atomicAdd(&p.hint_sum[3 * head + 1], s_x);
                atomicAdd(&p.hint_sum[3 * head + 2], s_n);
            }
        }
    }

    // bitonic sort of each token's k candidates: lanes 0-31 sort token 2 it, lanes 32-63 token 2 it + 1;
    // order (z descending, id ascending); lane e ends up with rank e.
    const lds_f32* const wcv = (lds_f32*)(sm + kOffVal) + wv * 2 * CAPL * 32;     // this wavefront's lists
    const lds_u16* const wci = (lds_u16*)(sm + kOffId) + wv * 2 * CAPL * 32;
    int32_t* ids_h = p.ids + (size_t)head * p.T * k;
    float* vals_h = p.vals + (size_t)head * p.T * k;
    const int wtok = tok_ok && !failed ? tok : -1;          // row this lane's token is written to
    for (int it = 0; it < 16; ++it) {
        const int t = 2 * it + half;
        const int trow = __shfl(wtok, t);
        if (!__any(trow >= 0)) continue;
        const int clo = __shfl(cnt, t), chi = __shfl(cnt, t + 32);
        const int e = n;
        const bool valid = e < clo + chi;
        const int slot = e < clo ? e : CAPL + (e - clo);
        const int el = (valid ? slot : 0) * 32 + t;
        unsigned kv = valid ? ordered_key(wcv[el]) : 0u;
        unsigned id = valid ? (unsigned)wci[el] : 0xFFFFu;
#pragma unroll
        for (int s = 2; s <= 32; s <<= 1) {
#pragma unroll
            for (int d = s >> 1; d > 0; d >>= 1) {
                unsigned pk = (unsigned)__shfl_xor((int)kv, d), pid = (unsigned)__shfl_xor((int)id, d);
                bool lower = (lane & d) == 0;
                bool dir = s == 32 ? true : ((lane & s) == 0);
                bool mine_before = kv > pk || (kv == pk && id < pid);
                bool keep = mine_before == (lower == dir);
                kv = keep ? kv : pk;
                id = keep ? id : pid;
            }
        }
        if (e < k && trow >= 0) {
            size_t o = (size_t)trow * k + e;
            ids_h[o] = (int32_t)id;
            vals_h[o] = fmaxf(key_value(kv), 0.f);
        }
    }
}

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
__global__ void enc_stream_post_kernel(const unsigned* hint_out, const float* hint_sum, float* hint, int n_heads) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= n_heads) return;
    const float r = hint_out[2 * h] == 0xFFFFFFFFu ? -INFINITY : key_value(hint_out[2 * h]);
    const float a = hint_out[2 * h + 1] == 0xFFFFFFFFu ? -INFINITY : key_value(hint_out[2 * h + 1]);
    const float s_tau = hint_sum[3 * h], s_x = hint_sum[3 * h + 1], s_n = hint_sum[3 * h + 2];
    const float waste_r = r > -INFINITY ? s_tau - r * s_x : INFINITY;
    const float waste_a = a > -INFINITY ? s_tau - a * s_n : INFINITY;
    const bool use_r = waste_r <= waste_a;
    hint[2 * h] = use_r ? r : -INFINITY;
    hint[2 * h + 1] = use_r ? -INFINITY : a;
}

template <int ABL>
int launch_fast(EncParams p, hipStream_t st) {
    auto kern = sae_encode_topk_fast_kernel<ABL>;
    static bool attr_set = false;
    if (!attr_set) {
        S3_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
        attr_set = true;
    }
    p.tiles_per_head = (p.T + kTokWG - 1) / kTokWG;
    p.capt = 2 * CAPL;
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.n_heads * p.tiles_per_head)), dim3(kThreads), kLdsBytes, st, p);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // namespace

bool s3_encode_fast_ok(int dtype, int d_head, int n_feat, int k) {
    return dtype == S3_BF16 && d_head == DH && k <= 32 && n_feat % (4 * kFT) == 0;
}

static int fast_dispatch(EncParams p, hipStream_t st);

int s3_encode_fast_launch(EncParams p, hipStream_t st) {
    p.mode = 0;
    p.hint_in = nullptr; p.hint_out = nullptr; p.hint_sum = nullptr; p.redo_list = nullptr; p.redo_cnt = nullptr;
    return fast_dispatch(p, st);
}

size_t s3_encode_fast_stream_workspace(int n_heads, int T) {
    return s3_align((size_t)n_heads * 4) + s3_align((size_t)n_heads * 8) + s3_align((size_t)n_heads * 12) +
           s3_align((size_t)n_heads * T * 4);
}

// Main pass from the carried bounds, redo pass (from -inf) for the tokens whose bound was too high, then this
// call's minima become the bounds for the next call.  All on `st`; nothing is read back.
int s3_encode_fast_stream(EncParams p, float* hint, void* ws, hipStream_t st) {
    char* base = (char*)ws;
    p.redo_cnt = (int32_t*)base;
    p.hint_out = (unsigned*)(base + s3_align((size_t)p.n_heads * 4));
    p.hint_sum = (float*)(base + s3_align((size_t)p.n_heads * 4) + s3_align((size_t)p.n_heads * 8));
    p.redo_list = (int32_t*)(base + s3_align((size_t)p.n_heads * 4) + s3_align((size_t)p.n_heads * 8) +
                             s3_align((size_t)p.n_heads * 12));
    p.hint_in = hint;
    const int nb = (3 * p.n_heads + 255) / 256;
    hipLaunchKernelGGL(enc_stream_prep_kernel, dim3(nb), dim3(256), 0, st, p.redo_cnt, p.hint_out, p.hint_sum, p.n_heads);
    p.margin = (float)env_int("S3_ENC_MARGIN", (int)(kHintMargin * 1000.f + 0.5f)) * 1e-3f;   // per mille, tuning
    p.mode = 1;
    int rc = fast_dispatch(p, st);
    if (rc) return rc;
    p.mode = 2;
    rc = fast_dispatch(p, st);
    if (rc) return rc;
    hipLaunchKernelGGL(enc_stream_post_kernel, dim3(nb), dim3(256), 0, st, p.hint_out, p.hint_sum, hint, p.n_heads);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

static int fast_dispatch(EncParams p, hipStream_t st) {
    static_assert(CAPL >= 32 + kGuard, "a lane must be able to hold k survivors and one more group");
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of one CU");
    p.soft = env_int("S3_ENC_SOFT", 33);                           // list length that asks for a voted refresh (0 = off)
    if (p.soft < 0 || p.soft > CAPL - kGuard) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: bad S3_ENC_SOFT");
    switch (p.ablate) {       // tuning builds: parts of the kernel compiled out (results are then meaningless)
        case 0: return launch_fast<0>(p, st);
        case 1: return launch_fast<kNoHits>(p, st);
        case 16: return launch_fast<kProfile>(p, st);
        case 17: return launch_fast<kProfile | kNoHits>(p, st);
    }
    return s3_fail(S3_EINVAL, "s3_sae_encode_topk: S3_ENC_ABLATE %d is not built", p.ablate);
}

// Tuning aid (not part of the public interface): phase cycle sums of the last S3_ENC_ABLATE=16/17 launch.
extern "C" int s3_debug_profile(unsigned long long* out32) {
    S3_HIP(hipDeviceSynchronize());
    S3_HIP(hipMemcpyFromSymbol(out32, HIP_SYMBOL(s3_prof), sizeof(unsigned long long) * 32));
    return S3_OK;
}
