// Fast path of the fused SAE encoder + Top-k (Sec. 3.3) for bf16 inputs and k <= 32.
//
// Same method as the generic kernel (features on the MFMA M axis, per-token threshold tau,
// candidate lists in LDS, exact selection), laid out for two wavefronts per SIMD:
//
//   - workgroup = 8 wavefronts = 256 tokens; a stage of 64 features (two 32x32 MFMA tiles per
//     wavefront) is staged once per workgroup through LDS, double-buffered, one barrier per stage;
//     global loads run two stages ahead in two alternating register sets;
//   - b_enc rides in the GEMM: each staged W row carries the bias split exactly into three bf16
//     terms in its 16-byte pad, multiplied by a constant [1, 1, 1, 0...] operand in a ninth K step,
//     so accumulators start from the literal 0 and no bias is read or added by the vector ALU;
//   - wavefronts 0-3 run [MFMA(j), epilogue(j)], wavefronts 4-7 run [epilogue(j-1), MFMA(j)]: the
//     two wavefronts that share a SIMD are half a stage apart, so one feeds the matrix pipe while
//     the other runs the compare/append epilogue on the vector ALU;
//   - the epilogue tests 4 accumulators per uniform branch; each lane owns a fixed list of CAPL
//     slots, so "list nearly full" is one compare on the lane's write pointer after a group that
//     appended;
//   - threshold refreshes are voted per workgroup at the stage barrier, so that all wavefronts
//     refresh in the same stage instead of stalling each other one after the other; the refresh
//     loads the lane's candidates into registers once and narrows tau there;
//   - the final k candidates of a token are sorted with a 32-lane bitonic network (two tokens per
//     wavefront step) and written coalesced.
#include "s3_common.h"

#include <math.h>

#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kTokWG = 256;
constexpr int kFT = 64;          // features per stage
constexpr int CAPL = 40;         // list slots per lane (a token has two lanes)
constexpr int kGuard = 4;        // appends possible between two fullness checks
constexpr int ES = 2;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef __attribute__((address_space(3))) int lds_i32;

// compile-time ablation masks of the tuning builds (0 in the product kernel)
constexpr int kNoHits = 1, kNoLoads = 2, kNoEpilogue = 4, kNoMfma = 8;

__device__ __forceinline__ unsigned ordered_key(float v) {
    unsigned u = __float_as_uint(v);
    return u ^ ((unsigned)((int)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_value(unsigned k) {
    return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// One lane's candidate list: slot i lives at cv[32 i] / ci[32 i] (LDS address space, so that the
// compiler emits ds_read/ds_write rather than flat accesses).
struct List {
    lds_f32* cv;
    lds_u16* ci;
};

__device__ __forceinline__ int count_ge_regs(const float (&r)[CAPL], float m) {
    int c = 0;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) c += (r[i] >= m) ? 1 : 0;
    return c + __shfl_xor(c, 32);
}

struct Refreshed {
    int cnt;
    float tau;
};

// Tighten tau of every token of the wavefront and compact the lists.  A token with >= k candidates
// ends with between k and `target` of them (exactly k when target == k), all >= the new tau; every
// dropped candidate is below k kept ones (ties: higher feature id).  Counts are over both lanes of
// the token.  The search for tau brackets the k-th largest value between lo (count >= k) and hi
// (count < k) and alternates interpolation on the counts with plain halving.
__device__ __noinline__ Refreshed refresh_fast(List L, int k, int target, int cnt, float tau) {
    const int total = cnt + __shfl_xor(cnt, 32);
    const bool active = total >= k;
    float r[CAPL];
    uint16_t ids[CAPL];
#pragma unroll
    for (int i = 0; i < CAPL; ++i) {
        float v = L.cv[32 * i];
        ids[i] = L.ci[32 * i];
        r[i] = i < cnt ? v : -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) mx = fmaxf(mx, r[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    float lo = tau;
    if (__any(active && !(tau > -INFINITY))) {    // no finite threshold yet: start from the smallest candidate
        float mn = INFINITY;
#pragma unroll
        for (int i = 0; i < CAPL; ++i) mn = fminf(mn, i < cnt ? r[i] : INFINITY);
        mn = fminf(mn, __shfl_xor(mn, 32));
        if (!(tau > -INFINITY)) lo = mn;
    }
    float hi = mx;
    int clo = total, chi;
    bool done = !active || clo <= target;
    bool split_failed = false;
    {
        chi = count_ge_regs(r, mx);
        if (!done && chi >= k) { lo = mx; clo = chi; done = true; split_failed = true; }
    }
    const float want = 0.5f * (float)(k + target);
    bool interp = true;
    while (__any(!done)) {
        float half_mid = 0.5f * lo + 0.5f * hi;
        float t = fminf(fmaxf(((float)clo - want) / (float)(clo - chi), 0.125f), 0.875f);
        float mid = lo + (hi - lo) * t;
        if (!interp || !(mid > lo && mid < hi)) mid = half_mid;
        bool can = (mid > lo) && (mid < hi);
        int cm = count_ge_regs(r, mid);
        if (!done) {
            if (!can) { done = true; split_failed = true; }      // lo and hi are neighbouring floats
            else if (cm >= k) { lo = mid; clo = cm; if (clo <= target) done = true; }
            else { hi = mid; chi = cm; }
        }
        interp = !interp;
    }
    bool tie = active && split_failed && clo > target;
    int idcut = 0xFFFF;
    if (__any(tie)) {     // every candidate in [lo, hi) equals lo: keep the tied ones with the lowest ids (rare)
        int cgt = 0;
#pragma unroll
        for (int i = 0; i < CAPL; ++i) cgt += (r[i] > lo) ? 1 : 0;
        cgt += __shfl_xor(cgt, 32);
        const int need = k - cgt;
        int ilo = -1, ihi = 0xFFFF;
        for (int it = 0; it < 16; ++it) {
            int mid = (ilo + ihi) >> 1;
            int ce = 0;
#pragma unroll
            for (int i = 0; i < CAPL; ++i) ce += (r[i] == lo && i < cnt && (int)ids[i] <= mid) ? 1 : 0;
            ce += __shfl_xor(ce, 32);
            if (ce >= need) ihi = mid; else ilo = mid;
        }
        idcut = ihi;
    }
    int jw = 0;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) {
        float v = r[i];
        bool keep = (v > lo || (v == lo && i < cnt)) && !(tie && v == lo && (int)ids[i] > idcut);
        if (keep) {
            L.cv[32 * jw] = v;
            L.ci[32 * jw] = ids[i];
            ++jw;
        }
    }
    Refreshed out;
    out.cnt = jw;
    out.tau = active ? lo : tau;
    return out;
}

// fp32 -> three bf16 terms whose sum is the input exactly (8 significant bits each, by truncation)
__device__ __forceinline__ uint2 split_bias(float b) {
    unsigned u0 = __float_as_uint(b) & 0xFFFF0000u;
    float r1 = b - __uint_as_float(u0);
    unsigned u1 = __float_as_uint(r1) & 0xFFFF0000u;
    float r2 = r1 - __uint_as_float(u1);
    unsigned u2 = __float_as_uint(r2) & 0xFFFF0000u;
    return make_uint2((u0 >> 16) | u1, u2 >> 16);
}

template <int DH, int ABL>
__global__ __launch_bounds__(kThreads) void sae_encode_topk_fast_kernel(EncParams p) {
    constexpr int NS = DH / 16;
    constexpr int RB = DH * ES;
    constexpr int ROWB = RB + 16;          // W row + 16-byte pad that carries the bias terms
    constexpr int VR = RB / 16;
    constexpr int NV = kFT * VR / kThreads;
    static_assert(kFT * VR % kThreads == 0, "a stage must divide evenly over the workgroup");

    extern __shared__ __align__(16) char smem[];
    char* wst = smem;                                              // [2][kFT][ROWB]
    lds_i32* vote = (lds_i32*)(smem + 2 * kFT * ROWB);             // [4] refresh votes, slot = step & 3
    float* cval_all = (float*)(smem + 2 * kFT * ROWB + 16);        // [kWaves][2 CAPL][32]
    uint16_t* cid_all = (uint16_t*)(cval_all + kWaves * 2 * CAPL * 32);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront index as a scalar: branches on it are uniform
    const int n = lane & 31, half = lane >> 5;
    int head, tt;
    s3_block_to_tile(blockIdx.x, p.n_heads, p.tiles_per_head, head, tt);
    const int tok = tt * kTokWG + wv * 32 + n;
    const bool tok_ok = tok < p.T;

    const char* wh = p.w + (size_t)head * p.n_feat * RB;
    const float* bh = p.b + (size_t)head * p.n_feat;

    bf16x8 bfr[NS];
    {
        const char* row = p.x + ((size_t)head * p.T + (tok_ok ? tok : 0)) * RB;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint4 u = tok_ok ? *(const uint4*)(row + (16 * s + 8 * half) * ES) : make_uint4(0, 0, 0, 0);
            bfr[s] = __builtin_bit_cast(bf16x8, u);
        }
    }
    // B operand of the bias step: the low lane of a token multiplies the three bias terms by 1, the high lane by 0
    const bf16x8 bones = __builtin_bit_cast(bf16x8, half ? make_uint4(0, 0, 0, 0) : make_uint4(0x3F803F80u, 0x00003F80u, 0, 0));

    float* const wcv = cval_all + wv * 2 * CAPL * 32;             // this wavefront's value / id arrays
    uint16_t* const wci = cid_all + wv * 2 * CAPL * 32;
    lds_f32* const pv0 = (lds_f32*)(wcv + half * CAPL * 32 + n);   // this lane's list = its write pointers' origin
    lds_u16* const pi0 = (lds_u16*)(wci + half * CAPL * 32 + n);
    List L;
    L.cv = pv0;
    L.ci = pi0;
    lds_f32* pv = pv0;
    lds_u16* pi = pi0;
    lds_f32* const pv_full = pv0 + (CAPL - kGuard) * 32;           // above this a group of 4 may not fit
    lds_f32* const pv_soft = pv0 + p.soft * 32;                    // above this the lane asks for a voted refresh
    float tau = (ABL & kNoHits) ? INFINITY : -INFINITY;
    const int k = p.k;
    const int loose = min(k + (k >> 3) + 2, CAPL - kGuard);
    const int nst = (p.n_feat + kFT - 1) / kFT;
    const int nfull = p.n_feat / kFT;                              // stages before this one have all kFT rows

    // global -> register -> LDS copy of one stage: NV 16-byte pieces per thread, wavefront 0 also one bias per lane
    int goff[NV], loff[NV], grow[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int v = tid + i * kThreads;
        grow[i] = v / VR;
        goff[i] = grow[i] * RB + (v % VR) * 16;
        loff[i] = grow[i] * ROWB + (v % VR) * 16;
    }
    // The stage loop is written with macros over plain local variables (no closures), so that every piece
    // of state stays in registers.
    //
    // Two register sets (A, B): stage s travels in set s & 1, is requested two steps before it is used and
    // written to LDS one step before, so a load has two whole steps to arrive.
    uint4 wA0, wA1, wB0, wB1;
    uint2 bA = make_uint2(0, 0), bB = make_uint2(0, 0);
    wA1 = wB1 = make_uint4(0, 0, 0, 0);

#define S3_GLOAD(J, W0, W1, BR)                                                                              \
    do {                                                                                                     \
        const int j_ = (J);                                                                                  \
        const char* base_ = wh + (size_t)j_ * kFT * RB;                                                      \
        if (j_ < nfull) { /* hot path: no predication */                                                     \
            W0 = *(const uint4*)(base_ + goff[0]);                                                           \
            if (NV > 1) W1 = *(const uint4*)(base_ + goff[NV - 1]);                                          \
            if (wv == 0) BR = split_bias(bh[j_ * kFT + lane]);                                               \
        } else { /* last, partial stage: missing rows are zero with bias -inf */                             \
            const int left_ = p.n_feat - j_ * kFT;                                                           \
            W0 = grow[0] < left_ ? *(const uint4*)(base_ + goff[0]) : make_uint4(0, 0, 0, 0);                \
            if (NV > 1) W1 = grow[NV - 1] < left_ ? *(const uint4*)(base_ + goff[NV - 1]) : make_uint4(0, 0, 0, 0); \
            if (wv == 0) BR = lane < left_ ? split_bias(bh[j_ * kFT + lane]) : make_uint2(0xFF80u, 0);       \
        }                                                                                                    \
    } while (0)

#define S3_SSTORE(BUF, W0, W1, BR)                                                                           \
    do {                                                                                                     \
        char* base_ = wst + (BUF) * kFT * ROWB;                                                              \
        *(uint4*)(base_ + loff[0]) = W0;                                                                     \
        if (NV > 1) *(uint4*)(base_ + loff[NV - 1]) = W1;                                                    \
        if (wv == 0) *(uint4*)(base_ + lane * ROWB + RB) = make_uint4(BR.x, BR.y, 0, 0);                     \
    } while (0)

    f32x16 acc0, acc1;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

#define S3_MMA(CUR)                                                                                          \
    do {                                                                                                     \
        if (ABL & kNoMfma) break;                                                                            \
        const char* a0_ = wst + ((CUR) * kFT + n) * ROWB;                                                    \
        const char* a1_ = a0_ + 32 * ROWB;                                                                   \
        {   /* bias terms: same address for both lanes of a token */                                         \
            uint4 g0_ = *(const uint4*)(a0_ + RB), g1_ = *(const uint4*)(a1_ + RB);                          \
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, g0_), bones, zero, 0, 0, 0); \
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, g1_), bones, zero, 0, 0, 0); \
        }                                                                                                    \
        _Pragma("unroll") for (int s = 0; s < NS; s += 2) {   /* two K steps at a time keeps few fragments live */ \
            uint4 f00_ = *(const uint4*)(a0_ + 16 * half + 32 * s);                                          \
            uint4 f10_ = *(const uint4*)(a1_ + 16 * half + 32 * s);                                          \
            uint4 f01_ = *(const uint4*)(a0_ + 16 * half + 32 * s + 32);                                     \
            uint4 f11_ = *(const uint4*)(a1_ + 16 * half + 32 * s + 32);                                     \
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f00_), bfr[s], acc0, 0, 0, 0); \
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f10_), bfr[s], acc1, 0, 0, 0); \
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f01_), bfr[s + 1], acc0, 0, 0, 0); \
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f11_), bfr[s + 1], acc1, 0, 0, 0); \
        }                                                                                                    \
    } while (0)

#define S3_REFRESH(TARGET)                                                                                   \
    do {                                                                                                     \
        Refreshed r_ = refresh_fast(L, k, (TARGET), (int)(pv - pv0) >> 5, tau);                              \
        tau = r_.tau;                                                                                        \
        pv = pv0 + r_.cnt * 32;                                                                              \
        pi = pi0 + r_.cnt * 32;                                                                              \
    } while (0)

#define S3_APPEND(H, A, IDV)                                                                                 \
    if (H) {                                                                                                 \
        *pv = (A);                                                                                           \
        *pi = (uint16_t)(IDV);                                                                               \
        pv += 32;                                                                                            \
        pi += 32;                                                                                            \
    }

    // Compare/append of one group of 4 accumulators (features FB + 0..3): one uniform branch skips it when
    // no lane of the wavefront has a survivor.  Every lane has >= kGuard free slots at the start of a group
    // (checked after each group that appended).  The id base is made opaque inside the branch so that ids
    // are formed only when something is appended.
#define S3_GROUP(A0, A1, A2, A3, FB)                                                                         \
    do {                                                                                                     \
        const float a0_ = (A0), a1_ = (A1), a2_ = (A2), a3_ = (A3);                                          \
        const bool h0_ = a0_ > tau, h1_ = a1_ > tau, h2_ = a2_ > tau, h3_ = a3_ > tau;                       \
        if (__any(h0_ || h1_ || h2_ || h3_)) {                                                               \
            unsigned idb_ = (FB);                                                                            \
            asm volatile("" : "+v"(idb_));                                                                   \
            S3_APPEND(h0_, a0_, idb_ + 0)                                                                    \
            S3_APPEND(h1_, a1_, idb_ + 1)                                                                    \
            S3_APPEND(h2_, a2_, idb_ + 2)                                                                    \
            S3_APPEND(h3_, a3_, idb_ + 3)                                                                    \
            if (__any(pv > pv_full)) S3_REFRESH(loose); /* emergency: a list may not take another group */   \
        }                                                                                                    \
    } while (0)

    // Epilogue of the stage whose first feature is F0; STEPNO = current step; VOTED: the workgroup agreed in
    // the previous step to refresh now.
#define S3_EPILOGUE(F0, STEPNO, VOTED)                                                                       \
    do {                                                                                                     \
        if (ABL & kNoEpilogue) {                                                                             \
            asm volatile("" ::"v"(acc0[0]), "v"(acc1[0]), "v"(acc0[15]), "v"(acc1[15]));                     \
            break;                                                                                           \
        }                                                                                                    \
        if (VOTED) S3_REFRESH(loose);                                                                        \
        const unsigned fb_ = (unsigned)((F0) + half * 4);                                                    \
        S3_GROUP(acc0[0], acc0[1], acc0[2], acc0[3], fb_ + 0);                                               \
        S3_GROUP(acc0[4], acc0[5], acc0[6], acc0[7], fb_ + 8);                                               \
        S3_GROUP(acc0[8], acc0[9], acc0[10], acc0[11], fb_ + 16);                                            \
        S3_GROUP(acc0[12], acc0[13], acc0[14], acc0[15], fb_ + 24);                                          \
        S3_GROUP(acc1[0], acc1[1], acc1[2], acc1[3], fb_ + 32);                                              \
        S3_GROUP(acc1[4], acc1[5], acc1[6], acc1[7], fb_ + 40);                                              \
        S3_GROUP(acc1[8], acc1[9], acc1[10], acc1[11], fb_ + 48);                                            \
        S3_GROUP(acc1[12], acc1[13], acc1[14], acc1[15], fb_ + 56);                                          \
        if (__any(pv > pv_soft) && lane == 0) vote[(STEPNO) & 3] = 1;                                        \
    } while (0)

    // One step of the stage loop.  CUR = step & 1 is a literal (the loop is unrolled by two); LATE selects
    // the order of MFMA and epilogue.  (WL*, BL) is the register set to load stage j + 2 into, (WS*, BS) the
    // set whose stage j + 1 is written to LDS.
#define S3_STEP(J, CUR, LATE, WL0, WL1, BL, WS0, WS1, BS)                                                    \
    do {                                                                                                     \
        const int js_ = (J);                                                                                 \
        if (!(ABL & kNoLoads) && js_ + 2 < nst) S3_GLOAD(js_ + 2, WL0, WL1, BL);                             \
        const int voted_ = (p.soft > 0 && js_ > 0) ? __builtin_amdgcn_readfirstlane(vote[(js_ - 1) & 3]) : 0; \
        if (tid == 0 && js_ > 1) vote[(js_ - 2) & 3] = 0;                                                    \
        if (!(LATE)) {                                                                                       \
            S3_MMA(CUR);                                                                                     \
            S3_EPILOGUE(js_* kFT, js_, voted_);                                                              \
        } else {                                                                                             \
            if (js_ > 0) S3_EPILOGUE((js_ - 1) * kFT, js_, voted_);                                          \
            S3_MMA(CUR);                                                                                     \
        }                                                                                                    \
        if (!(ABL & kNoLoads) && js_ + 1 < nst) S3_SSTORE((CUR) ^ 1, WS0, WS1, BS);                          \
        __syncthreads();                                                                                     \
    } while (0)

    if (tid < 4) vote[tid] = 0;
    S3_GLOAD(0, wA0, wA1, bA);
    S3_SSTORE(0, wA0, wA1, bA);
    if (nst > 1) S3_GLOAD(1, wB0, wB1, bB);
    __syncthreads();

    // Wavefronts 0-3 (early) handle stage j in step j; wavefronts 4-7 (late) run the epilogue of stage j - 1
    // first, so that the two wavefronts of a SIMD use the matrix pipe and the vector ALU at different times.
    if (wv < kWaves / 2) {
        for (int j = 0; j < nst; j += 2) {
            S3_STEP(j, 0, false, wA0, wA1, bA, wB0, wB1, bB);
            if (j + 1 < nst) S3_STEP(j + 1, 1, false, wB0, wB1, bB, wA0, wA1, bA);
        }
    } else {
        for (int j = 0; j < nst; j += 2) {
            S3_STEP(j, 0, true, wA0, wA1, bA, wB0, wB1, bB);
            if (j + 1 < nst) S3_STEP(j + 1, 1, true, wB0, wB1, bB, wA0, wA1, bA);
        }
        S3_EPILOGUE((nst - 1) * kFT, nst, 0);
    }

    // exactly k per token, then a bitonic sort of each token's k candidates: lanes 0-31 sort token 2 it,
    // lanes 32-63 token 2 it + 1; order (z descending, id ascending); lane e ends up with rank e.
    S3_REFRESH(k);
    const int cnt = (int)(pv - pv0) >> 5;
    int32_t* ids_h = p.ids + (size_t)head * p.T * k;
    float* vals_h = p.vals + (size_t)head * p.T * k;
    const int tok0 = tt * kTokWG + wv * 32;
    for (int it = 0; it < 16; ++it) {
        if (tok0 + 2 * it >= p.T) break;
        const int t = 2 * it + half;
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
        if (e < k && tok0 + t < p.T) {
            size_t o = (size_t)(tok0 + t) * k + e;
            ids_h[o] = (int32_t)id;
            vals_h[o] = fmaxf(key_value(kv), 0.f);
        }
    }
}

template <int DH, int ABL>
int launch_fast(EncParams p, hipStream_t st) {
    constexpr int ROWB = DH * ES + 16;
    const size_t lds = 2 * kFT * ROWB + 16 + (size_t)kWaves * 2 * CAPL * 32 * (sizeof(float) + sizeof(uint16_t));
    auto kern = sae_encode_topk_fast_kernel<DH, ABL>;
    static bool attr_set = false;
    if (!attr_set) {
        S3_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    p.tiles_per_head = (p.T + kTokWG - 1) / kTokWG;
    p.capt = 2 * CAPL;
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.n_heads * p.tiles_per_head)), dim3(kThreads), lds, st, p);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // namespace

int s3_encode_fast_launch(EncParams p, int d_head, hipStream_t st) {
    static_assert(CAPL >= 32 + kGuard, "a lane must be able to hold k survivors and one more group");
    p.soft = env_int("S3_ENC_SOFT", 33);                           // list length that asks for a voted refresh (0 = off)
    if (p.soft < 0 || p.soft > CAPL - kGuard) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: bad S3_ENC_SOFT");
    if (d_head == 64) return launch_fast<64, 0>(p, st);
    if (d_head != 128) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: unsupported d_head %d", d_head);
    switch (p.ablate) {       // tuning builds: parts of the kernel compiled out (results are then meaningless)
        case 0: return launch_fast<128, 0>(p, st);
        case 1: return launch_fast<128, kNoHits>(p, st);
        case 7: return launch_fast<128, kNoHits | kNoLoads | kNoEpilogue>(p, st);
        case 11: return launch_fast<128, kNoHits | kNoLoads | kNoMfma>(p, st);
        case 13: return launch_fast<128, kNoHits | kNoEpilogue | kNoMfma>(p, st);
        case 15: return launch_fast<128, 15>(p, st);
    }
    return s3_fail(S3_EINVAL, "s3_sae_encode_topk: S3_ENC_ABLATE %d is not built", p.ablate);
}
