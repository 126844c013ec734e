// Fast path of the fused SAE encoder + Top-k (Sec. 3.3) for bf16 inputs and k <= 32.
//
// Same method as the generic kernel (features on the MFMA M axis, per-token threshold tau,
// candidate lists in LDS, exact selection), laid out for two wavefronts per SIMD:
//
//   - workgroup = 8 wavefronts = 256 tokens; a stage of 64 features (two 32x32 MFMA tiles per
//     wavefront) is staged once per workgroup through LDS, double-buffered, one barrier per stage;
//   - b_enc rides in the GEMM: each staged W row carries the bias split exactly into three bf16
//     terms in its 16-byte pad, multiplied by a constant [1, 1, 1, 0...] operand in a ninth K step,
//     so accumulators start from the literal 0 and no bias is read or added by the vector ALU;
//   - wavefronts 0-3 run [MFMA(j), epilogue(j)], wavefronts 4-7 run [epilogue(j-1), MFMA(j)]: the
//     two wavefronts that share a SIMD are half a stage apart, so one feeds the matrix pipe while
//     the other runs the compare/append epilogue on the vector ALU;
//   - the epilogue tests 4 accumulators per uniform branch; each lane owns a fixed list of CAPL
//     slots, so "list nearly full" is one compare on the lane's write pointer after a group that
//     appended;
//   - optimistic start: tau begins at mean + c * std of the token's first 64 pre-activations instead
//     of -inf.  This is only a guess: a token is accepted iff at least k of its pre-activations
//     exceeded tau (then nothing that was dropped can belong to its Top-k); if any token of the
//     workgroup fails the test, the workgroup runs again from tau = -inf;
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
__device__ __noinline__ Refreshed refresh_fast(List L, int k, int target, int cnt, float tau, unsigned long long* dbg) {
    const int total = cnt + __shfl_xor(cnt, 32);
    const bool active = total >= k;
    float r[CAPL];
#pragma unroll
    for (int i = 0; i < CAPL; ++i) {
        float v = L.cv[32 * i];
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
        if (dbg && (threadIdx.x & 63) == 0) atomicAdd(&dbg[5], 1ull);
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
            for (int i = 0; i < CAPL; ++i) {
                if (i < cnt) {
                    float v = L.cv[32 * i];
                    int id = L.ci[32 * i];
                    ce += (v == lo && id <= mid) ? 1 : 0;
                }
            }
            ce += __shfl_xor(ce, 32);
            if (ce >= need) ihi = mid; else ilo = mid;
        }
        idcut = ihi;
    }
    // compaction: all ids are fetched up front (one wait), then survivors are written back in order
    uint16_t ids[CAPL];
#pragma unroll
    for (int i = 0; i < CAPL; ++i) ids[i] = L.ci[32 * i];
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

template <int DH>
__global__ __launch_bounds__(kThreads) void sae_encode_topk_fast_kernel(EncParams p) {
    constexpr int NS = DH / 16;
    constexpr int RB = DH * ES;
    constexpr int ROWB = RB + 16;          // W row + 16-byte pad that carries the bias terms
    constexpr int VR = RB / 16;
    constexpr int NV = (kFT * VR + kThreads - 1) / kThreads;

    extern __shared__ __align__(16) char smem[];
    char* wst = smem;                                              // [2][kFT][ROWB]
    int* vote = (int*)(smem + 2 * kFT * ROWB);                     // [4] refresh votes (3 used, rotating)
    float* cval_all = (float*)(vote + 4);                          // [kWaves][2 CAPL][32]
    uint16_t* cid_all = (uint16_t*)(cval_all + kWaves * 2 * CAPL * 32);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront index as a scalar: branches on it are uniform
    const int n = lane & 31, half = lane >> 5;
    int head, tt;
    s3_block_to_tile(blockIdx.x, p.n_heads, p.tiles_per_head, head, tt);
    const int tok = tt * kTokWG + wv * 32 + n;
    const bool tok_ok = tok < p.T;

    const char* xh = p.x + (size_t)head * p.T * RB;
    const char* wh = p.w + (size_t)head * p.n_feat * RB;
    const float* bh = p.b + (size_t)head * p.n_feat;

    bf16x8 bfr[NS];
    {
        const char* row = xh + (size_t)(tok_ok ? tok : 0) * RB;
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
    lds_f32* const pv_full = pv0 + (CAPL - kGuard) * 32;           // above this a group of 4 may not fit
    lds_f32* const pv_soft = pv0 + p.soft * 32;                    // above this the lane asks for a voted refresh
    const int k = p.k;
    const int loose = min(k + (k >> 3) + 2, CAPL - kGuard);
    const int nst = (p.n_feat + kFT - 1) / kFT;
    // the second wavefront of each SIMD runs half a stage behind (which wavefronts share a SIMD: p.skew)
    const bool late = p.skew ? (wv & 1) : (wv >= kWaves / 2);

    // global -> register -> LDS copy of one stage: this thread's 16-byte pieces and (tid < kFT) one bias
    int goff[NV], loff[NV], grow[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int v = tid + i * kThreads;
        grow[i] = v < kFT * VR ? v / VR : 0x7FFFFFFF;
        int col = v % VR;
        goff[i] = grow[i] * RB + col * 16;
        loff[i] = grow[i] * ROWB + col * 16;
    }
    // Two register sets: stage s travels in set s & 1, is requested two steps before it is used and
    // written to LDS one step before, so a load has two whole steps to arrive.
    uint4 wset[2][NV];
    uint2 bset[2] = {make_uint2(0, 0), make_uint2(0, 0)};
    auto gload = [&](int j, uint4 (&wreg)[NV], uint2& breg) {
        const int left = p.n_feat - j * kFT;                      // rows of this stage that exist
        const char* base = wh + (size_t)j * kFT * RB;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            wreg[i] = grow[i] < left ? *(const uint4*)(base + goff[i]) : make_uint4(0, 0, 0, 0);
        if (tid < kFT) breg = tid < left ? split_bias(bh[j * kFT + tid]) : make_uint2(0xFF80u, 0);   // missing row: -inf
    };
    auto sstore = [&](int buf, const uint4 (&wreg)[NV], const uint2& breg) {
        char* base = wst + buf * kFT * ROWB;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (grow[i] != 0x7FFFFFFF) *(uint4*)(base + loff[i]) = wreg[i];
        if (tid < kFT) *(uint4*)(base + tid * ROWB + RB) = make_uint4(breg.x, breg.y, 0, 0);
    };

    f32x16 acc0, acc1;
    auto mma = [&](int cur) {
        const char* a0 = wst + (cur * kFT + n) * ROWB;
        const char* a1 = a0 + 32 * ROWB;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        uint4 f0[NS + 1], f1[NS + 1];
        f0[NS] = *(const uint4*)(a0 + RB);                        // bias terms (same address for both lanes of a token)
        f1[NS] = *(const uint4*)(a1 + RB);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            f0[s] = *(const uint4*)(a0 + 16 * half + 32 * s);
            f1[s] = *(const uint4*)(a1 + 16 * half + 32 * s);
        }
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f0[NS]), bones, zero, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f1[NS]), bones, zero, 0, 0, 0);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f0[s]), bfr[s], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f1[s]), bfr[s], acc1, 0, 0, 0);
        }
    };

    int cnt = 0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        lds_f32* pv = pv0;
        lds_u16* pi = pi0;
        float tau = p.ablate ? INFINITY : -INFINITY;
        bool guess = attempt == 0 && p.opt_c > 0.f && nst >= 4 && !p.ablate;    // optimistic start (first attempt only)
        if (tid < 4) vote[tid] = 0;
        gload(0, wset[0], bset[0]);
        sstore(0, wset[0], bset[0]);
        if (nst > 1) gload(1, wset[1], bset[1]);
        __syncthreads();

        // one step of the stage loop; PAR = j & 1 is a compile-time constant (the loop is unrolled by two)
        auto step = [&](const int j, auto par) {
            constexpr int cur = decltype(par)::value;
            if (j + 2 < nst && !(p.ablate & 2)) gload(j + 2, wset[cur], bset[cur]);
            // vote of the previous step (written before the last barrier); cleared two steps later
            const int voted = j > 0 ? __builtin_amdgcn_readfirstlane(vote[(j - 1) % 3]) : 0;
            if (tid == 0 && j > 1) vote[(j - 2) % 3] = 0;
            if (!late && j < nst && !(p.ablate & 8)) mma(cur);
            if (p.ablate & 4) {
                asm volatile("" ::"v"(acc0[0]), "v"(acc1[0]), "v"(acc0[15]), "v"(acc1[15]));
            } else if (late ? (j > 0) : (j < nst)) {
                if (guess) {    // the wavefront's first 64 pre-activations per token: tau = mean + c * std
                    float s1 = 0.f, s2 = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s1 += acc0[r] + acc1[r];
                        s2 = fmaf(acc0[r], acc0[r], fmaf(acc1[r], acc1[r], s2));
                    }
                    s1 += __shfl_xor(s1, 32);
                    s2 += __shfl_xor(s2, 32);
                    const float mean = s1 * (1.f / 64.f);
                    const float var = fmaxf(s2 * (1.f / 64.f) - mean * mean, 0.f);
                    const float t0 = mean + p.opt_c * sqrtf(var);
                    tau = (t0 == t0 && fabsf(t0) < INFINITY) ? t0 : -INFINITY;
                    guess = false;
                }
                if (voted && !p.ablate) {     // every wavefront of the workgroup refreshes in this step
                    if (p.dbg && lane == 0) atomicAdd(&p.dbg[1], 1ull);
                    Refreshed r = refresh_fast(L, k, loose, (int)(pv - pv0) >> 5, tau, p.dbg);
                    tau = r.tau;
                    pv = pv0 + r.cnt * 32;
                    pi = pi0 + r.cnt * 32;
                }
                // compare/append epilogue of one stage: 8 groups of 4 accumulators.  One uniform branch per
                // group skips it when no lane of the wavefront has a survivor.  Every lane has >= kGuard
                // free slots at the start of a group (checked after each group that appended).
                const unsigned fb = (unsigned)((late ? j - 1 : j) * kFT + half * 4);
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    const float a0 = g < 4 ? acc0[(g & 3) * 4 + 0] : acc1[(g & 3) * 4 + 0];
                    const float a1 = g < 4 ? acc0[(g & 3) * 4 + 1] : acc1[(g & 3) * 4 + 1];
                    const float a2 = g < 4 ? acc0[(g & 3) * 4 + 2] : acc1[(g & 3) * 4 + 2];
                    const float a3 = g < 4 ? acc0[(g & 3) * 4 + 3] : acc1[(g & 3) * 4 + 3];
                    const bool h0 = a0 > tau, h1 = a1 > tau, h2 = a2 > tau, h3 = a3 > tau;
                    if (__any(h0 || h1 || h2 || h3)) {
                        constexpr unsigned kIdBase = 0;
                        const unsigned idb = fb + (g >> 2) * 32 + (g & 3) * 8 + kIdBase;
                        if (h0) { *pv = a0; *pi = (uint16_t)(idb + 0); pv += 32; pi += 32; }
                        if (h1) { *pv = a1; *pi = (uint16_t)(idb + 1); pv += 32; pi += 32; }
                        if (h2) { *pv = a2; *pi = (uint16_t)(idb + 2); pv += 32; pi += 32; }
                        if (h3) { *pv = a3; *pi = (uint16_t)(idb + 3); pv += 32; pi += 32; }
                        if (__any(pv > pv_full)) {     // emergency: a list may not take another group
                            if (p.dbg && lane == 0) atomicAdd(&p.dbg[0], 1ull);
                            Refreshed r = refresh_fast(L, k, loose, (int)(pv - pv0) >> 5, tau, p.dbg);
                            tau = r.tau;
                            pv = pv0 + r.cnt * 32;
                            pi = pi0 + r.cnt * 32;
                        }
                    }
                }
                if (p.soft > 0 && __any(pv > pv_soft) && lane == 0) vote[j % 3] = 1;
            }
            if (late && j < nst && !(p.ablate & 8)) mma(cur);
            if (j + 1 < nst && !(p.ablate & 2)) sstore(cur ^ 1, wset[cur ^ 1], bset[cur ^ 1]);
            if (j < nst) __syncthreads();
        };
        for (int j = 0; j <= nst; j += 2) {
            step(j, std::integral_constant<int, 0>{});
            if (j + 1 <= nst) step(j + 1, std::integral_constant<int, 1>{});
        }

        // exactly k per token; a token with fewer than k candidates above its optimistic tau failed the guess
        Refreshed r = refresh_fast(L, k, k, (int)(pv - pv0) >> 5, tau, p.dbg);
        cnt = r.cnt;
        const int total = cnt + __shfl_xor(cnt, 32);
        const bool failed = tok_ok && total < k && !p.ablate;
        if (p.dbg) {
            if (failed && half == 0) atomicAdd(&p.dbg[2], 1ull);
            if (lane == 0) atomicAdd(&p.dbg[4], 1ull);
        }
        if (!__syncthreads_or(failed ? 1 : 0)) break;
    }

    // bitonic sort of each token's k candidates: lanes 0-31 sort token 2 it, lanes 32-63 token 2 it + 1;
    // order (z descending, id ascending); lane e ends up with rank e.
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

template <int DH>
int launch_fast(EncParams p, hipStream_t st) {
    constexpr int ROWB = DH * ES + 16;
    const size_t lds = 2 * kFT * ROWB + 4 * sizeof(int) + (size_t)kWaves * 2 * CAPL * 32 * (sizeof(float) + sizeof(uint16_t));
    auto kern = sae_encode_topk_fast_kernel<DH>;
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

// Tuning aid (not part of the public header): with S3_ENC_DBG=1 in the environment the fast kernel counts
// [0] emergency refreshes, [1] voted refreshes, [2] tokens whose optimistic start failed, [4] wavefront passes.
static unsigned long long* g_dbg = nullptr;

extern "C" int s3_debug_counters(unsigned long long* out8) {
    if (!g_dbg || !out8) return S3_EINVAL;
    if (hipDeviceSynchronize() != hipSuccess) return S3_EHIP;
    if (hipMemcpy(out8, g_dbg, 8 * sizeof(unsigned long long), hipMemcpyDeviceToHost) != hipSuccess) return S3_EHIP;
    if (hipMemset(g_dbg, 0, 8 * sizeof(unsigned long long)) != hipSuccess) return S3_EHIP;
    return S3_OK;
}

int s3_encode_fast_launch(EncParams p, int d_head, hipStream_t st) {
    p.dbg = nullptr;
    if (env_int("S3_ENC_DBG", 0)) {
        if (!g_dbg) {
            S3_HIP(hipMalloc(&g_dbg, 8 * sizeof(unsigned long long)));
            S3_HIP(hipMemset(g_dbg, 0, 8 * sizeof(unsigned long long)));
        }
        p.dbg = g_dbg;
    }
    static_assert(CAPL >= 32 + kGuard, "a lane must be able to hold k survivors and one more group");
    p.opt_c = 0.01f * (float)env_int("S3_ENC_OPT_C", 230);         // optimistic start: tau0 = mean + c * std
    p.skew = env_int("S3_ENC_SKEW", 1);
    p.soft = env_int("S3_ENC_SOFT", 33);                           // list length that asks for a voted refresh (0 = off)
    if (p.soft < 0 || p.soft > CAPL - kGuard) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: bad S3_ENC_SOFT");
    switch (d_head) {
        case 64: return launch_fast<64>(p, st);
        case 128: return launch_fast<128>(p, st);
    }
    return s3_fail(S3_EINVAL, "s3_sae_encode_topk: unsupported d_head %d", d_head);
}
