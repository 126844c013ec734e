// Fast path of the fused SAE encoder + Top-k (Sec. 3.3) for bf16 inputs and k <= 32.
//
// Same method as the generic kernel (features on the MFMA M axis, per-token threshold tau,
// candidate lists in LDS, exact selection), laid out for two wavefronts per SIMD:
//
//   - workgroup = 8 wavefronts = 256 tokens; a stage of 64 features (two 32x32 MFMA tiles per
//     wavefront) is staged once per workgroup through LDS, double-buffered, one barrier per stage;
//   - wavefronts 0-3 run [MFMA(j), epilogue(j)], wavefronts 4-7 run [epilogue(j-1), MFMA(j)]: the
//     two wavefronts that share a SIMD are half a stage apart, so one feeds the matrix pipe while
//     the other runs the compare/append epilogue on the vector ALU;
//   - each lane owns a fixed list of CAPL slots (no sharing with the other lane of its token), so
//     the "list nearly full" test is one compare on the lane's write pointer every 4 accumulators;
//   - the threshold refresh loads the lane's candidates into registers once and bisects there;
//   - the final k candidates of a token are sorted with a 32-lane bitonic network (two tokens per
//     wavefront step) and written coalesced.
#include "s3_common.h"

#include <math.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

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

// One lane's candidate list: slot i at element e0 + 32 i of the wavefront's arrays.
struct List {
    float* cv;
    uint16_t* ci;
    int e0;
};

__device__ __forceinline__ int count_ge_regs(const float (&r)[CAPL], float m) {
    int c = 0;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) c += (r[i] >= m) ? 1 : 0;
    return c + __shfl_xor(c, 32);
}

// Tighten tau of every token of the wavefront and compact the lists (see the generic kernel for the
// invariants).  After the call a token that had >= k candidates holds between k and `target`.
struct Refreshed {
    int cnt;
    float tau;
};
__device__ __forceinline__ Refreshed refresh_fast(const List& L, int k, int target, int cnt, float tau) {
    const int total = cnt + __shfl_xor(cnt, 32);
    const bool active = total >= k;
    float r[CAPL];
#pragma unroll
    for (int i = 0; i < CAPL; ++i) {
        float v = L.cv[L.e0 + 32 * i];
        r[i] = i < cnt ? v : -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) mx = fmaxf(mx, r[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    float lo = tau;
    if (__any(active && !(tau > -INFINITY))) {    // first refresh of a token: start from its smallest candidate
        float mn = INFINITY;
#pragma unroll
        for (int i = 0; i < CAPL; ++i) mn = fminf(mn, i < cnt ? r[i] : INFINITY);
        mn = fminf(mn, __shfl_xor(mn, 32));
        if (!(tau > -INFINITY)) lo = mn;
    }
    float hi = mx;
    int clo = total;
    bool done = !active || clo <= target;
    bool split_failed = false;
    {
        int cm = count_ge_regs(r, mx);
        if (!done && cm >= k) { lo = mx; clo = cm; done = true; split_failed = true; }
    }
    while (__any(!done)) {
        float mid = 0.5f * lo + 0.5f * hi;
        bool can = (mid > lo) && (mid < hi);
        int cm = count_ge_regs(r, mid);
        if (!done) {
            if (!can) { done = true; split_failed = true; }
            else if (cm >= k) { lo = mid; clo = cm; if (clo <= target) done = true; }
            else hi = mid;
        }
    }
    bool tie = active && split_failed && clo > target;
    int idcut = 0xFFFF;
    if (__any(tie)) {     // keep only the tied candidates with the lowest ids (rare)
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
                    float v = L.cv[L.e0 + 32 * i];
                    int id = L.ci[L.e0 + 32 * i];
                    ce += (v == lo && id <= mid) ? 1 : 0;
                }
            }
            ce += __shfl_xor(ce, 32);
            if (ce >= need) ihi = mid; else ilo = mid;
        }
        idcut = ihi;
    }
    int jw = 0;
#pragma unroll
    for (int i = 0; i < CAPL; ++i) {
        float v = r[i];
        bool keep = v > lo || (v == lo && i < cnt);
        if (keep) {
            uint16_t id = L.ci[L.e0 + 32 * i];
            if (!(tie && v == lo && (int)id > idcut)) {
                L.cv[L.e0 + 32 * jw] = v;
                L.ci[L.e0 + 32 * jw] = id;
                ++jw;
            }
        }
    }
    Refreshed out;
    out.cnt = jw;
    out.tau = active ? lo : tau;
    return out;
}

template <int DH>
__global__ __launch_bounds__(kThreads) void sae_encode_topk_fast_kernel(EncParams p) {
    constexpr int NS = DH / 16;
    constexpr int RB = DH * ES;
    constexpr int ROWB = RB + 16;
    constexpr int VR = RB / 16;
    constexpr int NV = (kFT * VR + kThreads - 1) / kThreads;

    extern __shared__ __align__(16) char smem[];
    char* wst = smem;                                              // [2][kFT][ROWB]
    float* bst = (float*)(smem + 2 * kFT * ROWB);                  // [2][kFT]
    float* cval_all = bst + 2 * kFT;                               // [kWaves][2 CAPL][32]
    uint16_t* cid_all = (uint16_t*)(cval_all + kWaves * 2 * CAPL * 32);

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
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

    List L;
    L.cv = cval_all + wv * 2 * CAPL * 32;
    L.ci = cid_all + wv * 2 * CAPL * 32;
    L.e0 = half * CAPL * 32 + n;
    // write pointers (LDS address space) of the next free slot in the value / id arrays
    lds_f32* const pv0 = (lds_f32*)(L.cv + L.e0);
    lds_u16* const pi0 = (lds_u16*)(L.ci + L.e0);
    lds_f32* pv = pv0;
    lds_u16* pi = pi0;
    lds_f32* const pv_full = pv0 + (CAPL - kGuard) * 32;           // above this a group of 4 may not fit
    float tau = p.ablate ? INFINITY : -INFINITY;
    const int k = p.k;
    const int loose = min(k + (k >> 3) + 2, CAPL - kGuard);

    const int nst = (p.n_feat + kFT - 1) / kFT;
    uint4 wreg[NV];
    float breg = 0.f;

    auto gload = [&](int j) {
        const int f0 = j * kFT;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            int v = tid + i * kThreads;
            int row = v / VR, col = v - row * VR;
            bool ok = (v < kFT * VR) && (f0 + row < p.n_feat);
            wreg[i] = ok ? *(const uint4*)(wh + (size_t)(f0 + row) * RB + col * 16) : make_uint4(0, 0, 0, 0);
        }
        if (tid < kFT) breg = (f0 + tid < p.n_feat) ? bh[f0 + tid] : -INFINITY;
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            int v = tid + i * kThreads;
            int row = v / VR, col = v - row * VR;
            if (v < kFT * VR) *(uint4*)(wst + (buf * kFT + row) * ROWB + col * 16) = wreg[i];
        }
        if (tid < kFT) bst[buf * kFT + tid] = breg;
    };

    f32x16 acc0, acc1;
    auto mma = [&](int cur) {
        const float* bs = bst + cur * kFT + half * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f32x4 b0 = *(const f32x4*)(bs + q * 8);
            f32x4 b1 = *(const f32x4*)(bs + 32 + q * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) { acc0[q * 4 + e] = b0[e]; acc1[q * 4 + e] = b1[e]; }
        }
        const char* a0 = wst + (cur * kFT + n) * ROWB + 16 * half;
        const char* a1 = a0 + 32 * ROWB;
        uint4 f0[NS], f1[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            f0[s] = *(const uint4*)(a0 + 32 * s);
            f1[s] = *(const uint4*)(a1 + 32 * s);
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f0[s]), bfr[s], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f1[s]), bfr[s], acc1, 0, 0, 0);
        }
    };

    gload(0);
    sstore(0);
    __syncthreads();

    // Wavefronts 4-7 run half a stage behind wavefronts 0-3: in step j the early ones do MFMA(j) then the
    // epilogue of stage j, the late ones the epilogue of stage j-1 then MFMA(j).
    const bool late = wv >= kWaves / 2;
    for (int j = 0; j <= nst; ++j) {
        const int cur = j & 1;
        if (j + 1 < nst) gload(j + 1);
        if (!late && j < nst) mma(cur);
        if (late ? (j > 0) : (j < nst)) {
            // compare/append epilogue of one stage (8 groups of 4 accumulators); a full list restarts
            // the walk at the group that did not fit, after the threshold refresh
            const unsigned fb = (unsigned)((late ? j - 1 : j) * kFT + half * 4);
            int g0 = 0;
            for (;;) {
                bool need = false;
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    if (!need && g >= g0) {
                        if (__any(pv > pv_full)) {
                            need = true;
                            g0 = g;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                float v = g < 4 ? acc0[(g & 3) * 4 + e] : acc1[(g & 3) * 4 + e];
                                if (v > tau) {
                                    *pv = v;
                                    *pi = (uint16_t)(fb + (g >> 2) * 32 + (g & 3) * 8 + e);
                                    pv += 32;
                                    pi += 32;
                                }
                            }
                        }
                    }
                }
                if (!need) break;
                Refreshed r = refresh_fast(L, k, loose, (int)(pv - pv0) >> 5, tau);
                tau = r.tau;
                pv = pv0 + r.cnt * 32;
                pi = pi0 + r.cnt * 32;
            }
        }
        if (late && j < nst) mma(cur);
        if (j + 1 < nst) sstore(cur ^ 1);
        if (j < nst) __syncthreads();
    }

    // exactly k per token, then a bitonic sort of each token's k candidates: lanes 0-31 sort token 2 it,
    // lanes 32-63 token 2 it + 1; order (z descending, id ascending); lane e ends up with rank e.
    int cnt;
    {
        Refreshed r = refresh_fast(L, k, k, (int)(pv - pv0) >> 5, tau);
        cnt = r.cnt;
    }
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
        unsigned kv = valid ? ordered_key(L.cv[el]) : 0u;
        unsigned id = valid ? (unsigned)L.ci[el] : 0xFFFFu;
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
    const size_t lds = 2 * kFT * ROWB + 2 * kFT * sizeof(float) + (size_t)kWaves * 2 * CAPL * 32 * (sizeof(float) + sizeof(uint16_t));
    auto kern = sae_encode_topk_fast_kernel<DH>;
    static bool attr_set = false;
    if (!attr_set) {
        S3_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    if (lds > 160 * 1024) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: fast path needs %zu bytes of LDS", lds);
    p.tiles_per_head = (p.T + kTokWG - 1) / kTokWG;
    p.capt = 2 * CAPL;
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.n_heads * p.tiles_per_head)), dim3(kThreads), lds, st, p);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // namespace

int s3_encode_fast_launch(EncParams p, int d_head, hipStream_t st) {
    static_assert(CAPL >= 32 + 4 + kGuard, "a lane must be able to hold k survivors, the loose margin and one group");
    switch (d_head) {
        case 64: return launch_fast<64>(p, st);
        case 128: return launch_fast<128>(p, st);
    }
    return s3_fail(S3_EINVAL, "s3_sae_encode_topk: unsupported d_head %d", d_head);
}
