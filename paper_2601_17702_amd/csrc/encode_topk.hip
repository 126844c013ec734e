// Fused SAE encoder + Top-k for gfx950 (Sec. 3.3: encoder equation and Top-K equation).
//
// One workgroup = 4 wavefronts = 128 tokens of one (layer, head).  A wavefront keeps its 32
// tokens' vectors in registers as the MFMA B operand for the whole kernel and walks over the
// SAE features in tiles of 32 (the MFMA A operand, staged once per workgroup through LDS,
// double-buffered).  With features on the M axis of the 32x32 MFMA, all 16 accumulators of a
// lane belong to ONE token (column) and 16 different features, so the Top-k state is per lane:
//
//   - the accumulator is initialised with b_enc (bias costs nothing in the epilogue);
//   - a running threshold tau per token (a certified lower bound on its k-th largest
//     pre-activation so far); an accumulator survives only if z > tau (one compare);
//   - survivors are appended to a small per-token candidate list in LDS (value fp32 + feature id
//     u16); the two lanes that share a token push from the two ends of the same list;
//   - when a list may overflow, the wavefront tightens tau for all its tokens by bisection on
//     the value (count candidates >= mid across the two lanes) and compacts the lists;
//   - after the last tile the lists are reduced to exactly k entries (ties: lower feature id)
//     and written in (z descending, id ascending) order with ReLU applied.
//
// The dense pre-activations never leave registers.  Selection is exact: every element that is
// dropped is smaller than k candidates that are kept (or ties one with a lower id).
#include "s3_common.h"

#include <math.h>
#include <stdlib.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kTokWave = 32;
constexpr int kTokWG = kWaves * kTokWave;
constexpr int kFT = 32;           // features per tile (MFMA M)
constexpr int kHeadroom = 32;     // free list slots required at the start of a tile (16 per lane)

__device__ __forceinline__ int wave_max_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
    return v;
}

// Candidate list of one token: `capt` slots, slot s of token n lives at element s * 32 + n.
// The low lane of the token (half 0) fills slots 0, 1, ...; the high lane fills capt-1, capt-2, ...
struct Cand {
    float* cv;
    uint16_t* ci;
    int base, step;   // element index of this lane's entry i is base + i * step
};

__device__ __forceinline__ int count_ge(const Cand& c, int cnt, int maxc, float m) {
    int local = 0;
    for (int i = 0; i < maxc; ++i) {
        float v = (i < cnt) ? c.cv[c.base + i * c.step] : -INFINITY;
        local += (i < cnt && v >= m) ? 1 : 0;
    }
    return local + __shfl_xor(local, 32);
}

// Tighten tau and compact.  After the call every token that had >= k candidates holds between
// k and `target` of them (exactly k when target == k), all >= the new tau, and every dropped
// candidate is beaten by k kept ones.
__device__ void refresh(const Cand& c, int k, int target, int& cnt, float& tau) {
    const int maxc = wave_max_i(cnt);
    const int total = cnt + __shfl_xor(cnt, 32);
    const bool active = total >= k;

    float mn = INFINITY, mx = -INFINITY;
    for (int i = 0; i < maxc; ++i) {
        if (i < cnt) {
            float v = c.cv[c.base + i * c.step];
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
        }
    }
    mn = fminf(mn, __shfl_xor(mn, 32));
    mx = fmaxf(mx, __shfl_xor(mx, 32));

    // invariant: count(v >= lo) = clo >= k; count(v >= hi) < k or hi == lo
    float lo = mn, hi = mx;
    int clo = total;
    bool done = !active || clo <= target;
    bool split_failed = false;
    {
        int cm = count_ge(c, cnt, maxc, mx);
        if (!done && cm >= k) { lo = mx; clo = cm; done = true; split_failed = true; }   // the k best all equal the maximum
    }
    while (__any(!done)) {
        float mid = 0.5f * lo + 0.5f * hi;
        bool can = (mid > lo) && (mid < hi);
        int cm = count_ge(c, cnt, maxc, mid);
        if (!done) {
            if (!can) { done = true; split_failed = true; }
            else if (cm >= k) { lo = mid; clo = cm; if (clo <= target) done = true; }
            else hi = mid;
        }
    }
    // Ties: lo and hi are neighbouring floats, so every candidate in [lo, hi) equals lo.  Keep
    // only the `need` tied candidates with the lowest feature ids (bisection on the id).
    bool tie = active && split_failed && clo > target;
    int idcut = 0xFFFF;
    if (__any(tie)) {
        int cgt = 0;
        for (int i = 0; i < maxc; ++i) {
            float v = (i < cnt) ? c.cv[c.base + i * c.step] : -INFINITY;
            cgt += (i < cnt && v > lo) ? 1 : 0;
        }
        cgt += __shfl_xor(cgt, 32);
        const int need = k - cgt;
        int ilo = -1, ihi = 0xFFFF;                 // count(id <= ilo) < need <= count(id <= ihi)
        for (int it = 0; it < 16; ++it) {
            int mid = (ilo + ihi) >> 1;
            int ce = 0;
            for (int i = 0; i < maxc; ++i) {
                if (i < cnt) {
                    float v = c.cv[c.base + i * c.step];
                    int id = c.ci[c.base + i * c.step];
                    ce += (v == lo && id <= mid) ? 1 : 0;
                }
            }
            ce += __shfl_xor(ce, 32);
            if (ce >= need) ihi = mid; else ilo = mid;
        }
        idcut = ihi;
    }
    int jw = 0;
    for (int i = 0; i < maxc; ++i) {
        if (i < cnt) {
            float v = c.cv[c.base + i * c.step];
            uint16_t id = c.ci[c.base + i * c.step];
            bool keep = (v > lo) || (v == lo && (!tie || (int)id <= idcut));
            if (keep) {
                c.cv[c.base + jw * c.step] = v;
                c.ci[c.base + jw * c.step] = id;
                ++jw;
            }
        }
    }
    cnt = jw;
    if (active) tau = lo;
}

template <int DT, int DH>
struct Frag;

// bf16: 32x32x16 MFMA, K step s covers stored columns [16 s, 16 s + 16); lane half h owns 8 of them.
template <int DH>
struct Frag<S3_BF16, DH> {
    static constexpr int ES = 2;
    static constexpr int NS = DH / 16;
    bf16x8 b[NS];
    __device__ __forceinline__ void load_b(const char* row, bool ok, int half) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint4 u = ok ? *(const uint4*)(row + (16 * s + 8 * half) * ES) : make_uint4(0, 0, 0, 0);
            b[s] = __builtin_bit_cast(bf16x8, u);
        }
    }
    __device__ __forceinline__ void mma(const char* arow, int half, f32x16& acc) const {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint4 u = *(const uint4*)(arow + (16 * s + 8 * half) * ES);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, u), b[s], acc, 0, 0, 0);
        }
    }
};

// fp32: 32x32x2 MFMA, lane half h owns stored columns [h DH/2, (h+1) DH/2); step s uses column h DH/2 + s.
template <int DH>
struct Frag<S3_FP32, DH> {
    static constexpr int ES = 4;
    static constexpr int NS = DH / 2;
    float b[NS];
    __device__ __forceinline__ void load_b(const char* row, bool ok, int half) {
#pragma unroll
        for (int s = 0; s < NS; s += 4) {
            f32x4 u = ok ? *(const f32x4*)(row + (half * NS + s) * ES) : f32x4{0, 0, 0, 0};
            b[s] = u[0]; b[s + 1] = u[1]; b[s + 2] = u[2]; b[s + 3] = u[3];
        }
    }
    __device__ __forceinline__ void mma(const char* arow, int half, f32x16& acc) const {
#pragma unroll
        for (int s = 0; s < NS; s += 4) {
            f32x4 u = *(const f32x4*)(arow + (half * NS + s) * ES);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(u[e], b[s + e], acc, 0, 0, 0);
        }
    }
};

template <int DT, int DH>
__global__ __launch_bounds__(kThreads) void sae_encode_topk_kernel(EncParams p) {
    using F = Frag<DT, DH>;
    constexpr int ES = F::ES;
    constexpr int RB = DH * ES;            // bytes of one W row
    constexpr int ROWB = RB + 16;          // padded LDS row (conflict-free 16-byte reads)
    constexpr int VR = RB / 16;            // 16-byte vectors per row
    constexpr int NV = (kFT * VR + kThreads - 1) / kThreads;

    extern __shared__ __align__(16) char smem[];
    char* wst = smem;                                              // [2][kFT][ROWB]
    float* bst = (float*)(smem + 2 * kFT * ROWB);                  // [2][kFT]
    float* cval_all = bst + 2 * kFT;                               // [kWaves][capt][32]
    uint16_t* cid_all = (uint16_t*)(cval_all + kWaves * p.capt * 32);

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = lane & 31, half = lane >> 5;
    int head, tt;
    s3_block_to_tile(blockIdx.x, p.n_heads, p.tiles_per_head, head, tt);
    const int tok = tt * kTokWG + wv * kTokWave + n;
    const bool tok_ok = tok < p.T;

    const char* xh = p.x + (size_t)head * p.T * RB;
    const char* wh = p.w + (size_t)head * p.n_feat * RB;
    const float* bh = p.b + (size_t)head * p.n_feat;

    F frag;
    frag.load_b(xh + (size_t)(tok_ok ? tok : 0) * RB, tok_ok, half);

    Cand c;
    c.cv = cval_all + wv * p.capt * 32;
    c.ci = cid_all + wv * p.capt * 32;
    c.base = half ? (p.capt - 1) * 32 + n : n;
    c.step = half ? -32 : 32;
    int cnt = 0;
    float tau = p.ablate ? INFINITY : -INFINITY;
    const int k = p.k;
    const int loose = min(k + (k >> 3) + 2, p.capt - p.headroom);

    const int ntiles = (p.n_feat + kFT - 1) / kFT;
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

    gload(0);
    sstore(0);
    __syncthreads();

    for (int j = 0; j < ntiles; ++j) {
        const int cur = j & 1;
        if (j + 1 < ntiles) gload(j + 1);

        {   // make room: worst case every accumulator of the tile (headroom 32) or of its first half (headroom 16,
            // used for k > 64 where LDS is short) is appended: 16 or 8 per lane, two lanes per token
            int used = cnt + __shfl_xor(cnt, 32);
            if (__any(used > p.capt - p.headroom)) refresh(c, k, loose, cnt, tau);
        }

        f32x16 acc;
        {
            const float* bs = bst + cur * kFT + half * 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 bq = *(const f32x4*)(bs + q * 8);
                acc[q * 4 + 0] = bq[0]; acc[q * 4 + 1] = bq[1]; acc[q * 4 + 2] = bq[2]; acc[q * 4 + 3] = bq[3];
            }
        }
        frag.mma(wst + (cur * kFT + n) * ROWB, half, acc);

        const int fb = j * kFT + half * 4;
        int wp = c.base + cnt * c.step;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            float v = acc[r];
            if (v > tau) {
                c.cv[wp] = v;
                c.ci[wp] = (uint16_t)(fb + (r >> 2) * 8 + (r & 3));
                wp += c.step;
                ++cnt;
            }
        }
        {   // room for the second half (never short when the tile started with 32 free slots)
            int used = cnt + __shfl_xor(cnt, 32);
            if (__any(used > p.capt - 16)) {
                refresh(c, k, loose, cnt, tau);
                wp = c.base + cnt * c.step;
            }
        }
#pragma unroll
        for (int r = 8; r < 16; ++r) {
            float v = acc[r];
            if (v > tau) {
                c.cv[wp] = v;
                c.ci[wp] = (uint16_t)(fb + (r >> 2) * 8 + (r & 3));
                wp += c.step;
                ++cnt;
            }
        }

        if (j + 1 < ntiles) sstore(cur ^ 1);
        __syncthreads();
    }

    // exactly k per token, then rank them: one candidate per lane, rank = number of candidates that beat it
    refresh(c, k, k, cnt, tau);
    int32_t* ids_h = p.ids + (size_t)head * p.T * k;
    float* vals_h = p.vals + (size_t)head * p.T * k;
    const int tok0 = tt * kTokWG + wv * kTokWave;
    for (int nn = 0; nn < kTokWave; ++nn) {
        if (tok0 + nn >= p.T) break;
        const int clo = __builtin_amdgcn_readfirstlane(__shfl(cnt, nn));
        const int chi = __builtin_amdgcn_readfirstlane(__shfl(cnt, nn + 32));
        for (int c0 = 0; c0 < clo + chi; c0 += 64) {         // one candidate per lane, 64 at a time (k may exceed 64)
            const int ci = c0 + lane;
            const bool mine = ci < clo + chi;
            const int slot = ci < clo ? ci : p.capt - 1 - (ci - clo);
            float v = mine ? c.cv[slot * 32 + nn] : -INFINITY;
            int id = mine ? (int)c.ci[slot * 32 + nn] : 0x7FFFFFFF;
            int rank = 0;
            for (int q = 0; q < clo; ++q) {
                float vq = c.cv[q * 32 + nn];
                int iq = c.ci[q * 32 + nn];
                rank += (vq > v || (vq == v && iq < id)) ? 1 : 0;
            }
            for (int q = 0; q < chi; ++q) {
                float vq = c.cv[(p.capt - 1 - q) * 32 + nn];
                int iq = c.ci[(p.capt - 1 - q) * 32 + nn];
                rank += (vq > v || (vq == v && iq < id)) ? 1 : 0;
            }
            if (mine && rank < k) {
                size_t o = (size_t)(tok0 + nn) * k + rank;
                ids_h[o] = id;
                vals_h[o] = fmaxf(v, 0.f);
            }
        }
    }
}

template <int DT, int DH>
int launch(const EncParams& p, int n_heads, hipStream_t st) {
    using F = Frag<DT, DH>;
    constexpr int ROWB = DH * F::ES + 16;
    size_t lds = 2 * kFT * ROWB + 2 * kFT * sizeof(float) + (size_t)kWaves * p.capt * 32 * (sizeof(float) + sizeof(uint16_t));
    auto kern = sae_encode_topk_kernel<DT, DH>;
    static S3LdsOnce once;             // per instantiation: allow the full 160 KB of LDS
    if (int rc = s3_allow_lds(once, (const void*)kern, 160 * 1024)) return rc;
    if (lds > 160 * 1024) return s3_fail(S3_EINVAL, "s3_sae_encode_topk: candidate lists need %zu bytes of LDS", lds);
    dim3 grid((unsigned)(n_heads * p.tiles_per_head));
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, st, p);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // namespace

#ifdef S3_TUNING
int env_int(const char* name, int dflt) {
    const char* s = getenv(name);
    return s && *s ? atoi(s) : dflt;
}
#endif

static int encode_impl(const char* who, const void* x, int dtype, int T, int d_head, const void* w_enc, const float* b_enc,
                       int n_feat, int k, int n_heads, int32_t* ids, float* vals, float* tau_hint, void* ws,
                       size_t ws_bytes, void* stream) {
    if (!x || !w_enc || !b_enc || !ids || !vals) return s3_fail(S3_EINVAL, "%s: null pointer", who);
    if (dtype != S3_BF16 && dtype != S3_FP32) return s3_fail(S3_EINVAL, "%s: dtype must be S3_BF16 or S3_FP32", who);
    if (d_head != 64 && d_head != 128 && d_head != 256)
        return s3_fail(S3_EINVAL, "%s: d_head %d not in {64, 128, 256}", who, d_head);
    if (T < 0 || n_heads < 1) return s3_fail(S3_EINVAL, "%s: T %d / n_heads %d out of range", who, T, n_heads);
    if (n_feat < 1 || n_feat > S3_MAX_FEAT) return s3_fail(S3_EINVAL, "%s: n_feat %d not in [1, %d]", who, n_feat, S3_MAX_FEAT);
    if (k < 1 || k > n_feat || k > S3_MAX_K) return s3_fail(S3_EINVAL, "%s: k %d not in [1, min(n_feat, %d)]", who, k, S3_MAX_K);
    if (((uintptr_t)x | (uintptr_t)w_enc) & 15) return s3_fail(S3_EINVAL, "%s: x and w_enc must be 16-byte aligned", who);
    if ((int64_t)n_heads * ((T + kTokWG - 1) / kTokWG) > 0x7FFFFFFFLL) return s3_fail(S3_EINVAL, "%s: grid too large", who);
    if (tau_hint) {
        if (!ws) return s3_fail(S3_EINVAL, "%s: null workspace", who);
        if ((uintptr_t)ws & 255) return s3_fail(S3_EINVAL, "%s: workspace must be 256-byte aligned", who);
        const size_t need = s3_encode_fast_stream_workspace(n_heads, T);
        if (ws_bytes < need) return s3_fail(S3_ECAPACITY, "%s: workspace %zu < %zu bytes", who, ws_bytes, need);
    }
    if (T == 0) return S3_OK;

    EncParams p;
    p.x = (const char*)x; p.w = (const char*)w_enc; p.b = b_enc; p.ids = ids; p.vals = vals;
    p.T = T; p.n_feat = n_feat; p.k = k; p.n_heads = n_heads;
    p.ablate = 0;
    p.fsplit = 1;
    bool fast = s3_encode_fast_ok(dtype, d_head, n_feat, k);
#ifdef S3_TUNING
    p.ablate = env_int("S3_ENC_ABLATE", 0);
    if (env_int("S3_ENC_GENERIC", 0)) fast = false;
#endif
    hipStream_t st = (hipStream_t)stream;
    if (fast)
        return tau_hint ? s3_encode_fast_stream(p, tau_hint, ws, st) : s3_encode_fast_launch(p, st);
    p.tiles_per_head = (T + kTokWG - 1) / kTokWG;
    // list capacity per token: k survivors + headroom for a run of appends + room for new candidates between refreshes;
    // the headroom is a whole tile's worth (32) where that fits the LDS, else half a tile's (16, re-checked mid-tile)
    const size_t fixed_lds = 2 * kFT * ((size_t)d_head * (dtype == S3_BF16 ? 2 : 4) + 16) + 2 * kFT * sizeof(float);
    auto lists_fit = [&](int c) { return fixed_lds + (size_t)kWaves * c * 32 * 6 <= 160 * 1024; };
    p.headroom = k <= 64 && lists_fit(k + kHeadroom + (k <= 32 ? 16 : 32)) ? kHeadroom : 16;
    int capt = k + p.headroom + (k <= 32 ? 16 : 32);
#ifdef S3_TUNING
    capt = env_int("S3_ENC_CAPT", capt);
    if (capt < k + p.headroom + 4 || capt > 512) return s3_fail(S3_EINVAL, "%s: bad S3_ENC_CAPT %d", who, capt);
#endif
    p.capt = capt;
#define S3_CASE(DT, DH) if (dtype == DT && d_head == DH) return launch<DT, DH>(p, n_heads, st);
    S3_CASE(S3_BF16, 64) S3_CASE(S3_BF16, 128) S3_CASE(S3_BF16, 256)
    S3_CASE(S3_FP32, 64) S3_CASE(S3_FP32, 128) S3_CASE(S3_FP32, 256)
#undef S3_CASE
    return s3_fail(S3_EINVAL, "%s: unsupported configuration", who);
}

extern "C" int s3_sae_encode_topk(const void* x, int dtype, int T, int d_head, const void* w_enc,
                                  const float* b_enc, int n_feat, int k, int n_heads, int32_t* ids,
                                  float* vals, void* stream) {
    return encode_impl("s3_sae_encode_topk", x, dtype, T, d_head, w_enc, b_enc, n_feat, k, n_heads, ids, vals, nullptr,
                       nullptr, 0, stream);
}

extern "C" size_t s3_sae_encode_topk_stream_workspace(int n_heads, int T) {
    if (n_heads < 1 || T < 0) return 0;
    return s3_encode_fast_stream_workspace(n_heads, T);
}

extern "C" int s3_sae_encode_topk_stream(const void* x, int dtype, int T, int d_head, const void* w_enc,
                                         const float* b_enc, int n_feat, int k, int n_heads, int32_t* ids,
                                         float* vals, float* tau_hint, void* ws, size_t ws_bytes, void* stream) {
    if (!tau_hint) return s3_fail(S3_EINVAL, "s3_sae_encode_topk_stream: null tau_hint");
    return encode_impl("s3_sae_encode_topk_stream", x, dtype, T, d_head, w_enc, b_enc, n_feat, k, n_heads, ids, vals,
                       tau_hint, ws, ws_bytes, stream);
}
