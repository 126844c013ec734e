// One optimisation step of the Top-K SAE (Sec. 3.3: encoder, Top-K and decoder equations; App. B.3: Adam, batches of
// 4096 tokens, k = 128) on the mean squared reconstruction error, entirely on the GPU:
//
//   1. u = bf16(x - b_dec), bf16(W_enc)                       the encoder's operands in the inference path's format
//   2. (ids, zhat) = TopK(W_enc u + b_enc)                    the fused encoder of this library (s3_sae_encode_topk)
//   3. per token: xhat = zhat W_dec + b_dec, g = 2 (xhat - x) / (B d), dz = (g . W_dec[id]) [zhat > 0],
//      du = sum_i dz_i W_enc[id_i], and the token's part of the loss
//   4. inverted index of the batch: feature -> the (token, slot) pairs that selected it (s3_index_build on the
//      flattened ids, one posting per pair) -- the same structure the retrieval path builds, used here to turn the
//      scatter of the weight gradients into one ordered sum per feature
//   5. per feature: dW_dec[f] = sum zhat g_t, dW_enc[f] = sum dz u_t, db_enc[f] = sum dz over its postings, in
//      posting order (no atomics: the sums are the same from run to run)
//   6. db_dec = sum_t (g_t - du_t), loss = sum of the parts / (B d), both in a fixed order
//   7. Adam on all four parameter arrays
//
// The backward pass holds the selection fixed and treats the bf16 rounding of the encoder's operands as the identity.
#include "s3_common.h"

#include <math.h>

namespace {

constexpr int DH = 128;              // d_head of the fast encoder
constexpr int kTokThreads = 256;     // four tokens / four features per workgroup, one wavefront each
constexpr int kChunk = 32;           // tokens per partial column sum

__device__ __forceinline__ uint16_t bf16_rne(float v) {      // finite inputs
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Sum over the 64 lanes in a fixed order (lane shifts inside rows of 16, then across rows), returned to every lane.
#define S3_DPP_ADD(X, CTRL, ROWS) X += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(X), CTRL, ROWS, 0xf, false))
__device__ __forceinline__ float wave_sum(float x) {
    S3_DPP_ADD(x, 0x111, 0xf);
    S3_DPP_ADD(x, 0x112, 0xf);
    S3_DPP_ADD(x, 0x114, 0xf);
    S3_DPP_ADD(x, 0x118, 0xf);
    S3_DPP_ADD(x, 0x142, 0xa);
    S3_DPP_ADD(x, 0x143, 0xc);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
#undef S3_DPP_ADD

__global__ void tr_prep_kernel(const float* x, const float* b_dec, const float* w_enc, uint16_t* u_bf, uint16_t* w_bf,
                               int64_t n_x, int64_t n_w) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_x) u_bf[i] = bf16_rne(x[i] - b_dec[i & (DH - 1)]);
    if (i < n_w) w_bf[i] = bf16_rne(w_enc[i]);
}

struct TokArgs {
    const float* x;
    const float* w_dec;
    const float* b_dec;
    const uint16_t* w_bf;
    const int32_t* ids;
    const float* vals;
    float* g;
    float* dz;
    float* du;
    double* lossp;
    int B, k;
    float scale;          // 2 / (B d)
};

// Step 3: one wavefront per token; lane l holds columns 2 l and 2 l + 1.  The token's ids and values are read once
// (entry i in lane i % 64, register i / 64; k <= 128) and handed out by readlane, and the decoder rows are fetched
// four at a time, so that no load waits for the previous row's arithmetic; the sums keep the order of the entries.
__global__ __launch_bounds__(kTokThreads) void tr_token_kernel(TokArgs a) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (kTokThreads / 64) + (threadIdx.x >> 6);
    if (t >= a.B) return;
    const int32_t* __restrict__ ids = a.ids + (size_t)t * a.k;
    const float* __restrict__ vals = a.vals + (size_t)t * a.k;
    const float* __restrict__ w_dec = a.w_dec;
    const uint16_t* __restrict__ w_bf = a.w_bf;
    int my_id[2];
    float my_v[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = lane + 64 * r;
        my_id[r] = i < a.k ? ids[i] : 0;
        my_v[r] = i < a.k ? vals[i] : 0.f;
    }
    const float2 xv = *(const float2*)(a.x + (size_t)t * DH + 2 * lane);
    float2 acc = *(const float2*)(a.b_dec + 2 * lane);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int kk = min(a.k - 64 * r, 64);
        for (int i0 = 0; i0 < kk; i0 += 4) {
            float2 row[4];
            float v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {        // entries past the end repeat the group's first one with value 0
                const int i = i0 + q < kk ? i0 + q : i0;
                const int f = __builtin_amdgcn_readlane(my_id[r], i);
                v[q] = i0 + q < kk ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_v[r]), i)) : 0.f;
                row[q] = *(const float2*)(w_dec + (size_t)f * DH + 2 * lane);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc.x += v[q] * row[q].x;
                acc.y += v[q] * row[q].y;
            }
        }
    }
    const float rx = acc.x - xv.x, ry = acc.y - xv.y;
    const float part = wave_sum(rx * rx + ry * ry);
    if (lane == 0) a.lossp[t] = (double)part;
    const float gx = rx * a.scale, gy = ry * a.scale;
    *(float2*)(a.g + (size_t)t * DH + 2 * lane) = make_float2(gx, gy);
    float dux = 0.f, duy = 0.f;
    float* __restrict__ dz_out = a.dz + (size_t)t * a.k;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int kk = min(a.k - 64 * r, 64);
        for (int i0 = 0; i0 < kk; i0 += 4) {
            float2 row[4];
            uint32_t we[4];
            float v[4], dz[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = i0 + q < kk ? i0 + q : i0;
                const int f = __builtin_amdgcn_readlane(my_id[r], i);
                v[q] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_v[r]), i));
                row[q] = *(const float2*)(w_dec + (size_t)f * DH + 2 * lane);
                we[q] = *(const uint32_t*)(w_bf + (size_t)f * DH + 2 * lane);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {        // four independent reductions: their lane shifts interleave
                const float dot = wave_sum(gx * row[q].x + gy * row[q].y);
                dz[q] = (i0 + q < kk && v[q] > 0.f) ? dot : 0.f;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (lane == 0 && i0 + q < kk) dz_out[64 * r + i0 + q] = dz[q];
                dux += dz[q] * __uint_as_float(we[q] << 16);
                duy += dz[q] * __uint_as_float(we[q] & 0xFFFF0000u);
            }
        }
    }
    *(float2*)(a.du + (size_t)t * DH + 2 * lane) = make_float2(dux, duy);
}

struct FeatArgs {
    const int32_t* offsets;
    const int32_t* slots;
    const float* vals;
    const float* dz;
    const float* g;
    const uint16_t* u_bf;
    float* g_w_enc;
    float* g_b_enc;
    float* g_w_dec;
    int n_feat, k;
    uint32_t kinv;        // ceil(2^32 / k): slot / k for slot < 2^24
};

// Step 5: one wavefront per feature; its postings (flat slot = token * k + slot in the row, ascending) are taken 64 at
// a time -- each lane fetches one posting's scalars, then the wavefront walks them in order.
__global__ __launch_bounds__(kTokThreads) void tr_feature_kernel(FeatArgs a) {
    const int lane = threadIdx.x & 63;
    const int f = blockIdx.x * (kTokThreads / 64) + (threadIdx.x >> 6);
    if (f >= a.n_feat) return;
    const int beg = a.offsets[f], end = a.offsets[f + 1];
    float ex = 0.f, ey = 0.f, dx = 0.f, dy = 0.f, sb = 0.f;
    for (int j0 = beg; j0 < end; j0 += 64) {
        const int n = min(64, end - j0);
        int my_t = 0;
        float my_v = 0.f, my_dz = 0.f;
        if (lane < n) {
            const int s = a.slots[j0 + lane];
            my_t = a.k == 1 ? s : (int)(((uint64_t)(uint32_t)s * a.kinv) >> 32);
            my_v = a.vals[s];
            my_dz = a.dz[s];
        }
        for (int q0 = 0; q0 < n; q0 += 4) {      // four postings' rows in flight; the sums keep the posting order
            float2 gv[4];
            uint32_t uu[4];
            float v[4], dz[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {        // postings past the end repeat the last one with weights 0
                const int q = min(q0 + j, n - 1);
                const int t = __builtin_amdgcn_readlane(my_t, q);
                v[j] = q0 + j < n ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_v), q)) : 0.f;
                dz[j] = q0 + j < n ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_dz), q)) : 0.f;
                gv[j] = *(const float2*)(a.g + (size_t)t * DH + 2 * lane);
                uu[j] = *(const uint32_t*)(a.u_bf + (size_t)t * DH + 2 * lane);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                dx += v[j] * gv[j].x;
                dy += v[j] * gv[j].y;
                ex += dz[j] * __uint_as_float(uu[j] << 16);
                ey += dz[j] * __uint_as_float(uu[j] & 0xFFFF0000u);
                sb += dz[j];
            }
        }
    }
    *(float2*)(a.g_w_enc + (size_t)f * DH + 2 * lane) = make_float2(ex, ey);
    *(float2*)(a.g_w_dec + (size_t)f * DH + 2 * lane) = make_float2(dx, dy);
    if (lane == 0) a.g_b_enc[f] = sb;
}

// Step 6, first half: column sums of g - du and the loss parts of one chunk of tokens, rows in order.
__global__ __launch_bounds__(DH) void tr_colpart_kernel(const float* g, const float* du, const double* lossp, int B,
                                                        float* colpart, double* losspart) {
    const int c = threadIdx.x, t0 = blockIdx.x * kChunk, t1 = min(B, t0 + kChunk);
    float s = 0.f;
    for (int t = t0; t < t1; ++t) s += g[(size_t)t * DH + c] - du[(size_t)t * DH + c];
    colpart[(size_t)blockIdx.x * DH + c] = s;
    if (c == 0) {
        double l = 0.0;
        for (int t = t0; t < t1; ++t) l += lossp[t];
        losspart[blockIdx.x] = l;
    }
}
// second half: the chunks in order (eight loads in flight; the loss parts are summed by a wavefront of their own)
__global__ __launch_bounds__(2 * DH) void tr_colfin_kernel(const float* __restrict__ colpart, const double* __restrict__ losspart,
                                                           int nchunk, double inv_n, float* g_b_dec, float* loss_out) {
    const int c = threadIdx.x;
    if (c < DH) {
        float s = 0.f;
        for (int q0 = 0; q0 < nchunk; q0 += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = q0 + j < nchunk ? colpart[(size_t)(q0 + j) * DH + c] : 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        }
        g_b_dec[c] = s;
    } else if (c == DH) {
        double l = 0.0;
        for (int q0 = 0; q0 < nchunk; q0 += 8) {
            double v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = q0 + j < nchunk ? losspart[q0 + j] : 0.0;
#pragma unroll
            for (int j = 0; j < 8; ++j) l += v[j];
        }
        loss_out[0] = (float)(l * inv_n);
    }
}

struct AdamArgs {
    float* p[4];
    int64_t end[4];       // end of each parameter array in the packed order W_enc | b_enc | W_dec | b_dec
    const float* grad;
    float* m;
    float* v;
    float lr, b1, b2, eps, c1, c2;      // c1 = 1 - b1^t, c2 = 1 - b2^t
};

__global__ void tr_adam_kernel(AdamArgs a) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.end[3]) return;
    const int seg = i < a.end[0] ? 0 : (i < a.end[1] ? 1 : (i < a.end[2] ? 2 : 3));
    float* p = a.p[seg] + (i - (seg ? a.end[seg - 1] : 0));
    const float g = a.grad[i];
    const float m = a.b1 * a.m[i] + (1.f - a.b1) * g;
    const float v = a.b2 * a.v[i] + (1.f - a.b2) * g * g;
    a.m[i] = m;
    a.v[i] = v;
    *p -= a.lr * (m / a.c1) / (sqrtf(v / a.c2) + a.eps);
}

struct Layout {
    size_t u_bf, w_bf, ids, vals, part_ids, part_vals, g, dz, du, lossp, offsets, slots, grads, colpart, losspart, iws, total, iws_bytes;
};

Layout layout(int B, int n_feat, int k) {
    Layout L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += s3_align(bytes); return at; };
    const size_t P = 2 * (size_t)n_feat * DH + n_feat + DH;
    const int nchunk = (B + kChunk - 1) / kChunk;
    L.u_bf = take((size_t)B * DH * 2);
    L.w_bf = take((size_t)n_feat * DH * 2);
    L.ids = take((size_t)B * k * 4);
    L.vals = take((size_t)B * k * 4);
    const bool split = s3_encode_fast_split_pays(1, B, n_feat, k);     // the encoder then runs on two halves of the features
    L.part_ids = take(split ? (size_t)2 * B * k * 4 : 0);
    L.part_vals = take(split ? (size_t)2 * B * k * 4 : 0);
    L.g = take((size_t)B * DH * 4);
    L.dz = take((size_t)B * k * 4);
    L.du = take((size_t)B * DH * 4);
    L.lossp = take((size_t)B * 8);
    L.offsets = take((size_t)(n_feat + 1) * 4);
    L.slots = take((size_t)B * k * 4);
    L.grads = take(P * 4);
    L.colpart = take((size_t)nchunk * DH * 4);
    L.losspart = take((size_t)nchunk * 8);
    L.iws_bytes = s3_index_build_workspace(B * k, 1, n_feat);
    L.iws = take(L.iws_bytes);
    L.total = o;
    return L;
}

bool shape_ok(int B, int d_head, int n_feat, int k) {
    return d_head == DH && B >= 1 && k >= 1 && k <= n_feat && (int64_t)B * k <= (1 << 24) &&
           s3_encode_fast_ok(S3_BF16, d_head, n_feat, k) && n_feat <= S3_MAX_FEAT;
}

}  // namespace

extern "C" {

size_t s3_sae_train_workspace(int B, int d_head, int n_feat, int k) {
    if (!shape_ok(B, d_head, n_feat, k)) return 0;
    return layout(B, n_feat, k).total;
}

int s3_sae_train_step(const float* x, int B, int d_head, int n_feat, int k, float* w_enc, float* b_enc, float* w_dec,
                      float* b_dec, float* adam_m, float* adam_v, float lr, float beta1, float beta2, float eps,
                      int step, float* loss_out, int32_t* ids_out, float* grads_out, void* ws, size_t ws_bytes,
                      void* stream) {
    if (!shape_ok(B, d_head, n_feat, k))
        return s3_fail(S3_EINVAL, "s3_sae_train_step: B %d, d_head %d, n_feat %d, k %d not supported (d_head 128, "
                       "n_feat a multiple of 128, k <= 128, B * k <= 2^24)", B, d_head, n_feat, k);
    if (!x || !w_enc || !b_enc || !w_dec || !b_dec || !adam_m || !adam_v || !loss_out || !ws)
        return s3_fail(S3_EINVAL, "s3_sae_train_step: null pointer");
    if (step < 1 || !(lr >= 0.f) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f))
        return s3_fail(S3_EINVAL, "s3_sae_train_step: step %d, lr %g, beta1 %g, beta2 %g, eps %g out of range", step,
                       (double)lr, (double)beta1, (double)beta2, (double)eps);
    const Layout L = layout(B, n_feat, k);
    if (ws_bytes < L.total) return s3_fail(S3_ECAPACITY, "s3_sae_train_step: workspace %zu < %zu bytes", ws_bytes, L.total);
    if ((uintptr_t)ws & 255) return s3_fail(S3_EINVAL, "s3_sae_train_step: workspace must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    char* base = (char*)ws;
    uint16_t* u_bf = (uint16_t*)(base + L.u_bf);
    uint16_t* w_bf = (uint16_t*)(base + L.w_bf);
    int32_t* ids = ids_out ? ids_out : (int32_t*)(base + L.ids);
    float* vals = (float*)(base + L.vals);
    float* g = (float*)(base + L.g);
    float* dz = (float*)(base + L.dz);
    float* du = (float*)(base + L.du);
    double* lossp = (double*)(base + L.lossp);
    int32_t* offsets = (int32_t*)(base + L.offsets);
    int32_t* slots = (int32_t*)(base + L.slots);
    float* grads = grads_out ? grads_out : (float*)(base + L.grads);
    float* colpart = (float*)(base + L.colpart);
    double* losspart = (double*)(base + L.losspart);
    const int64_t n_x = (int64_t)B * DH, n_w = (int64_t)n_feat * DH;
    const int64_t n_max = n_x > n_w ? n_x : n_w;

    hipLaunchKernelGGL(tr_prep_kernel, dim3((unsigned)((n_max + 255) / 256)), dim3(256), 0, st, x, (const float*)b_dec,
                       (const float*)w_enc, u_bf, w_bf, n_x, n_w);
    int rc;
    if (s3_encode_fast_split_pays(1, B, n_feat, k)) {
        // one head and a few thousand tokens are too few token tiles for the chip: the features go in two halves
        EncParams p;
        p.x = (const char*)u_bf; p.w = (const char*)w_bf; p.b = b_enc; p.ids = ids; p.vals = vals;
        p.T = B; p.n_feat = n_feat; p.k = k; p.n_heads = 1; p.ablate = 0; p.fsplit = 1;
        rc = s3_encode_fast_split(p, (int32_t*)(base + L.part_ids), (float*)(base + L.part_vals), st);
    } else {
        rc = s3_sae_encode_topk(u_bf, S3_BF16, B, DH, w_bf, b_enc, n_feat, k, 1, ids, vals, stream);
    }
    if (rc) return rc;
    TokArgs ta{x, w_dec, b_dec, w_bf, ids, vals, g, dz, du, lossp, B, k, 2.0f / ((float)B * (float)DH)};
    hipLaunchKernelGGL(tr_token_kernel, dim3((unsigned)((B + 3) / 4)), dim3(kTokThreads), 0, st, ta);
    rc = s3_index_build(ids, nullptr, B * k, 1, n_feat, offsets, slots, base + L.iws, L.iws_bytes, stream);
    if (rc) return rc;
    float* g_w_enc = grads;
    float* g_b_enc = g_w_enc + n_w;
    float* g_w_dec = g_b_enc + n_feat;
    float* g_b_dec = g_w_dec + n_w;
    FeatArgs fa{offsets, slots, vals, dz, g, u_bf, g_w_enc, g_b_enc, g_w_dec, n_feat, k,
                k > 1 ? (uint32_t)(((1ull << 32) + (uint32_t)k - 1) / (uint32_t)k) : 0u};
    hipLaunchKernelGGL(tr_feature_kernel, dim3((unsigned)((n_feat + 3) / 4)), dim3(kTokThreads), 0, st, fa);
    const int nchunk = (B + kChunk - 1) / kChunk;
    hipLaunchKernelGGL(tr_colpart_kernel, dim3((unsigned)nchunk), dim3(DH), 0, st, (const float*)g, (const float*)du,
                       (const double*)lossp, B, colpart, losspart);
    hipLaunchKernelGGL(tr_colfin_kernel, dim3(1), dim3(2 * DH), 0, st, (const float*)colpart, (const double*)losspart, nchunk,
                       1.0 / ((double)B * DH), g_b_dec, loss_out);
    AdamArgs aa;
    aa.p[0] = w_enc; aa.p[1] = b_enc; aa.p[2] = w_dec; aa.p[3] = b_dec;
    aa.end[0] = n_w; aa.end[1] = n_w + n_feat; aa.end[2] = 2 * n_w + n_feat; aa.end[3] = 2 * n_w + n_feat + DH;
    aa.grad = grads; aa.m = adam_m; aa.v = adam_v;
    aa.lr = lr; aa.b1 = beta1; aa.b2 = beta2; aa.eps = eps;
    aa.c1 = (float)(1.0 - pow((double)beta1, (double)step));
    aa.c2 = (float)(1.0 - pow((double)beta2, (double)step));
    hipLaunchKernelGGL(tr_adam_kernel, dim3((unsigned)((aa.end[3] + 255) / 256)), dim3(256), 0, st, aa);
    S3_HIP(hipGetLastError());
    return S3_OK;
}

}  // extern "C"
