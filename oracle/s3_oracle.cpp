// CPU oracle for the S3-Attention hot path.  TEST INFRASTRUCTURE ONLY.
//
// Plain, slow, fp64, written straight from the paper's definitions so that it can be checked
// against the paper by eye.  It shares no code with the HIP library and is loaded only by the
// tests, by the smoke check and by the benchmark's cpu_baseline leg; the product path never
// calls it.  Every function below is pinned by CPU tests against closed forms, hand-computed
// cases, brute force and library routines (no function here is "parity unpinned").  Where the
// paper leaves a step open (the smoothing weights, the suppression rule, how a span grows), the
// reading taken is stated at the function.
//
// All pointers are host pointers.  bf16 inputs arrive as uint16 bit patterns and are widened
// exactly; nothing is rounded before the fp64 arithmetic.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <map>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

inline double widen(const void* p, int dtype, size_t i) {
    if (dtype == 1) return (double)((const float*)p)[i];
    uint32_t u = (uint32_t)((const uint16_t*)p)[i] << 16;   // bf16 -> fp32 is exact
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

struct Index {                                   // Sec. 3.4: inverted index I[f] -> positions
    std::map<int32_t, std::vector<int32_t>> lists;
    int64_t n_postings = 0;
};

}  // namespace

extern "C" {

// Sec. 3.3, encoder equation: z = W_enc (x - b_dec) + b_enc with b_dec folded into b_enc
// (b_enc_eff = b_enc - W_enc b_dec), then the Top-K equation.  Selection is made on the
// pre-activation z (full sort by z descending, feature id ascending on exact ties), so that a
// row always yields exactly k ids; the stored activation is ReLU(z).
//   x [T, d] and w [n_feat, d] in dtype (0 = bf16 bits, 1 = fp32), b [n_feat] fp32.
//   ids [T, k], vals [T, k] (ReLU(z) rounded to fp32), zsel [T, k] fp64 (may be null),
//   gap [T] fp64 (may be null): (z_(k) - z_(k+1)) / |z_(k)|, +inf when k == n_feat.
//   zdense [T, n_feat] fp64 (may be null).
int orc_encode_topk(const void* x, int dtype, int T, int d, const void* w, const float* b,
                    int n_feat, int k, int32_t* ids, float* vals, double* zsel, double* gap,
                    double* zdense) {
    if (T < 0 || d <= 0 || n_feat <= 0 || k <= 0 || k > n_feat) return -1;
    std::vector<double> wd((size_t)n_feat * d);
    for (size_t i = 0; i < wd.size(); ++i) wd[i] = widen(w, dtype, i);
#pragma omp parallel
    {
        std::vector<double> xr(d), z(n_feat);
        std::vector<int32_t> order(n_feat);
#pragma omp for schedule(dynamic, 8)
        for (int t = 0; t < T; ++t) {
            for (int c = 0; c < d; ++c) xr[c] = widen(x, dtype, (size_t)t * d + c);
            for (int f = 0; f < n_feat; ++f) {
                double acc = 0.0;
                const double* wf = &wd[(size_t)f * d];
                for (int c = 0; c < d; ++c) acc += xr[c] * wf[c];
                z[f] = acc + (double)b[f];
            }
            if (zdense) std::memcpy(zdense + (size_t)t * n_feat, z.data(), sizeof(double) * n_feat);
            for (int f = 0; f < n_feat; ++f) order[f] = f;
            std::sort(order.begin(), order.end(), [&](int32_t a, int32_t c) {
                if (z[a] != z[c]) return z[a] > z[c];
                return a < c;
            });
            for (int j = 0; j < k; ++j) {
                int32_t f = order[j];
                ids[(size_t)t * k + j] = f;
                vals[(size_t)t * k + j] = (float)std::max(z[f], 0.0);
                if (zsel) zsel[(size_t)t * k + j] = z[f];
            }
            if (gap) {
                if (k == n_feat) gap[t] = INFINITY;
                else {
                    double zk = z[order[k - 1]], zn = z[order[k]];
                    gap[t] = (zk - zn) / std::fabs(zk);
                }
            }
        }
    }
    return 0;
}

// Sec. 3.3, encoder equation at chosen entries only: z[t, j] = W_enc[ids[t, j]] . x[t] + b[ids[t, j]] (b_dec folded
// as above), fp64, channels ascending.  Lets a test look up the pre-activation of any feature of any row without
// the dense [T, n_feat] array.  ids [T, m] in [0, n_feat), z [T, m].
int orc_preact_at(const void* x, int dtype, int T, int d, const void* w, const float* b, int n_feat,
                  const int32_t* ids, int m, double* z) {
    if (T < 0 || d <= 0 || n_feat <= 0 || m < 0) return -1;
    for (size_t i = 0; i < (size_t)T * m; ++i)
        if (ids[i] < 0 || ids[i] >= n_feat) return -1;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < m; ++j) {
            const size_t f = (size_t)ids[(size_t)t * m + j];
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += widen(x, dtype, (size_t)t * d + c) * widen(w, dtype, f * d + c);
            z[(size_t)t * m + j] = acc + (double)b[f];
        }
    return 0;
}

// Sec. 3.4, index update equation: for every feature f in F_t, I[f] <- I[f] U {t}, tokens taken
// in the order given; positions are absolute.
void* orc_index_new(void) { return new Index(); }
void orc_index_free(void* h) { delete (Index*)h; }

int orc_index_append(void* h, const int32_t* ids, const int32_t* positions, int T, int k) {
    Index* ix = (Index*)h;
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            ix->lists[ids[(size_t)t * k + j]].push_back(positions[t]);
            ix->n_postings++;
        }
    return 0;
}

int64_t orc_index_postings(void* h) { return ((Index*)h)->n_postings; }

// Contiguous form of the same index (the paper's recommended production layout, Sec. 3.4
// "CPU Index Size"): lists concatenated by ascending feature id; offsets [n_feat + 1].
int orc_index_export(void* h, int n_feat, int32_t* offsets, int32_t* positions) {
    Index* ix = (Index*)h;
    int64_t o = 0;
    for (int f = 0; f < n_feat; ++f) {
        offsets[f] = (int32_t)o;
        auto it = ix->lists.find(f);
        if (it == ix->lists.end()) continue;
        for (int32_t p : it->second) positions[o++] = p;
    }
    offsets[n_feat] = (int32_t)o;
    for (auto& kv : ix->lists)
        if (kv.first < 0 || kv.first >= n_feat) return -1;
    return 0;
}

// App. D.2 / App. E: IDF(f) = 1 / (log(1 + freq(f)) + 1), natural log, freq = posting-list length.
double orc_idf(int64_t freq) { return 1.0 / (std::log(1.0 + (double)freq) + 1.0); }

// Sec. 3.5 scoring equation and App. D.2: S[t] += a_f^(Q) * IDF(f) for every position t in I[f],
// for every (query vector, slot) pair; pairs naming the same feature add up.  App. E's hard
// threshold: a feature with freq > max_freq is skipped (max_freq <= 0 disables the rule).
// Adds one (layer, head) index into S [L] (fp64); call once per head to sum over heads/layers.
int orc_score_accumulate(void* h, const int32_t* qids, const float* qvals, int nq, int k,
                         int32_t max_freq, double* S, int64_t L) {
    Index* ix = (Index*)h;
    for (int q = 0; q < nq; ++q)
        for (int j = 0; j < k; ++j) {
            int32_t f = qids[(size_t)q * k + j];
            auto it = ix->lists.find(f);
            if (it == ix->lists.end()) continue;
            int64_t freq = (int64_t)it->second.size();
            if (max_freq > 0 && freq > max_freq) continue;
            double wgt = (double)qvals[(size_t)q * k + j] * orc_idf(freq);
            for (int32_t p : it->second) {
                if (p < 0 || p >= L) return -1;
                S[p] += wgt;
            }
        }
    return 0;
}

// Sec. 3.5 "Adaptive Granularity", smoothing step, read as a box kernel of width span_len
// summed (not averaged) over valid windows only: W[s] = sum_{t=s}^{s+len-1} S[t],
// s in [0, L - len]; len is clamped to L.  Returns the number of windows.
int64_t orc_pool(const double* S, int64_t L, int span_len, double* W) {
    int64_t len = std::min<int64_t>(span_len, L);
    int64_t nw = L - len + 1;
    for (int64_t s = 0; s < nw; ++s) {
        double acc = 0.0;
        for (int64_t t = s; t < s + len; ++t) acc += S[t];
        W[s] = acc;
    }
    return nw;
}

// Sec. 3.5, peak selection with non-maximum suppression, read as: repeat top_b times -- take the
// best remaining window (ties -> smallest start); with nms, suppress every window overlapping it
// (|s' - s| < span_len).  Stops early when nothing is left.  Returns n_found.
int orc_topb(const double* W, int64_t nw, int span_len, int top_b, int nms, int32_t* starts,
             double* scores) {
    std::vector<char> dead(nw, 0);
    int found = 0;
    for (int r = 0; r < top_b; ++r) {
        int64_t best = -1;
        for (int64_t s = 0; s < nw; ++s)
            if (!dead[s] && (best < 0 || W[s] > W[best])) best = s;
        if (best < 0) break;
        starts[found] = (int32_t)best;
        scores[found] = W[best];
        ++found;
        if (nms) {
            for (int64_t s = std::max<int64_t>(0, best - span_len + 1);
                 s < std::min<int64_t>(nw, best + span_len); ++s)
                dead[s] = 1;
        } else {
            dead[best] = 1;
        }
    }
    return found;
}

// ---- the rest of Phase 2 and the set operations of Phase 3 (Sec. 3.5 "Adaptive Granularity", Sec. 3.6, Alg. 1) ----

// Smoothing kernels for the density curve.  The paper fixes only the sizes (App. B.3: 48, 8 for QA), not the
// weights; three shapes are offered, each normalised to sum 1 so that the curve stays in the units of S:
// kind 0 box (1/K each), 1 triangular (w_j proportional to min(j + 1, K - j)), 2 Gaussian centred at (K - 1) / 2
// with sigma = K / 6.
int orc_smoothing_kernel(int kind, int K, double* g) {
    if (K < 1 || kind < 0 || kind > 2) return -1;
    double sum = 0.0;
    for (int j = 0; j < K; ++j) {
        double v = 1.0;
        if (kind == 1) v = (double)std::min(j + 1, K - j);
        if (kind == 2) {
            const double u = ((double)j - 0.5 * (K - 1)) / ((double)K / 6.0);
            v = std::exp(-0.5 * u * u);
        }
        g[j] = v;
        sum += v;
    }
    for (int j = 0; j < K; ++j) g[j] /= sum;
    return 0;
}

// Alg. 1 Phase 2, S' <- Conv1D(S): D[t] = sum_j g[j] * S[t + j - floor(K / 2)], same length as S, zeros outside
// (tap floor(K / 2) sits on t; cross-correlation form, which equals convolution for the symmetric kernels above).
int orc_conv1d(const double* S, int64_t L, const double* g, int K, double* D) {
    if (L < 0 || K < 1) return -1;
    const int64_t c = K / 2;
    for (int64_t t = 0; t < L; ++t) {
        double acc = 0.0;
        for (int j = 0; j < K; ++j) {
            const int64_t u = t + j - c;
            if (u >= 0 && u < L) acc += g[j] * S[u];
        }
        D[t] = acc;
    }
    return 0;
}

// Alg. 1 Phase 2, NMS_Select(S', N): density peaks by greedy non-maximum suppression.  Repeat up to n_centers
// times: the largest remaining density (ties -> smallest position) becomes a centre if it is positive; every
// position within `radius` of it is suppressed.  Returns the number of centres.
int orc_nms_peaks(const double* D, int64_t L, int n_centers, int radius, int32_t* centers, double* peak) {
    std::vector<char> dead(L, 0);
    int found = 0;
    for (int r = 0; r < n_centers; ++r) {
        int64_t best = -1;
        for (int64_t t = 0; t < L; ++t)
            if (!dead[t] && (best < 0 || D[t] > D[best])) best = t;
        if (best < 0 || !(D[best] > 0.0)) break;
        centers[found] = (int32_t)best;
        peak[found] = D[best];
        ++found;
        for (int64_t t = std::max<int64_t>(0, best - radius); t <= std::min<int64_t>(L - 1, best + radius); ++t) dead[t] = 1;
    }
    return found;
}

// Sec. 3.5: "for each peak, we retrieve a variable-length span", read as the region around the centre where the
// density stays at or above rel * D[centre] (the cut falls where the evidence thins out), at most max_half
// positions to either side: lo and hi are inclusive.
void orc_grow_span(const double* D, int64_t L, int32_t c, double rel, int max_half, int32_t* lo, int32_t* hi) {
    const double thr = rel * D[c];
    int64_t a = c, b = c;
    while (a - 1 >= 0 && c - (a - 1) <= max_half && D[a - 1] >= thr) --a;
    while (b + 1 < L && (b + 1) - c <= max_half && D[b + 1] >= thr) ++b;
    *lo = (int32_t)a;
    *hi = (int32_t)b;
}

// Sec. 3.6 / Alg. 1 Phase 3: Idx_final = Idx_S3 U Idx_lexical U LeadTail as a set of positions: the union of the
// spans [lo_i, hi_i], of an externally supplied index list (positions outside [0, L) are ignored) and of the first
// `lead` and last `tail` positions.  mask [L] gets 0 / 1; idx gets the selected positions in ascending order.
// Returns their number.
int64_t orc_fuse(int64_t L, const int32_t* lo, const int32_t* hi, int n_spans, const int32_t* extra, int64_t n_extra,
                 int lead, int tail, unsigned char* mask, int32_t* idx) {
    for (int64_t t = 0; t < L; ++t) mask[t] = 0;
    for (int i = 0; i < n_spans; ++i)
        for (int64_t t = std::max<int64_t>(lo[i], 0); t <= std::min<int64_t>(hi[i], L - 1); ++t) mask[t] = 1;
    for (int64_t i = 0; i < n_extra; ++i)
        if (extra[i] >= 0 && extra[i] < L) mask[extra[i]] = 1;
    for (int64_t t = 0; t < std::min<int64_t>(lead, L); ++t) mask[t] = 1;
    for (int64_t t = std::max<int64_t>(0, L - tail); t < L; ++t) mask[t] = 1;
    int64_t n = 0;
    for (int64_t t = 0; t < L; ++t)
        if (mask[t]) idx[n++] = (int32_t)t;
    return n;
}

// ---- compact postings (Sec. 3.4 "CPU Index Size": contiguous integer arrays with delta encoding and optional
// stop-feature pruning) ----
// The form taken here: positions are cut into blocks of 2^block_log2; a posting is stored as its 16-bit offset
// from the start of its block (the delta against the block base), and the postings are ordered block by block, inside a
// block list by list (ascending feature id), inside a list in list order.  cstart [nblk * n_feat + 1] gives where the
// segment of (block b, feature f) starts (entry b * n_feat + f; the next entry is its end); cfreq [n_feat] is the
// length of each list that was kept.  A list longer than prune_freq is dropped whole when prune_freq > 0 (stop
// feature).  Lists must ascend in position and lie below nblk << block_log2.  Returns the number of postings
// kept, or -1 if a list does not ascend / leaves the range.
int64_t orc_compact_encode(const int32_t* offsets, const int32_t* positions, int n_feat, int nblk, int block_log2,
                           int32_t prune_freq, int32_t* cstart, uint16_t* delta, int32_t* cfreq) {
    if (block_log2 < 1 || block_log2 > 16 || nblk < 1) return -1;
    int64_t o = 0;
    for (int f = 0; f < n_feat; ++f) {
        const int32_t len = offsets[f + 1] - offsets[f];
        cfreq[f] = (prune_freq > 0 && len > prune_freq) ? 0 : len;
        for (int32_t i = offsets[f]; i < offsets[f + 1]; ++i) {
            if (positions[i] < 0 || (positions[i] >> block_log2) >= nblk) return -1;
            if (i > offsets[f] && positions[i] <= positions[i - 1]) return -1;
        }
    }
    for (int b = 0; b < nblk; ++b)
        for (int f = 0; f < n_feat; ++f) {
            cstart[(size_t)b * n_feat + f] = (int32_t)o;
            if (cfreq[f] == 0) continue;
            for (int32_t i = offsets[f]; i < offsets[f + 1]; ++i)
                if ((positions[i] >> block_log2) == b) delta[o++] = (uint16_t)(positions[i] - (b << block_log2));
        }
    cstart[(size_t)nblk * n_feat] = (int32_t)o;
    return o;
}

// The inverse: plain CSR (offsets [n_feat + 1], positions) of the lists that were kept.
int64_t orc_compact_decode(const int32_t* cstart, const uint16_t* delta, int n_feat, int nblk, int block_log2,
                           int32_t* offsets, int32_t* positions) {
    int64_t o = 0;
    for (int f = 0; f < n_feat; ++f) {
        offsets[f] = (int32_t)o;
        for (int b = 0; b < nblk; ++b)
            for (int32_t i = cstart[(size_t)b * n_feat + f]; i < cstart[(size_t)b * n_feat + f + 1]; ++i)
                positions[o++] = (b << block_log2) + (int32_t)delta[i];
    }
    offsets[n_feat] = (int32_t)o;
    return o;
}

// ---- SAE training step (Sec. 3.3: encoder, Top-K and decoder equations; App. B.3: Adam, learning rate 1e-3,
// batches of 4096 tokens, k = 128) ----
// The paper trains the Top-K SAE by reconstruction and states no other term, so the objective taken is the mean
// squared reconstruction error over the batch, L = sum_t |xhat_t - x_t|^2 / (B d), with
//     u_t = x_t - b_dec,  z_t = W_enc u_t + b_enc,  (ids, ReLU(z)) = TopK(z_t, k) as in orc_encode_topk,
//     xhat_t = sum_i zhat_{t,i} W_dec[id_{t,i}] + b_dec.
// Gradients are those of L with the selection held fixed (the Top-K passes gradient to the selected entries only,
// ReLU to the positive ones):
//     g_t = 2 (xhat_t - x_t) / (B d),  dzhat_{t,i} = g_t . W_dec[id],  dz_{t,i} = dzhat_{t,i} [zhat_{t,i} > 0],
//     dW_dec[f] = sum zhat g_t,  dW_enc[f] = sum dz u_t,  db_enc[f] = sum dz  (sums over the (t, i) with id = f),
//     db_dec = sum_t (g_t - sum_i dz_{t,i} W_enc[id_{t,i}]).
// round_bf16 = 1: the encoder sees its operands in the storage format of the inference path, u = bf16(fl32(x - b_dec))
// and bf16(W_enc) (round to nearest even), and the backward pass uses those same rounded operands (the rounding
// itself is treated as the identity); 0: nothing is rounded (the form that finite differences can check).
// ids_in: null, or a selection [B, k] to use instead of the oracle's own (ids of a row distinct, in [0, n_feat)).
// Parameters are fp64 arrays: w_enc, w_dec [n_feat, d]; b_enc [n_feat]; b_dec [d].  Gradient outputs have the same
// shapes; ids_out [B, k] (may be null).  Returns 0, or -1 on invalid arguments.
static float bf16_rne(float v) {
    uint32_t u;
    std::memcpy(&u, &v, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);      // finite inputs only
    u &= 0xFFFF0000u;
    float r;
    std::memcpy(&r, &u, 4);
    return r;
}

float orc_bf16_round(float v) { return bf16_rne(v); }

int orc_sae_loss_grad(const float* x, int B, int d, int n_feat, int k, const double* w_enc, const double* b_enc,
                      const double* w_dec, const double* b_dec, int round_bf16, const int32_t* ids_in,
                      int32_t* ids_out, double* loss, double* g_w_enc, double* g_b_enc, double* g_w_dec,
                      double* g_b_dec) {
    if (B <= 0 || d <= 0 || n_feat <= 0 || k <= 0 || k > n_feat) return -1;
    std::vector<double> we((size_t)n_feat * d);
    for (size_t i = 0; i < we.size(); ++i) we[i] = round_bf16 ? (double)bf16_rne((float)w_enc[i]) : w_enc[i];
    std::fill(g_w_enc, g_w_enc + (size_t)n_feat * d, 0.0);
    std::fill(g_w_dec, g_w_dec + (size_t)n_feat * d, 0.0);
    std::fill(g_b_enc, g_b_enc + n_feat, 0.0);
    std::fill(g_b_dec, g_b_dec + d, 0.0);
    double total = 0.0;
    const double scale = 1.0 / ((double)B * d);
    std::vector<double> u(d), z(n_feat), xh(d), g(d), du(d);
    std::vector<int32_t> order(n_feat), sel(k);
    for (int t = 0; t < B; ++t) {
        for (int c = 0; c < d; ++c) {
            if (round_bf16) u[c] = (double)bf16_rne(x[(size_t)t * d + c] - (float)b_dec[c]);
            else u[c] = (double)x[(size_t)t * d + c] - b_dec[c];
        }
        if (ids_in) {
            for (int i = 0; i < k; ++i) {
                sel[i] = ids_in[(size_t)t * k + i];
                if (sel[i] < 0 || sel[i] >= n_feat) return -1;
            }
        } else {
            for (int f = 0; f < n_feat; ++f) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += u[c] * we[(size_t)f * d + c];
                z[f] = acc + b_enc[f];
                order[f] = f;
            }
            std::sort(order.begin(), order.end(), [&](int32_t a, int32_t c) {
                if (z[a] != z[c]) return z[a] > z[c];
                return a < c;
            });
            for (int i = 0; i < k; ++i) sel[i] = order[i];
        }
        std::vector<double> zh(k);
        for (int i = 0; i < k; ++i) {
            const int32_t f = sel[i];
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += u[c] * we[(size_t)f * d + c];
            zh[i] = std::max(acc + b_enc[f], 0.0);
            if (ids_out) ids_out[(size_t)t * k + i] = f;
        }
        for (int c = 0; c < d; ++c) xh[c] = b_dec[c];
        for (int i = 0; i < k; ++i)
            for (int c = 0; c < d; ++c) xh[c] += zh[i] * w_dec[(size_t)sel[i] * d + c];
        for (int c = 0; c < d; ++c) {
            const double r = xh[c] - (double)x[(size_t)t * d + c];
            total += r * r;
            g[c] = 2.0 * r * scale;
            du[c] = 0.0;
        }
        for (int i = 0; i < k; ++i) {
            const int32_t f = sel[i];
            double dzh = 0.0;
            for (int c = 0; c < d; ++c) dzh += g[c] * w_dec[(size_t)f * d + c];
            const double dz = zh[i] > 0.0 ? dzh : 0.0;
            for (int c = 0; c < d; ++c) {
                g_w_dec[(size_t)f * d + c] += zh[i] * g[c];
                g_w_enc[(size_t)f * d + c] += dz * u[c];
                du[c] += dz * we[(size_t)f * d + c];
            }
            g_b_enc[f] += dz;
        }
        for (int c = 0; c < d; ++c) g_b_dec[c] += g[c] - du[c];
    }
    *loss = total * scale;
    return 0;
}

// Adam (App. B.3 names the optimiser and the learning rate; beta1, beta2, eps are the caller's): for step t >= 1
//     m <- b1 m + (1 - b1) g,  v <- b2 v + (1 - b2) g^2,  p <- p - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).
int orc_adam(double* p, double* m, double* v, const double* grad, int64_t n, double lr, double b1, double b2,
             double eps, int step) {
    if (step < 1) return -1;
    const double c1 = 1.0 - std::pow(b1, (double)step), c2 = 1.0 - std::pow(b2, (double)step);
    for (int64_t i = 0; i < n; ++i) {
        m[i] = b1 * m[i] + (1.0 - b1) * grad[i];
        v[i] = b2 * v[i] + (1.0 - b2) * grad[i] * grad[i];
        p[i] -= lr * (m[i] / c1) / (std::sqrt(v[i] / c2) + eps);
    }
    return 0;
}

// Number of host threads orc_encode_topk uses (rows are independent; nothing else is threaded).
int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

}  // extern "C"
