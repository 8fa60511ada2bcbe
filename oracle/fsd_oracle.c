/*
 * fsd_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, float64 CPU statement of the candidate-verification step of
 * Fuzzy Speculative Decoding, written directly from the paper's definitions.
 * Only the tests, the smoke check and the bench's cpu_baseline leg may call it;
 * the HIP library shares no code, header, table or helper with this file.
 *
 * What follows the paper:
 *   - softmax of a logits row ("next token distributions", Sec. 4 below eq. 4)
 *   - KL(target || draft), JS, TV                       (App. C.1, C.2, C.3)
 *   - FSD acceptance: accept position i iff Div <= T    (Sec. 4, eq. 4; Fig. 1
 *     caption and App. D word the rejection as "exceeds T", which is the
 *     reading taken here -- it differs from the strict "<" only at Div == T)
 *   - stop at the first rejection, emit one token drawn from the unmodified
 *     target distribution at that position (Sec. 4, paragraph after eq. 4);
 *     when every candidate is accepted the token comes from the target row
 *     after the last candidate (the usual bonus token of Sec. 3's SD loop)
 *   - strict SD: accept iff min(1, p/q) > y, y ~ U(0,1) (Sec. 3, eq. 1-2);
 *     on rejection resample from the positive part of p - q, normalised
 *     (Sec. 3, eq. 3, read as the rule of the works cited there)
 *   - strict SD over a token tree (the family Sec. 2 cites): children tried in
 *     index order with the residual update of eq. 3 after every rejection
 *   - token trees (Sec. 6.4): a node carries the acceptance bit of
 *     (target row of its parent context, its own draft row); the deepest node
 *     whose ancestors are all accepted wins, lowest index on ties.
 *
 * What the paper leaves open and this file fixes (the HIP side implements the
 * same published/specified procedures independently):
 *   - random numbers: Philox4x32-10 (Salmon et al., SC'11), key = seed,
 *     counter = ((idx>>2) | stream<<30, b, offset_lo, offset_hi), word idx&3;
 *     stream 0 = Gumbel noise over the vocabulary, stream 1 = SD uniforms
 *   - u = (2*(word>>9) + 1) * 2^-24, exact in binary32, inside (0,1)
 *   - Gumbel noise G = -flog(-flog(u)) where flog is a binary32 routine made
 *     only of IEEE-exact operations (see flog32 below), so that token ids can
 *     be compared bit for bit; the score z + G is one rounded binary32 add and
 *     the token is the argmax, lowest index on ties.
 *
 * parity pins: tests/test_oracle_pins.py (closed forms, bounds, brute force at
 * V=8, Philox known-answer vectors, chi-square of the sampler, SD frequencies).
 * Unpinned: nothing the paper prints is numeric for this step, so agreement
 * with the authors' own implementation ("T-scale parity") is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

#define ORACLE_DIV_KL 0
#define ORACLE_DIV_JS 1
#define ORACLE_DIV_TV 2

#define ORACLE_SAMPLE 0
#define ORACLE_GREEDY 1

#define ST_NONFINITE 1 /* NaN, +inf, or a row that is -inf everywhere, in a row the method reads */
#define ST_BAD_PARENT 2 /* tree: parent index outside [-1, j) */
#define ST_TOO_DEEP 4   /* tree: a node deeper than max_depth */
#define ST_BAD_TOKEN 8  /* strict SD: candidate token id outside [0, V) */

/* thread count of the loops over sequences (timing only: the arithmetic does not depend on it) */
void fsd_oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int fsd_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ loads */

static float bf16_bits_to_float(uint16_t h) {
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, 4);
    return f;
}

/* element i of a row-major logits buffer, as the binary32 value it encodes */
static float load_f(const void* base, size_t i, int dt) {
    if (dt == ORACLE_BF16) return bf16_bits_to_float(((const uint16_t*)base)[i]);
    return ((const float*)base)[i];
}

/* ------------------------------------------------------------ Philox4x32 */

void fsd_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* the 32-bit word the method draws for (stream, sequence b, index idx) */
uint32_t fsd_oracle_random_word(uint64_t seed, uint64_t offset, uint32_t stream, uint32_t b, uint32_t idx) {
    uint32_t ctr[4] = {(idx >> 2) | (stream << 30), b, (uint32_t)offset, (uint32_t)(offset >> 32)};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    fsd_oracle_philox4x32_10(ctr, key, out);
    return out[idx & 3];
}

/* ---------------------------------------------- binary32 Gumbel transform */

/* uniform in (0,1): an odd 24-bit integer times 2^-24, exact in binary32 */
float fsd_oracle_word_to_uniform(uint32_t w) {
    return (float)(((w >> 9) << 1) | 1u) * 0x1p-24f;
}

/* natural log of a positive normal binary32 number from exact operations only:
 * x = 2^e * m with m in [sqrt(1/2), sqrt(2)); ln m = 2 atanh(s), s = (m-1)/(m+1),
 * atanh series to s^11 in Horner form with fused multiply-adds. */
float fsd_oracle_flog32(float x) {
    uint32_t bits;
    memcpy(&bits, &x, 4);
    int e = (int)(bits >> 23) - 127;
    uint32_t mb = (bits & 0x007FFFFFu) | 0x3F800000u;
    float m;
    memcpy(&m, &mb, 4);
    if (m >= 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }
    float num = m - 1.0f;
    float den = m + 1.0f;
    float s = num / den;
    float s2 = s * s;
    float poly = 0x1.745d18p-4f;              /* 1/11 */
    poly = fmaf(poly, s2, 0x1.c71c72p-4f);    /* 1/9  */
    poly = fmaf(poly, s2, 0x1.24924ap-3f);    /* 1/7  */
    poly = fmaf(poly, s2, 0x1.99999ap-3f);    /* 1/5  */
    poly = fmaf(poly, s2, 0x1.555556p-2f);    /* 1/3  */
    poly = fmaf(poly, s2, 1.0f);
    float lnm = (2.0f * s) * poly;
    return fmaf((float)e, 0x1.62e43p-1f, lnm);
}

float fsd_oracle_gumbel(uint32_t w) {
    float u = fsd_oracle_word_to_uniform(w);
    float t = -fsd_oracle_flog32(u);
    return -fsd_oracle_flog32(t);
}

/* ----------------------------------------------------------- row softmax */

/* log-sum-exp of one row in float64; *bad set when the row holds NaN or +inf
 * or is -inf everywhere (no distribution exists). */
static double row_lse(const void* base, size_t off, long V, int dt, int* bad) {
    double m = -INFINITY;
    int b = 0;
    for (long v = 0; v < V; ++v) {
        double z = (double)load_f(base, off + (size_t)v, dt);
        if (isnan(z) || z == INFINITY) b = 1;
        if (z > m) m = z;
    }
    if (m == -INFINITY) b = 1;
    if (b) { *bad = 1; return NAN; }
    double S = 0.0;
    for (long v = 0; v < V; ++v) S += exp((double)load_f(base, off + (size_t)v, dt) - m);
    return m + log(S);
}

/* KL(p||q), JS(p,q), TV(p,q) for p = softmax(target row), q = softmax(draft row)
 * (App. C.1-C.3), natural logarithm, 0 log 0 = 0.  out = {KL, JS, TV};
 * lse = {lse_target, lse_draft}. Returns non-zero when either row is unusable. */
int fsd_oracle_pair(const void* target, size_t toff, const void* draft, size_t doff, long V, int dt,
                    double out[3], double lse[2]) {
    int bad = 0;
    double lt = row_lse(target, toff, V, dt, &bad);
    double ld = row_lse(draft, doff, V, dt, &bad);
    if (lse) { lse[0] = lt; lse[1] = ld; }
    if (bad) { out[0] = out[1] = out[2] = NAN; return ST_NONFINITE; }
    double kl = 0.0, js = 0.0, tv = 0.0;
    for (long v = 0; v < V; ++v) {
        double lp = (double)load_f(target, toff + (size_t)v, dt) - lt;
        double lq = (double)load_f(draft, doff + (size_t)v, dt) - ld;
        double p = exp(lp), q = exp(lq);
        double m = 0.5 * (p + q);
        if (p > 0.0) {
            kl += p * (lp - lq);
            js += 0.5 * p * log(p / m);
        }
        if (q > 0.0) js += 0.5 * q * log(q / m);
        tv += fabs(p - q);
    }
    out[0] = kl; out[1] = js; out[2] = 0.5 * tv;
    return 0;
}

/* -------------------------------------------------------------- sampling */

/* Token from softmax(row) by Gumbel-max (mode SAMPLE) or argmax (GREEDY).
 * gap (optional) = best score minus runner-up, a diagnostic for near ties. */
static int32_t sample_row(const void* base, size_t off, long V, int dt, int mode, uint64_t seed,
                          uint64_t offset, uint32_t b, float* gap) {
    float best = -INFINITY, second = -INFINITY;
    int32_t arg = -1;
    for (long v = 0; v < V; ++v) {
        float z = load_f(base, off + (size_t)v, dt);
        float score = z;
        if (mode == ORACLE_SAMPLE) {
            float g = fsd_oracle_gumbel(fsd_oracle_random_word(seed, offset, 0u, b, (uint32_t)v));
            score = z + g;
        }
        if (score > best || arg < 0) {
            if (arg >= 0) second = best;
            best = score; arg = (int32_t)v;
        } else if (score > second) {
            second = score;
        }
    }
    if (gap) *gap = best - second;
    return arg;
}

/* the row holds a usable distribution */
static int row_is_bad(const void* base, size_t off, long V, int dt) {
    int bad = 0;
    (void)row_lse(base, off, V, dt, &bad);
    return bad;
}

/* -------------------------------------------------------------- FSD chain */

/* target [B,K+1,V], draft [B,K,V], cand [B,K].  Outputs: accept_len [B],
 * out_tokens [B,K+1] (-1 padded), divs [B,K] (float64, chosen divergence),
 * row_status [B], gap [B] (may be NULL).  seq_offset: the arrays hold sequences
 * seq_offset .. seq_offset+B-1 of a larger batch (it only enters the random
 * stream, whose counter carries the sequence index). */
int fsd_oracle_verify_chain(const void* target, const void* draft, const int32_t* cand, int B, int K,
                            long V, int dt, int div_kind, double T, int mode, uint64_t seed,
                            uint64_t offset, int seq_offset, int32_t* accept_len, int32_t* out_tokens,
                            double* divs, int32_t* row_status, float* gap) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int status = 0;
        int n = K;
        for (int i = 0; i < K; ++i) {
            double d3[3];
            size_t toff = ((size_t)b * (size_t)(K + 1) + (size_t)i) * (size_t)V;
            size_t doff = ((size_t)b * (size_t)K + (size_t)i) * (size_t)V;
            status |= fsd_oracle_pair(target, toff, draft, doff, V, dt, d3, NULL);
            double d = d3[div_kind];
            divs[(size_t)b * K + i] = d;
            int ok = (d <= T); /* NaN compares false */
            if (!ok && i < n) n = i;
        }
        size_t soff = ((size_t)b * (size_t)(K + 1) + (size_t)n) * (size_t)V;
        if (!status && row_is_bad(target, soff, V, dt)) status |= ST_NONFINITE;
        for (int i = 0; i <= K; ++i) out_tokens[(size_t)b * (K + 1) + i] = -1;
        if (gap) gap[b] = INFINITY;
        if (status) {
            accept_len[b] = 0;
        } else {
            accept_len[b] = n;
            for (int i = 0; i < n; ++i) out_tokens[(size_t)b * (K + 1) + i] = cand[(size_t)b * K + i];
            out_tokens[(size_t)b * (K + 1) + n] =
                sample_row(target, soff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), gap ? &gap[b] : NULL);
        }
        row_status[b] = status;
    }
    return 0;
}

/* --------------------------------------------------------------- FSD tree */

/* target [B,N+1,V] (row 0 = root context, row j+1 = context after node j),
 * draft [B,N,V], node_tokens [B,N], parent [B,N] (-1 = child of the root,
 * parent[j] < j).  Outputs: path_len [B], path_nodes [B,max_depth] (-1 padded),
 * out_tokens [B,max_depth+1] (-1 padded), divs [B,N], row_status [B]. */
static int32_t sample_row_warped(const void* base, size_t off, long V, int dt, int mode, uint64_t seed,
                                 uint64_t offset, uint32_t b, float inv_temp, int top_k, double top_p,
                                 float* gap, float* threshold, double* slack);

/* warped != 0: the token is drawn with the sampling-method warpers (see sample_row_warped) */
static int verify_tree_impl(const void* target, const void* draft, const int32_t* node_tokens,
                            const int32_t* parent, int B, int N, int max_depth, long V, int dt,
                            int div_kind, double T, int mode, uint64_t seed, uint64_t offset,
                            int seq_offset, int32_t* path_len, int32_t* path_nodes, int32_t* out_tokens, double* divs,
                            int32_t* row_status, float* gap, int warped, float inv_temp, int top_k, double top_p,
                            float* threshold, double* slack) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int status = 0;
        const int32_t* par = parent + (size_t)b * N;
        int* depth = (int*)malloc(sizeof(int) * (size_t)(N > 0 ? N : 1));
        char* live = (char*)malloc((size_t)(N > 0 ? N : 1));
        for (int j = 0; j < N; ++j)
            if (par[j] < -1 || par[j] >= j) status |= ST_BAD_PARENT;
        int win = -1, win_depth = 0;
        if (!(status & ST_BAD_PARENT)) {
            for (int j = 0; j < N; ++j) {
                depth[j] = par[j] < 0 ? 1 : depth[par[j]] + 1;
                if (depth[j] > max_depth) status |= ST_TOO_DEEP;
            }
        }
        for (int j = 0; j < N; ++j) {
            double d3[3];
            double d = NAN;
            if (!(status & ST_BAD_PARENT)) {
                size_t toff = ((size_t)b * (size_t)(N + 1) + (size_t)(par[j] + 1)) * (size_t)V;
                size_t doff = ((size_t)b * (size_t)N + (size_t)j) * (size_t)V;
                status |= fsd_oracle_pair(target, toff, draft, doff, V, dt, d3, NULL);
                d = d3[div_kind];
            }
            divs[(size_t)b * N + j] = d;
            if (!(status & ST_BAD_PARENT)) {
                int ok = (d <= T);
                live[j] = (char)(ok && (par[j] < 0 || live[par[j]]));
                if (live[j] && depth[j] > win_depth) { win = j; win_depth = depth[j]; }
            }
        }
        size_t soff = ((size_t)b * (size_t)(N + 1) + (size_t)(win + 1)) * (size_t)V;
        if (!status && row_is_bad(target, soff, V, dt)) status |= ST_NONFINITE;
        for (int i = 0; i < max_depth; ++i) path_nodes[(size_t)b * max_depth + i] = -1;
        for (int i = 0; i <= max_depth; ++i) out_tokens[(size_t)b * (max_depth + 1) + i] = -1;
        if (gap) gap[b] = INFINITY;
        if (status) {
            path_len[b] = 0;
        } else {
            path_len[b] = win_depth;
            int j = win;
            for (int i = win_depth - 1; i >= 0; --i) {
                path_nodes[(size_t)b * max_depth + i] = j;
                out_tokens[(size_t)b * (max_depth + 1) + i] = node_tokens[(size_t)b * N + j];
                j = par[j];
            }
            if (warped) {
                float g32 = INFINITY;
                out_tokens[(size_t)b * (max_depth + 1) + win_depth] =
                    sample_row_warped(target, soff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), inv_temp,
                                      top_k, top_p, &g32, &threshold[b], &slack[b]);
                if (gap) gap[b] = g32;
            } else {
                out_tokens[(size_t)b * (max_depth + 1) + win_depth] =
                    sample_row(target, soff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), gap ? &gap[b] : NULL);
            }
        }
        row_status[b] = status;
        free(depth);
        free(live);
    }
    return 0;
}

int fsd_oracle_verify_tree(const void* target, const void* draft, const int32_t* node_tokens,
                           const int32_t* parent, int B, int N, int max_depth, long V, int dt,
                           int div_kind, double T, int mode, uint64_t seed, uint64_t offset,
                           int seq_offset, int32_t* path_len, int32_t* path_nodes, int32_t* out_tokens, double* divs,
                           int32_t* row_status, float* gap) {
    return verify_tree_impl(target, draft, node_tokens, parent, B, N, max_depth, V, dt, div_kind, T, mode, seed, offset,
                            seq_offset, path_len, path_nodes, out_tokens, divs, row_status, gap, 0, 1.0f, 0, 1.0, NULL,
                            NULL);
}

/* fsd_oracle_verify_tree with the warpers applied where the token is drawn (Sec. 4: the sampling
 * method is the user's); extra outputs threshold [B], slack [B] as in the chain version. */
int fsd_oracle_verify_tree_warped(const void* target, const void* draft, const int32_t* node_tokens,
                                  const int32_t* parent, int B, int N, int max_depth, long V, int dt,
                                  int div_kind, double T, int mode, uint64_t seed, uint64_t offset,
                                  int seq_offset, float inv_temp, int top_k, double top_p, int32_t* path_len,
                                  int32_t* path_nodes, int32_t* out_tokens, double* divs, int32_t* row_status,
                                  float* gap, float* threshold, double* slack) {
    for (int b = 0; b < B; ++b) { threshold[b] = NAN; slack[b] = INFINITY; }
    return verify_tree_impl(target, draft, node_tokens, parent, B, N, max_depth, V, dt, div_kind, T, mode, seed, offset,
                            seq_offset, path_len, path_nodes, out_tokens, divs, row_status, gap, 1, inv_temp, top_k,
                            top_p, threshold, slack);
}

/* -------------------------------------------------------------- strict SD */

/* Token from the normalised positive part of p - q by Gumbel-max over
 * ln(p_v - q_v) + G_v; falls back to p when p == q everywhere. */
static int32_t sample_residual(const void* target, size_t toff, const void* draft, size_t doff, long V,
                               int dt, int mode, uint64_t seed, uint64_t offset, uint32_t b,
                               double lse_t, double lse_d, double* gap) {
    double best = -INFINITY, second = -INFINITY;
    int32_t arg = -1;
    for (long v = 0; v < V; ++v) {
        double p = exp((double)load_f(target, toff + (size_t)v, dt) - lse_t);
        double q = exp((double)load_f(draft, doff + (size_t)v, dt) - lse_d);
        double r = p - q;
        if (!(r > 0.0)) continue;
        double score = log(r);
        if (mode == ORACLE_SAMPLE)
            score += (double)fsd_oracle_gumbel(fsd_oracle_random_word(seed, offset, 0u, b, (uint32_t)v));
        if (score > best || arg < 0) {
            if (arg >= 0) second = best;
            best = score; arg = (int32_t)v;
        } else if (score > second) {
            second = score;
        }
    }
    if (gap) *gap = best - second;
    return arg;
}

/* Same tensors as the chain call.  log_ratio [B,K] = ln p(x_i) - ln q(x_i);
 * margin [B,K] = min(0, log_ratio) - ln u_i (accepted iff > 0), for near-tie
 * reporting; gap [B] = sampler runner-up gap (float64). */
int sd_oracle_verify_chain(const void* target, const void* draft, const int32_t* cand, int B, int K,
                           long V, int dt, int mode, uint64_t seed, uint64_t offset, int seq_offset,
                           int32_t* accept_len, int32_t* out_tokens, double* log_ratio, double* margin,
                           int32_t* row_status, double* gap) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int status = 0;
        int n = K;
        double lse_n[2] = {NAN, NAN};
        for (int i = 0; i < K; ++i) {
            size_t toff = ((size_t)b * (size_t)(K + 1) + (size_t)i) * (size_t)V;
            size_t doff = ((size_t)b * (size_t)K + (size_t)i) * (size_t)V;
            int bad = 0;
            double lt = row_lse(target, toff, V, dt, &bad);
            double ld = row_lse(draft, doff, V, dt, &bad);
            int32_t x = cand[(size_t)b * K + i];
            double ratio = NAN, mar = NAN;
            int ok = 0;
            if (bad) status |= ST_NONFINITE;
            if (x < 0 || x >= V) status |= ST_BAD_TOKEN;
            if (!bad && x >= 0 && x < V) {
                double lp = (double)load_f(target, toff + (size_t)x, dt) - lt;
                double lq = (double)load_f(draft, doff + (size_t)x, dt) - ld;
                ratio = (lp == -INFINITY) ? -INFINITY : lp - lq;
                double u = (double)fsd_oracle_word_to_uniform(
                    fsd_oracle_random_word(seed, offset, 1u, (uint32_t)(b + seq_offset), (uint32_t)i));
                double thr = ratio < 0.0 ? ratio : 0.0; /* ln min(1, p/q) */
                mar = thr - log(u);
                ok = (mar > 0.0); /* min(1,p/q) > u */
            }
            log_ratio[(size_t)b * K + i] = ratio;
            margin[(size_t)b * K + i] = mar;
            if (!ok && i < n) { n = i; lse_n[0] = lt; lse_n[1] = ld; }
        }
        size_t soff = ((size_t)b * (size_t)(K + 1) + (size_t)n) * (size_t)V;
        if (!status && row_is_bad(target, soff, V, dt)) status |= ST_NONFINITE;
        for (int i = 0; i <= K; ++i) out_tokens[(size_t)b * (K + 1) + i] = -1;
        if (gap) gap[b] = INFINITY;
        if (status) {
            accept_len[b] = 0;
        } else {
            accept_len[b] = n;
            for (int i = 0; i < n; ++i) out_tokens[(size_t)b * (K + 1) + i] = cand[(size_t)b * K + i];
            int32_t y = -1;
            if (n < K) {
                size_t doff = ((size_t)b * (size_t)K + (size_t)n) * (size_t)V;
                y = sample_residual(target, soff, draft, doff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset),
                                    lse_n[0], lse_n[1], gap ? &gap[b] : NULL);
            }
            if (y < 0) {
                float g32;
                y = sample_row(target, soff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), &g32);
                if (gap) gap[b] = (double)g32;
            }
            out_tokens[(size_t)b * (K + 1) + n] = y;
        }
        row_status[b] = status;
    }
    return 0;
}

/* ------------------------------------- strict SD over a token tree */

/* Strict (distribution-preserving) verification of a token tree: the tree
 * analogue of sd_oracle_verify_chain.  The paper only names this family of
 * methods (Sec. 2, "verifying more tokens with tree-structured proposals");
 * the procedure here is the published multi-round rejection rule of that
 * family, stated for this library's tree layout:
 *
 *   at the current context with target distribution p, the children are tried
 *   in index order; child j (token x_j, proposed from its own draft
 *   distribution q_j) is accepted iff min(1, p(x_j)/q_j(x_j)) > y_j (Sec. 3,
 *   eq. 1-2, y_j = the SD uniform of index j); on acceptance the walk moves to
 *   the context after node j; on rejection p is replaced by the normalised
 *   positive part of p - q_j (Sec. 3, eq. 3) before the next child is tried.
 *   When no child is accepted the token is drawn from the current p: the
 *   target row itself at a node without children, else the residual of the
 *   last rejection.
 *
 * With one child per node this is sd_oracle_verify_chain, bit for bit.
 * log_ratio [B,N] = ln p(x_j) - ln q_j(x_j) with the p in force when node j was
 * tried, margin [B,N] as in the chain (NaN for nodes never tried). */
int sd_oracle_verify_tree(const void* target, const void* draft, const int32_t* node_tokens,
                          const int32_t* parent, int B, int N, int max_depth, long V, int dt, int mode,
                          uint64_t seed, uint64_t offset, int seq_offset, int32_t* path_len,
                          int32_t* path_nodes, int32_t* out_tokens, double* log_ratio, double* margin,
                          int32_t* row_status, double* gap) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int status = 0;
        const int32_t* par = parent + (size_t)b * N;
        const int32_t* tok = node_tokens + (size_t)b * N;
        int* depth = (int*)malloc(sizeof(int) * (size_t)(N > 0 ? N : 1));
        double* lse_d = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double* p = (double*)malloc(sizeof(double) * (size_t)V);   /* the distribution in force */
        double* r = (double*)malloc(sizeof(double) * (size_t)V);   /* positive part of p - q, not normalised */
        for (int j = 0; j < N; ++j) {
            log_ratio[(size_t)b * N + j] = NAN;
            margin[(size_t)b * N + j] = NAN;
            if (par[j] < -1 || par[j] >= j) status |= ST_BAD_PARENT;
            if (tok[j] < 0 || tok[j] >= V) status |= ST_BAD_TOKEN;
        }
        if (!(status & ST_BAD_PARENT)) {
            for (int j = 0; j < N; ++j) {
                depth[j] = par[j] < 0 ? 1 : depth[par[j]] + 1;
                if (depth[j] > max_depth) status |= ST_TOO_DEEP;
                int bad = 0;
                (void)row_lse(target, ((size_t)b * (size_t)(N + 1) + (size_t)(par[j] + 1)) * (size_t)V, V, dt, &bad);
                lse_d[j] = row_lse(draft, ((size_t)b * (size_t)N + (size_t)j) * (size_t)V, V, dt, &bad);
                if (bad) status |= ST_NONFINITE;
            }
        }
        for (int i = 0; i < max_depth; ++i) path_nodes[(size_t)b * max_depth + i] = -1;
        for (int i = 0; i <= max_depth; ++i) out_tokens[(size_t)b * (max_depth + 1) + i] = -1;
        if (gap) gap[b] = INFINITY;
        path_len[b] = 0;
        if (!status) {
            int cur = -1, n = 0;
            int32_t y = -1;
            for (;;) {
                const size_t toff = ((size_t)b * (size_t)(N + 1) + (size_t)(cur + 1)) * (size_t)V;
                int bad = 0;
                const double lt = row_lse(target, toff, V, dt, &bad);
                if (bad) { status |= ST_NONFINITE; break; }
                int nrej = 0, next = -1;
                for (int j = cur + 1; j < N && next < 0; ++j) {
                    if (par[j] != cur) continue;
                    const size_t doff = ((size_t)b * (size_t)N + (size_t)j) * (size_t)V;
                    const int32_t x = tok[j];
                    const double lq = (double)load_f(draft, doff + (size_t)x, dt) - lse_d[j];
                    double lp;
                    if (nrej == 0) lp = (double)load_f(target, toff + (size_t)x, dt) - lt;
                    else lp = p[x] > 0.0 ? log(p[x]) : -INFINITY;
                    const double ratio = (lp == -INFINITY) ? -INFINITY : lp - lq;
                    const double u = (double)fsd_oracle_word_to_uniform(
                        fsd_oracle_random_word(seed, offset, 1u, (uint32_t)(b + seq_offset), (uint32_t)j));
                    const double thr = ratio < 0.0 ? ratio : 0.0;
                    const double mar = thr - log(u);
                    log_ratio[(size_t)b * N + j] = ratio;
                    margin[(size_t)b * N + j] = mar;
                    if (mar > 0.0) { next = j; break; }
                    /* rejected: p <- positive part of p - q_j, normalised (kept as it is if that part is empty) */
                    double Z = 0.0;
                    for (long v = 0; v < V; ++v) {
                        const double pv = (nrej == 0) ? exp((double)load_f(target, toff + (size_t)v, dt) - lt) : p[v];
                        const double qv = exp((double)load_f(draft, doff + (size_t)v, dt) - lse_d[j]);
                        const double d = pv - qv;
                        if (nrej == 0) p[v] = pv;
                        r[v] = d > 0.0 ? d : 0.0;
                        Z += r[v];
                    }
                    if (Z > 0.0) {
                        for (long v = 0; v < V; ++v) p[v] = r[v] / Z;
                        ++nrej;
                    }
                }
                if (next >= 0) {
                    path_nodes[(size_t)b * max_depth + n] = next;
                    out_tokens[(size_t)b * (max_depth + 1) + n] = tok[next];
                    ++n;
                    cur = next;
                    continue;
                }
                /* nobody accepted: the token comes from the distribution in force */
                if (nrej > 0) {
                    double best = -INFINITY, second = -INFINITY;
                    for (long v = 0; v < V; ++v) {
                        if (!(r[v] > 0.0)) continue;
                        double score = log(r[v]);
                        if (mode == ORACLE_SAMPLE)
                            score += (double)fsd_oracle_gumbel(
                                fsd_oracle_random_word(seed, offset, 0u, (uint32_t)(b + seq_offset), (uint32_t)v));
                        if (score > best || y < 0) {
                            if (y >= 0) second = best;
                            best = score; y = (int32_t)v;
                        } else if (score > second) {
                            second = score;
                        }
                    }
                    if (gap) gap[b] = best - second;
                }
                if (y < 0) {
                    float g32;
                    y = sample_row(target, toff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), &g32);
                    if (gap) gap[b] = (double)g32;
                }
                break;
            }
            if (!status) {
                path_len[b] = n;
                out_tokens[(size_t)b * (max_depth + 1) + n] = y;
            } else {
                for (int i = 0; i < max_depth; ++i) path_nodes[(size_t)b * max_depth + i] = -1;
                for (int i = 0; i <= max_depth; ++i) out_tokens[(size_t)b * (max_depth + 1) + i] = -1;
            }
        }
        row_status[b] = status;
        free(depth); free(lse_d); free(p); free(r);
    }
    return 0;
}

/* ------------------------------------------------- reducible FSD (rFSD) */

/* Sec. 4.3 ("Reducing FSD to standard SD"): position i is accepted iff the
 * divergence of its two distributions is within T (the FSD rule, with the same
 * "<=" reading as fsd_oracle_verify_chain) OR the strict SD test of Sec. 3
 * eq. 1-2 accepts the candidate token (same uniforms as sd_oracle_verify_chain).
 * At the first rejection the token is resampled from the normalised positive
 * part of p - q (Sec. 3 eq. 3), otherwise from the row after the last candidate.
 * Outputs as sd_oracle_verify_chain plus divs [B,K]. */
int rfsd_oracle_verify_chain(const void* target, const void* draft, const int32_t* cand, int B, int K,
                             long V, int dt, int div_kind, double T, int mode, uint64_t seed,
                             uint64_t offset, int seq_offset, int32_t* accept_len, int32_t* out_tokens,
                             double* divs, double* log_ratio, double* margin, int32_t* row_status,
                             double* gap) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int status = 0;
        int n = K;
        double lse_n[2] = {NAN, NAN};
        for (int i = 0; i < K; ++i) {
            size_t toff = ((size_t)b * (size_t)(K + 1) + (size_t)i) * (size_t)V;
            size_t doff = ((size_t)b * (size_t)K + (size_t)i) * (size_t)V;
            double d3[3], lse2[2];
            int pst = fsd_oracle_pair(target, toff, draft, doff, V, dt, d3, lse2);
            status |= pst;
            double d = d3[div_kind];
            divs[(size_t)b * K + i] = d;
            int32_t x = cand[(size_t)b * K + i];
            double ratio = NAN, mar = NAN;
            int sd_ok = 0;
            if (x < 0 || x >= V) status |= ST_BAD_TOKEN;
            if (!pst && x >= 0 && x < V) {
                double lp = (double)load_f(target, toff + (size_t)x, dt) - lse2[0];
                double lq = (double)load_f(draft, doff + (size_t)x, dt) - lse2[1];
                ratio = (lp == -INFINITY) ? -INFINITY : lp - lq;
                double u = (double)fsd_oracle_word_to_uniform(
                    fsd_oracle_random_word(seed, offset, 1u, (uint32_t)(b + seq_offset), (uint32_t)i));
                double thr = ratio < 0.0 ? ratio : 0.0;
                mar = thr - log(u);
                sd_ok = (mar > 0.0);
            }
            log_ratio[(size_t)b * K + i] = ratio;
            margin[(size_t)b * K + i] = mar;
            int ok = (d <= T) || sd_ok;
            if (!ok && i < n) { n = i; lse_n[0] = lse2[0]; lse_n[1] = lse2[1]; }
        }
        size_t soff = ((size_t)b * (size_t)(K + 1) + (size_t)n) * (size_t)V;
        if (!status && row_is_bad(target, soff, V, dt)) status |= ST_NONFINITE;
        for (int i = 0; i <= K; ++i) out_tokens[(size_t)b * (K + 1) + i] = -1;
        if (gap) gap[b] = INFINITY;
        if (status) {
            accept_len[b] = 0;
        } else {
            accept_len[b] = n;
            for (int i = 0; i < n; ++i) out_tokens[(size_t)b * (K + 1) + i] = cand[(size_t)b * K + i];
            int32_t y = -1;
            if (n < K) {
                size_t doff = ((size_t)b * (size_t)K + (size_t)n) * (size_t)V;
                y = sample_residual(target, soff, draft, doff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset),
                                    lse_n[0], lse_n[1], gap ? &gap[b] : NULL);
            }
            if (y < 0) {
                float g32;
                y = sample_row(target, soff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), &g32);
                if (gap) gap[b] = (double)g32;
            }
            out_tokens[(size_t)b * (K + 1) + n] = y;
        }
        row_status[b] = status;
    }
    return 0;
}

/* ------------------------------------------ sampling-method warpers (chain) */

static int cmp_float_desc(const void* a, const void* b) {
    float x = *(const float*)a, y = *(const float*)b;
    return (x < y) - (x > y);
}

/* The token of softmax-sampling with the usual warpers, applied in this order to the row's logits
 * (Sec. 4: the token is drawn with "whatever sampling method the user sets"):
 *   temperature  s_v = z_v * inv_temp, one binary32 multiply (inv_temp = binary32(1/temperature));
 *   top-k        keep the entries with s_v >= the top_k-th largest s (ties at it are all kept);
 *   top-p        with q = softmax of the kept s, keep s_v >= t, t the largest value with
 *                sum_{s_v >= t} q_v >= top_p (ties kept);
 * then Gumbel-max over the kept entries on s_v + G_v, the random stream of sample_row.
 * threshold (out) = the smallest kept s; slack (out) = how far the nucleus mass at the decision
 * was from top_p on the nearer side (tiny = a binary32 evaluation may keep one value more or less). */
static int32_t sample_row_warped(const void* base, size_t off, long V, int dt, int mode, uint64_t seed,
                                 uint64_t offset, uint32_t b, float inv_temp, int top_k, double top_p,
                                 float* gap, float* threshold, double* slack) {
    float* sv = (float*)malloc(sizeof(float) * (size_t)V);
    float* srt = (float*)malloc(sizeof(float) * (size_t)V);
    for (long v = 0; v < V; ++v) {
        float z = load_f(base, off + (size_t)v, dt);
        sv[v] = z * inv_temp;
        srt[v] = sv[v];
    }
    qsort(srt, (size_t)V, sizeof(float), cmp_float_desc);
    float t = -INFINITY;
    long nk = V;
    if (top_k > 0 && top_k < V) {
        t = srt[top_k - 1];
        nk = top_k;
        while (nk < V && srt[nk] == t) ++nk; /* ties */
    }
    *slack = INFINITY;
    if (top_p < 1.0) {
        double m = (double)srt[0], Z = 0.0;
        for (long i = 0; i < nk; ++i) Z += exp((double)srt[i] - m);
        double cum = 0.0;
        long i = 0;
        float tp = srt[nk - 1];
        while (i < nk) {
            long j = i;
            double blk = 0.0;
            while (j < nk && srt[j] == srt[i]) { blk += exp((double)srt[j] - m); ++j; }
            double before = cum / Z;
            cum += blk;
            double after = cum / Z;
            if (fabs(before - top_p) < *slack && i > 0) *slack = fabs(before - top_p);
            if (fabs(after - top_p) < *slack) *slack = fabs(after - top_p);
            if (after >= top_p) { tp = srt[i]; break; }
            i = j;
        }
        if (tp > t) t = tp;
    }
    *threshold = t;
    float best = -INFINITY, second = -INFINITY;
    int32_t arg = -1;
    for (long v = 0; v < V; ++v) {
        if (!(sv[v] >= t)) continue;
        float score = sv[v];
        if (mode == ORACLE_SAMPLE) {
            float g = fsd_oracle_gumbel(fsd_oracle_random_word(seed, offset, 0u, b, (uint32_t)v));
            score = sv[v] + g;
        }
        if (score > best || arg < 0) {
            if (arg >= 0) second = best;
            best = score; arg = (int32_t)v;
        } else if (score > second) {
            second = score;
        }
    }
    if (gap) *gap = best - second;
    free(sv);
    free(srt);
    return arg;
}

/* fsd_oracle_verify_chain with the warpers above applied where the token is drawn.
 * Extra outputs: threshold [B] (smallest kept scaled logit), slack [B]. */
int fsd_oracle_verify_chain_warped(const void* target, const void* draft, const int32_t* cand, int B, int K,
                                   long V, int dt, int div_kind, double T, int mode, uint64_t seed,
                                   uint64_t offset, int seq_offset, float inv_temp, int top_k, double top_p,
                                   int32_t* accept_len, int32_t* out_tokens, double* divs,
                                   int32_t* row_status, float* gap, float* threshold, double* slack) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int status = 0;
        int n = K;
        for (int i = 0; i < K; ++i) {
            double d3[3];
            size_t toff = ((size_t)b * (size_t)(K + 1) + (size_t)i) * (size_t)V;
            size_t doff = ((size_t)b * (size_t)K + (size_t)i) * (size_t)V;
            status |= fsd_oracle_pair(target, toff, draft, doff, V, dt, d3, NULL);
            double d = d3[div_kind];
            divs[(size_t)b * K + i] = d;
            int ok = (d <= T);
            if (!ok && i < n) n = i;
        }
        size_t soff = ((size_t)b * (size_t)(K + 1) + (size_t)n) * (size_t)V;
        if (!status && row_is_bad(target, soff, V, dt)) status |= ST_NONFINITE;
        for (int i = 0; i <= K; ++i) out_tokens[(size_t)b * (K + 1) + i] = -1;
        gap[b] = INFINITY;
        threshold[b] = NAN;
        slack[b] = INFINITY;
        if (status) {
            accept_len[b] = 0;
        } else {
            accept_len[b] = n;
            for (int i = 0; i < n; ++i) out_tokens[(size_t)b * (K + 1) + i] = cand[(size_t)b * K + i];
            out_tokens[(size_t)b * (K + 1) + n] =
                sample_row_warped(target, soff, V, dt, mode, seed, offset, (uint32_t)(b + seq_offset), inv_temp, top_k,
                                  top_p, &gap[b], &threshold[b], &slack[b]);
        }
        row_status[b] = status;
    }
    return 0;
}
