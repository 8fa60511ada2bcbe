// Acceptance (chain prefix, tree path, strict SD, reducible FSD) and the Gumbel-max draw.
// Part of libfsd (gfx950); included by fsd_kernels.hip, which holds the host side and the C ABI.
#ifndef FSD_CSRC_ACCEPT_SAMPLE_H_
#define FSD_CSRC_ACCEPT_SAMPLE_H_

#include "device_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// kernel 2: acceptance + extra token

struct SampleParams {
    const char* target;
    const char* draft;        // strict SD only
    const int32_t* tokens;    // cand [B,K] or node_tokens [B,N]
    const int32_t* parent;    // tree only
    int rows;                 // K or N
    int max_depth;            // tree only
    long V;
    long nslots;
    int sps;                  // slots per sampler workgroup
    int GS;
    float T;
    int mode;
    unsigned seed_lo, seed_hi, off_lo, off_hi;
    int32_t* out_len;
    int32_t* out_tokens;
    int32_t* path_nodes;      // tree only
    int32_t* row_status;      // optional
    const float* thr;         // optional [B]: warpers, smallest kept scaled logit of the sampled row
    float inv_temp;           // warpers: binary32(1 / temperature), 1 otherwise
    unsigned spin_limit;      // bounded wait for the other workgroups' shares
    int clear_arrive;         // a call without a clearing kernel: the arrival slots are cleared here (see pair_kernel.h)
    Ws ws;
};

struct Best { float score; int idx; };

__device__ __forceinline__ Best better(Best a, Best b) {
    return (b.score > a.score || (b.score == a.score && b.idx < a.idx)) ? b : a;
}
__device__ __forceinline__ Best wave_best(Best v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Best other{__shfl_xor(v.score, o), __shfl_xor(v.idx, o)};
        v = better(v, other);
    }
    return v;
}

template <bool BF16, bool ALIGNED, int KIND>
__global__ __launch_bounds__(kWG) void accept_sample(SampleParams P) {
    constexpr int VE = Slot<BF16>::VE;
    constexpr int ES = BF16 ? 2 : 4;
    extern __shared__ int s_dyn[];   // tree: par[N], anc[N], acc[N], dep[N]
    __shared__ int s_n, s_st, s_key, s_last;
    __shared__ Best s_best[8];
    __shared__ int s_bad[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gs = blockIdx.x, b = blockIdx.y;
    const int rows = P.rows;

    if (tid == 0) { s_n = rows; s_st = 0; s_key = 0; }
    if (P.clear_arrive) {
        // the reduction kernel has ended: its wavefronts' slots go back to zero, so that the same call
        // replayed from a captured graph, with the same number, does not find them set
        uint4* const slots = reinterpret_cast<uint4*>(P.ws.arrive);
        const long nthreads = static_cast<long>(gridDim.x) * gridDim.y * kWG;
        for (long i = (static_cast<long>(b) * gridDim.x + gs) * kWG + tid; i < kMaxArrive / 2; i += nthreads)
            slots[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    __syncthreads();

    // ---- which positions are accepted
    int n = 0;         // accepted prefix length / path depth
    int sample_row = 0;
    int winner = -1;
    int nchain = 0;    // strict SD on a tree: rejected siblings whose draft rows shape the residual
    if constexpr (KIND == KIND_CHAIN || KIND == KIND_SD || KIND == KIND_RFSD) {
        for (int i = tid; i < rows; i += kWG) {
            const int pr = b * rows + i;
            const int st = P.ws.pst[pr];
            bool ok = false;
            if constexpr (KIND == KIND_CHAIN || KIND == KIND_RFSD) {
                ok = (P.ws.div[pr] <= P.T);   // Sec. 4 eq. 4 (NaN compares false)
            }
            if constexpr (KIND == KIND_SD || KIND == KIND_RFSD) {   // reducible FSD (Sec. 4.3): either rule accepts
                // Sec. 3 eq. 1-2 in the log domain: min(1, p/q) > u  <=>  min(0, ln p - ln q) - ln u > 0
                const double ratio = P.ws.lr[pr];
                const U4 r = philox4x32_10((static_cast<unsigned>(i) >> 2) | (1u << 30), static_cast<unsigned>(b),
                                           P.off_lo, P.off_hi, P.seed_lo, P.seed_hi);
                const unsigned wsel = (i & 3) == 0 ? r.x : (i & 3) == 1 ? r.y : (i & 3) == 2 ? r.z : r.w;
                const double u = static_cast<double>(word_to_uniform(wsel));
                const double thr = ratio < 0.0 ? ratio : 0.0;
                ok = ok || (thr - log(u) > 0.0);
            }
            if (st) atomicOr(&s_st, st);
            if (!ok) atomicMin(&s_n, i);
        }
        __syncthreads();
        n = s_n;
        sample_row = n;
    } else if constexpr (KIND == KIND_TREESD) {
        // the walk kernel has decided: depth, last node, and the residual chain the token comes from
        // (if the walk gave up on a bounded wait it may have written nothing: the header is then
        // whatever an earlier call left, so nothing in it is trusted)
        const int* hdr = P.ws.tsd + static_cast<size_t>(b) * (4 + rows);
        const bool gave_up = failure_flagged(P.ws);
        if (tid == 0) s_st = gave_up ? FSD_ROW_INTERNAL : hdr[0];
        n = gave_up ? 0 : hdr[1];
        sample_row = gave_up ? 0 : hdr[2] + 1;
        nchain = gave_up ? 0 : hdr[3];
        if (n < 0 || n > P.max_depth || sample_row < 0 || sample_row > rows || nchain < 0 || nchain > rows) {
            n = 0; sample_row = 0; nchain = 0;
            if (tid == 0) s_st = FSD_ROW_INTERNAL;
        }
        int* ch = s_dyn;
        float* iz = reinterpret_cast<float*>(s_dyn + rows);
        float* ldv = reinterpret_cast<float*>(s_dyn + 2 * rows);
        for (int m = tid; m < nchain; m += kWG) {
            const int c = hdr[4 + m];
            ch[m] = c;
            iz[m] = P.ws.tsd_invz[static_cast<size_t>(b) * rows + m];
            ldv[m] = static_cast<float>(P.ws.lse2[2 * (static_cast<size_t>(b) * rows + c) + 1]);
        }
        __syncthreads();
    } else {
        int* par = s_dyn;
        int* anc = s_dyn + rows;
        int* acc = s_dyn + 2 * rows;
        int* dep = s_dyn + 3 * rows;
        for (int j = tid; j < rows; j += kWG) {
            const int pr = b * rows + j;
            int p = P.parent[pr];
            if (p < -1 || p >= j) { atomicOr(&s_st, FSD_ROW_BAD_PARENT); p = -1; }
            const int st = P.ws.pst[pr];
            if (st) atomicOr(&s_st, st);
            par[j] = p; anc[j] = p; dep[j] = 1;
            acc[j] = (P.ws.div[pr] <= P.T) ? 1 : 0;
        }
        __syncthreads();
        // pointer jumping: after r rounds anc[j] is the 2^r-th ancestor, acc/dep cover that stretch
        for (int span = 1; span < rows; span <<= 1) {
            int na[kMaxRows / kWG], nacc[kMaxRows / kWG], nd[kMaxRows / kWG];
#pragma unroll
            for (int q = 0; q < kMaxRows / kWG; ++q) {
                const int j = tid + q * kWG;
                if (j < rows) {
                    const int a = anc[j];
                    na[q] = a; nacc[q] = acc[j]; nd[q] = dep[j];
                    if (a >= 0) { na[q] = anc[a]; nacc[q] = acc[j] & acc[a]; nd[q] = dep[j] + dep[a]; }
                }
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < kMaxRows / kWG; ++q) {
                const int j = tid + q * kWG;
                if (j < rows) { anc[j] = na[q]; acc[j] = nacc[q]; dep[j] = nd[q]; }
            }
            __syncthreads();
        }
        for (int j = tid; j < rows; j += kWG) {
            if (dep[j] > P.max_depth) atomicOr(&s_st, FSD_ROW_TOO_DEEP);
            if (acc[j]) atomicMax(&s_key, (dep[j] << 11) | (kMaxRows - 1 - j));   // deepest, then lowest index
        }
        __syncthreads();
        const int key = s_key;
        if (key) { n = key >> 11; winner = kMaxRows - 1 - (key & (kMaxRows - 1)); }
        sample_row = winner + 1;
    }
    int status = s_st;
    if (status & FSD_ROW_BAD_PARENT) status &= ~FSD_ROW_TOO_DEEP;   // depths mean nothing in a malformed tree
    if (failure_flagged(P.ws)) status |= FSD_ROW_INTERNAL;   // a bounded wait of the reduction kernel expired

    // ---- Gumbel-max over this workgroup's share of the sampled target row
    const char* trow = P.target + (static_cast<size_t>(b) * (rows + 1) + sample_row) * static_cast<size_t>(P.V) * ES;
    bool residual = false;
    const char* drow = nullptr;
    float lt = 0.0f, ld = 0.0f;
    if constexpr (KIND == KIND_TREESD) {
        if (nchain > 0 && !status) {
            residual = true;
            lt = static_cast<float>(P.ws.lse2[2 * (static_cast<size_t>(b) * rows + s_dyn[nchain - 1])]);
        }
    }
    if constexpr (KIND == KIND_SD || KIND == KIND_RFSD) {
        if (n < rows) {   // rejected at n: the residual of Sec. 3 eq. 3 needs the draft row as well
            residual = true;
            drow = P.draft + (static_cast<size_t>(b) * rows + n) * static_cast<size_t>(P.V) * ES;
            lt = static_cast<float>(P.ws.lse2[2 * (b * rows + n)]);
            ld = static_cast<float>(P.ws.lse2[2 * (b * rows + n) + 1]);
        }
    }
    Best best{neg_inf(), 0x7FFFFFFF}, rbest{neg_inf(), 0x7FFFFFFF};
    int bad = 0;
    if (!status) {
        const long s0 = static_cast<long>(gs) * P.sps;
        const long s1 = (s0 + P.sps < P.nslots) ? s0 + P.sps : P.nslots;
        // thr, rthr: scores the winner is known to reach (see the bounds below)
        float thr = neg_inf(), rthr = neg_inf();
        const float thr_b = P.thr ? P.thr[b] : neg_inf();
        // the trip count is the same for every lane: the thresholds are wavefront reductions
        // the next round's slot is requested before this round's is worked on: the loads of the rounds
        // overlap with the arithmetic instead of each being waited for in turn
        uint4 raw_next = load_slot<BF16, ALIGNED>(trow, (s0 + tid < s1) ? s0 + tid : s1 - 1, P.V);
        for (long sb = s0; sb < s1; sb += kWG) {
            const long s = sb + tid;
            const bool live = s < s1;
            float z[VE], zd[VE], lnr[VE];
            const uint4 raw = raw_next;
            if (sb + kWG < s1) raw_next = load_slot<BF16, ALIGNED>(trow, (s + kWG < s1) ? s + kWG : s1 - 1, P.V);
            unpack<BF16>(raw, z);
            if (P.thr && P.mode == FSD_SAMPLE) {
                // temperature, then the kept set of top-k / top-p: everything else leaves the draw
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    bad |= !(z[e] < __builtin_inff());
                    const float sv = __fmul_rn(z[e], P.inv_temp);
                    z[e] = (sv >= thr_b) ? sv : neg_inf();
                }
            }
            if (live) {
            float rres[VE];   // strict SD on a tree: p after the chain's rejections, minus the last draft row
            if constexpr (KIND == KIND_TREESD) {
                if (residual) {
                    const int* ch = s_dyn;
                    const float* iz = reinterpret_cast<const float*>(s_dyn + rows);
                    const float* ldv = reinterpret_cast<const float*>(s_dyn + 2 * rows);
#pragma unroll
                    for (int e = 0; e < VE; ++e) rres[e] = hw_exp2(fmaf(z[e], kLog2e, -lt));
                    for (int m = 0; m < nchain; ++m) {
                        const char* dr = P.draft + (static_cast<size_t>(b) * rows + ch[m]) * static_cast<size_t>(P.V) * ES;
                        const uint4 rawd = load_slot<BF16, ALIGNED>(dr, s, P.V);
                        unpack<BF16>(rawd, zd);
                        const float ldm = ldv[m];
                        if (m + 1 < nchain) {
                            const float izm = iz[m];
#pragma unroll
                            for (int e = 0; e < VE; ++e)
                                rres[e] = fmaxf(rres[e] - hw_exp2(fmaf(zd[e], kLog2e, -ldm)), 0.0f) * izm;
                        } else {
#pragma unroll
                            for (int e = 0; e < VE; ++e) rres[e] = rres[e] - hw_exp2(fmaf(zd[e], kLog2e, -ldm));
                        }
                    }
                }
            } else if (residual) {
                const uint4 rawd = load_slot<BF16, ALIGNED>(drow, s, P.V);
                unpack<BF16>(rawd, zd);
            }
            // ln of the residual's entries (-inf where it has no mass)
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                bad |= !(z[e] < __builtin_inff());
                lnr[e] = neg_inf();
                if (residual) {
                    float r;
                    if constexpr (KIND == KIND_TREESD) {
                        r = rres[e];
                    } else {
                        const float p = hw_exp2(fmaf(z[e], kLog2e, -lt));
                        const float qq = hw_exp2(fmaf(zd[e], kLog2e, -ld));
                        r = p - qq;
                    }
                    if (r > 0.0f) lnr[e] = hw_log2(r) * static_cast<float>(kLn2);
                }
            }
            }
            if (P.mode == FSD_SAMPLE) {
                // Bounds of a variate from the position c of the leading one of m = (1 - u) 2^24 alone
                // (c = clz(m) - 8, so 2^-(c+1) <= 1 - u < 2^-c), G = -ln(-ln u) and -ln u between 1 - u and
                // (1 - u)/u:
                //     (c - 1) ln2 <= G <= (c + 1) ln2       (c >= 1; G >= -ln(24 ln2) = -2.8116 always)
                // The largest lower bound of a score in the wavefront is a score the winner must reach, so
                // an entry whose upper bound stays below it (or below a score already seen) cannot be the
                // argmax: its variate, two exact-operation logarithms, is never evaluated.  1e-3 covers
                // the rounding of that routine by a wide margin.
                float gub[VE];
                unsigned w[VE];
                float lo = neg_inf(), rlo = neg_inf();
                if (live) {
#pragma unroll
                    for (int blk = 0; blk < VE / 4; ++blk) {
                        const long e0 = s * VE + blk * 4;
                        const U4 r = philox4x32_10(static_cast<unsigned>(e0 >> 2), static_cast<unsigned>(b), P.off_lo,
                                                   P.off_hi, P.seed_lo, P.seed_hi);
                        w[blk * 4 + 0] = r.x; w[blk * 4 + 1] = r.y; w[blk * 4 + 2] = r.z; w[blk * 4 + 3] = r.w;
                    }
#pragma unroll
                    for (int e = 0; e < VE; ++e) {
                        const unsigned m = 0x00FFFFFFu ^ ((w[e] >> 9) << 1);   // (1 - u) 2^24, odd, >= 1
                        const float c = static_cast<float>(__clz(static_cast<int>(m)) - 8);
                        gub[e] = fmaf(c, 0.693148f, 0.693148f + 1e-3f);
                        const float glb = (c >= 1.0f) ? fmaf(c, 0.693147f, -0.693148f - 1e-3f) : -2.82f;
                        lo = fmaxf(lo, __fadd_rn(z[e], glb));      // (max() drops the NaN of a NaN logit)
                        rlo = fmaxf(rlo, __fadd_rn(lnr[e], glb));
                    }
                }
                thr = fmaxf(thr, wave_max(lo));
                if (residual) rthr = fmaxf(rthr, wave_max(rlo));
                // The entries that are left, at most a few per wavefront: every lane works through its own,
                // lowest index first (one pass of the loop serves one entry of every lane that has any).
                unsigned todo = 0;
                if (live) {
#pragma unroll
                    for (int e = 0; e < VE; ++e) {
                        const bool may = !(__fadd_rn(z[e], gub[e]) < thr) || (residual && !(__fadd_rn(lnr[e], gub[e]) < rthr));
                        todo |= may ? (1u << e) : 0u;
                    }
                }
                while (__any(todo != 0)) {
                    if (todo != 0) {
                        const int e = __builtin_ctz(todo);
                        todo &= todo - 1;
                        float zz = z[0], ll = lnr[0];
                        unsigned ww = w[0];
#pragma unroll
                        for (int i = 1; i < VE; ++i) {
                            zz = (e == i) ? z[i] : zz;
                            ll = (e == i) ? lnr[i] : ll;
                            ww = (e == i) ? w[i] : ww;
                        }
                        const int idx = static_cast<int>(s * VE + e);
                        const float g = gumbel(ww);
                        const float score = __fadd_rn(zz, g);
                        if (score > best.score) best = Best{score, idx};
                        if (ll > neg_inf()) {
                            const float rs = __fadd_rn(ll, g);
                            if (rs > rbest.score) rbest = Best{rs, idx};
                        }
                    }
                }
            } else if (live) {
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    const int idx = static_cast<int>(s * VE + e);
                    if (z[e] > best.score) best = Best{z[e], idx};
                    if (lnr[e] > rbest.score) rbest = Best{lnr[e], idx};
                }
            }
            if (P.mode == FSD_SAMPLE) {
                thr = fmaxf(thr, wave_max(best.score));
                if (residual) rthr = wave_max(rbest.score);
            }
        }
    }
    best = wave_best(best);
    rbest = wave_best(rbest);
    bad = __any(bad);
    if (lane == 0) { s_best[wave] = best; s_best[4 + wave] = rbest; s_bad[wave] = bad; }
    __syncthreads();
    if (tid == 0) {
        Best m = s_best[0], r = s_best[4];
        int bd = s_bad[0];
        for (int k = 1; k < 4; ++k) { m = better(m, s_best[k]); r = better(r, s_best[4 + k]); bd |= s_bad[k]; }
        // The share of this workgroup: three words that say by themselves whether they have arrived.  The
        // sampler's shares are cleared with the exchange words at the start of the call and a posted
        // word is never zero (the index goes out plus one, the flag with bit 1 set), so nothing has to
        // order these stores before the count below: whoever merges looks until the words are there.
        unsigned long long* slot = P.ws.spart + (static_cast<size_t>(b) * P.GS + gs) * 4;
        __hip_atomic_store(slot + 0, (static_cast<unsigned long long>(__float_as_uint(m.score)) << 32) | (static_cast<unsigned>(m.idx) + 1u), __ATOMIC_RELAXED, AGENT);
        __hip_atomic_store(slot + 1, (static_cast<unsigned long long>(__float_as_uint(r.score)) << 32) | (static_cast<unsigned>(r.idx) + 1u), __ATOMIC_RELAXED, AGENT);
        __hip_atomic_store(slot + 2, static_cast<unsigned long long>(bd ? 3 : 2), __ATOMIC_RELAXED, AGENT);
        const unsigned prev = __hip_atomic_fetch_add(P.ws.sdone + static_cast<size_t>(b) * kSdoneStride, 1u, __ATOMIC_RELAXED, AGENT);
        s_last = (prev == static_cast<unsigned>(P.GS) - 1u) ? 1 : 0;
    }
    __syncthreads();
    if (!s_last) return;

    // ---- the last workgroup of the sequence merges the shares and writes the outputs
    if (wave == 0) {   // one share per lane: the loads of all shares are in flight together
        Best m{neg_inf(), 0x7FFFFFFF}, r{neg_inf(), 0x7FFFFFFF};
        int bd = 0;
        bool late = false;
        for (int k = lane; k < P.GS; k += 64) {
            const unsigned long long* slot = P.ws.spart + (static_cast<size_t>(b) * P.GS + k) * 4;
            // every workgroup of the sequence has counted itself, so its words are on their way: normally
            // they are there at the first look (bounded wait otherwise)
            unsigned long long w0 = 0, w1 = 0, w2 = 0;
            for (unsigned polls = 0;; ++polls) {
                w0 = __hip_atomic_load(slot + 0, __ATOMIC_RELAXED, AGENT);
                w1 = __hip_atomic_load(slot + 1, __ATOMIC_RELAXED, AGENT);
                w2 = __hip_atomic_load(slot + 2, __ATOMIC_RELAXED, AGENT);
                if ((w0 != 0 && w1 != 0 && w2 != 0) || polls >= P.spin_limit) break;
                __builtin_amdgcn_s_sleep(1);
            }
            if (w0 == 0 || w1 == 0 || w2 == 0) { late = true; continue; }
            bd |= static_cast<int>(w2 & 1);
            m = better(m, Best{__uint_as_float(static_cast<unsigned>(w0 >> 32)), static_cast<int>(static_cast<unsigned>(w0) - 1u)});
            r = better(r, Best{__uint_as_float(static_cast<unsigned>(w1 >> 32)), static_cast<int>(static_cast<unsigned>(w1) - 1u)});
        }
        m = wave_best(m);
        r = wave_best(r);
        bd = __any(bd);
        late = __any(late);
        if (lane == 0) {
            int st = status;
            if (late) st |= FSD_ROW_INTERNAL;   // a share never arrived (never expected)
            if (!st && (bd || m.idx == 0x7FFFFFFF)) st |= FSD_ROW_NONFINITE;
            const int tok = (residual && r.idx != 0x7FFFFFFF) ? r.idx : m.idx;
            s_st = st;
            s_key = tok;
        }
    }
    __syncthreads();
    status = s_st;
    const int token = s_key;
    if (status) n = 0;
    const int width = (KIND == KIND_TREE || KIND == KIND_TREESD) ? P.max_depth + 1 : rows + 1;
    int32_t* out = P.out_tokens + static_cast<size_t>(b) * width;
    if constexpr (KIND == KIND_TREESD) {
        // the walk has written the path and its tokens; add the drawn token, or take it all back
        if (status) {
            int32_t* pn = P.path_nodes + static_cast<size_t>(b) * P.max_depth;
            for (int i = tid; i < P.max_depth; i += kWG) pn[i] = -1;
            for (int i = tid; i < width; i += kWG) out[i] = -1;
        } else if (tid == 0) {
            out[n] = token;
        }
    } else if constexpr (KIND == KIND_TREE) {
        int32_t* pn = P.path_nodes + static_cast<size_t>(b) * P.max_depth;
        for (int i = tid; i < P.max_depth; i += kWG) pn[i] = -1;
        for (int i = tid; i < width; i += kWG) out[i] = (i == n && !status) ? token : -1;
        __syncthreads();
        if (tid == 0 && !status) {
            const int* par = s_dyn;
            int jn = winner;
            for (int i = n - 1; i >= 0 && jn >= 0; --i) {
                pn[i] = jn;
                out[i] = P.tokens[static_cast<size_t>(b) * rows + jn];
                jn = par[jn];
            }
        }
    } else {
        for (int i = tid; i < width; i += kWG) {
            int v = -1;
            if (!status) {
                if (i < n) v = P.tokens[static_cast<size_t>(b) * rows + i];
                else if (i == n) v = token;
            }
            out[i] = v;
        }
    }
    if (tid == 0) {
        P.out_len[b] = n;
        if (P.row_status) P.row_status[b] = status;
        // The last workgroup of the last sequence to finish: every workgroup of this kernel has posted its
        // share by now, and so has looked at the failure word, which nothing looks at after this kernel.
        // It goes back to zero, so that the same call replayed from a captured graph, with the same
        // number, does not find a failure of the last time.
        const unsigned done = atomicAdd(P.ws.counters + 4, 1u);
        if (done == gridDim.y - 1) {
            __hip_atomic_store(reinterpret_cast<unsigned long long*>(P.ws.counters + 2), 0ull, __ATOMIC_RELAXED, AGENT);
        }
    }
}

}  // namespace

#endif  // FSD_CSRC_ACCEPT_SAMPLE_H_
