// Temperature / top-k / top-p: the smallest kept scaled logit of the row a token is drawn from.
// Part of libfsd (gfx950); included by fsd_kernels.hip, which holds the host side and the C ABI.
#ifndef FSD_CSRC_WARP_SELECT_H_
#define FSD_CSRC_WARP_SELECT_H_

#include "device_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// sampling-method warpers (Sec. 4: the token is drawn with "whatever sampling method the user
// sets"): temperature, then top-k, then top-p, in that order, on the row the token is drawn from.
// One workgroup per sequence finds the smallest kept scaled logit s = z inv_temp:
//   top-k   the k-th largest s, by a radix select over the order-preserving 32-bit image of s
//           (four 8-bit digits, counted from the top);
//   top-p   the largest t with sum_{s >= t} e^(s - max) >= top_p sum_{kept} e^(s - max), by the same
//           select on weights; the weights are 2^40 fixed-point integers, so that the sums do not
//           depend on the order of the atomic additions (results are the same run to run).
// Ties at either threshold are kept.  accept_sample then drops every entry below the threshold.
// Correct first: a row is passed over once per digit by a single workgroup, which costs far more
// than the draw itself when top-k or top-p is on.

__device__ __forceinline__ unsigned ordered_key(float x) {
    const unsigned u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(unsigned k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

struct WarpParams {
    const char* target;
    const int32_t* parent;   // tree: [B,N]; NULL for a chain
    int rows;             // K or N
    long V;
    long nslots;
    float T;
    float inv_temp;
    int top_k;            // 0 = off
    float top_p;          // 1 = off
    float* thr;           // [B] out
    Ws ws;
};

constexpr int kWarpWG = 1024;

// KEEP: the row fits 16 slots per thread (bfloat16 rows up to 131072 entries) and is read once into
// registers; otherwise every pass streams it again, four loads in flight per thread.
constexpr int kWarpKeep = 16;
constexpr int kWarpList = 8192;   // entries the select can finish from LDS
constexpr int kWarpFastK = 512;   // largest top-k (and the candidate depth for top-p alone) of the short way

template <bool BF16, bool ALIGNED, bool KEEP>
__global__ __launch_bounds__(kWarpWG) void warp_select(WarpParams P) {
    constexpr int VE = Slot<BF16>::VE;
    constexpr int ES = BF16 ? 2 : 4;
    __shared__ unsigned long long s_hist[256];
    __shared__ unsigned s_cnt[256];
    __shared__ unsigned long long s_wtot[4];
    __shared__ unsigned s_lkey[kWarpList];
    __shared__ float s_red[kWarpWG / 64];
    __shared__ int s_n, s_st, s_nlist, s_fits;
    __shared__ unsigned s_tmax[kWarpWG];
    __shared__ unsigned long long s_wsum[kWarpWG / 64];
    __shared__ unsigned s_prefix, s_mask, s_match;
    __shared__ unsigned long long s_need;
    __shared__ float s_max;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;

    // ---- the row the token will be drawn from: the first rejected position, or the row after the last
    // (chain); the row after the deepest node whose ancestors are all accepted, lowest index on ties (tree)
    if (tid == 0) { s_n = P.rows; s_st = 0; s_match = 0u; }
    __syncthreads();
    if (P.parent == nullptr) {
        for (int i = tid; i < P.rows; i += kWarpWG) {
            const int pr = b * P.rows + i;
            if (P.ws.pst[pr]) atomicOr(&s_st, 1);
            if (!(P.ws.div[pr] <= P.T)) atomicMin(&s_n, i);
        }
        __syncthreads();
    } else {
        // pointer jumping over the parents, as in accept_sample; the list's memory is free until the select
        const int rows = P.rows;
        int* par = reinterpret_cast<int*>(s_lkey);
        int* anc = par + rows;
        int* acc = anc + rows;
        int* dep = acc + rows;
        for (int j = tid; j < rows; j += kWarpWG) {
            const int pr = b * rows + j;
            int p = P.parent[pr];
            if (p < -1 || p >= j) { atomicOr(&s_st, 1); p = -1; }   // accept_sample reports it
            if (P.ws.pst[pr]) atomicOr(&s_st, 1);
            par[j] = p; anc[j] = p; dep[j] = 1;
            acc[j] = (P.ws.div[pr] <= P.T) ? 1 : 0;
        }
        __syncthreads();
        constexpr int PER = kMaxRows / kWarpWG;
        for (int span = 1; span < rows; span <<= 1) {
            int na[PER], nacc[PER], nd[PER];
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int j = tid + q * kWarpWG;
                if (j < rows) {
                    const int a = anc[j];
                    na[q] = a; nacc[q] = acc[j]; nd[q] = dep[j];
                    if (a >= 0) { na[q] = anc[a]; nacc[q] = acc[j] & acc[a]; nd[q] = dep[j] + dep[a]; }
                }
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int j = tid + q * kWarpWG;
                if (j < rows) { anc[j] = na[q]; acc[j] = nacc[q]; dep[j] = nd[q]; }
            }
            __syncthreads();
        }
        for (int j = tid; j < rows; j += kWarpWG) {
            if (acc[j]) atomicMax(&s_match, (static_cast<unsigned>(dep[j]) << 11) | static_cast<unsigned>(kMaxRows - 1 - j));
        }
        __syncthreads();
        const unsigned key = s_match;
        if (tid == 0) s_n = key ? (kMaxRows - 1 - static_cast<int>(key & (kMaxRows - 1))) + 1 : 0;
        __syncthreads();
    }
    if (s_st || failure_flagged(P.ws)) {   // nothing will be drawn for this sequence
        if (tid == 0) P.thr[b] = neg_inf();
        return;
    }
    const char* row = P.target + (static_cast<size_t>(b) * (P.rows + 1) + s_n) * static_cast<size_t>(P.V) * ES;

    uint4 kept[KEEP ? kWarpKeep : 1];
    if constexpr (KEEP) {
#pragma unroll
        for (int c = 0; c < kWarpKeep; ++c) {
            const long sl = static_cast<long>(c) * kWarpWG + tid;
            kept[c] = load_slot<BF16, ALIGNED>(row, sl < P.nslots ? sl : P.nslots - 1, P.V);
        }
    }
    // one pass over the row: f(scaled logit, key) for every entry
    auto for_slot = [&](const uint4& raw, long sl, auto&& f) __attribute__((always_inline)) {
        float z[VE];
        unpack<BF16>(raw, z);
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            if (ALIGNED || sl * VE + e < P.V) {   // aligned rows have no ragged last slot
                const float sv = __fmul_rn(z[e], P.inv_temp);
                f(sv, ordered_key(sv));
            }
        }
    };
    auto for_each = [&](auto&& f) __attribute__((always_inline)) {
        if constexpr (KEEP) {
#pragma unroll
            for (int c = 0; c < kWarpKeep; ++c) {
                const long sl = static_cast<long>(c) * kWarpWG + tid;
                // the copy is made opaque: what is derived from the kept words (scaled values, keys) would
                // otherwise be hoisted out of the passes and kept as well, far beyond the register file
                uint4 r = kept[c];
                asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w));
                if (sl < P.nslots) for_slot(r, sl, f);
            }
        } else {
            constexpr int CH = 4;
            for (long base = 0; base < P.nslots; base += static_cast<long>(kWarpWG) * CH) {
                uint4 raw[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const long sl = base + static_cast<long>(c) * kWarpWG + tid;
                    raw[c] = load_slot<BF16, ALIGNED>(row, sl < P.nslots ? sl : P.nslots - 1, P.V);
                }
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const long sl = base + static_cast<long>(c) * kWarpWG + tid;
                    if (sl < P.nslots) for_slot(raw[c], sl, f);
                }
            }
        }
    };
    // the workgroup's maximum of m, left in s_max
    auto block_max = [&](float m) __attribute__((always_inline)) {
        m = wave_max(m);
        __syncthreads();
        if (lane == 0) s_red[wave] = m;
        __syncthreads();
        if (tid == 0) {
            float mm = s_red[0];
            for (int w = 1; w < kWarpWG / 64; ++w) mm = fmaxf(mm, s_red[w]);
            s_max = mm;
        }
        __syncthreads();
    };
    // Histogram additions of one thread, merged while consecutive entries fall in the same bin (the
    // leading digit of nearly every entry of a row is the same: adding them one by one would
    // serialise the whole workgroup on one LDS word).  s_hist takes the weights (1 per entry for
    // top-k), s_cnt the number of entries.
    struct Run { int bin; unsigned n; unsigned long long sum; };
    auto run_flush = [&](Run& r) __attribute__((always_inline)) {
        if (r.n) { atomicAdd(&s_hist[r.bin], r.sum); atomicAdd(&s_cnt[r.bin], r.n); }
        r.n = 0;
        r.sum = 0;
    };
    auto run_add = [&](Run& r, int bin, unsigned long long w) __attribute__((always_inline)) {
        if (bin != r.bin) { run_flush(r); r.bin = bin; }
        r.sum += w;
        r.n += 1;
    };
    // From the top: the digit at which the accumulated histogram reaches s_need; updates prefix and
    // need and leaves the number of entries that share the new prefix in s_match.  The 256 sums from
    // the top come from a parallel scan (a single thread walking the bins costs more than a pass
    // over the row); need_of(total), if given, first derives s_need from the histogram's total.
    auto pick_from_top = [&](int shift, auto&& need_of) __attribute__((always_inline)) {
        __syncthreads();
        unsigned long long h = 0, v = 0;
        if (tid < 256) {
            h = s_hist[tid];
            v = h;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned long long x = __shfl_down(v, o);
                if (lane + o < 64) v += x;
            }
            if (lane == 0) s_wtot[wave] = v;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = wave + 1; w < 4; ++w) v += s_wtot[w];   // v = everything in bins >= tid
            if (tid == 0) need_of(v);
        }
        __syncthreads();
        if (tid < 256) {
            const unsigned long long need = s_need, above = v - h;
            const bool here = (v >= need && above < need) || (tid == 0 && v < need);
            if (here) {
                s_prefix |= static_cast<unsigned>(tid) << shift;
                s_mask |= 255u << shift;
                s_need = need - above;
                s_match = s_cnt[tid];
            }
        }
        __syncthreads();
    };
    // Radix select from the top over an array of order-preserving keys in LDS, 8 bits a pass: the
    // smallest key whose entries, together with everything above them, weigh at least s_need.
    // wgt(sv, key) gives an entry's weight (0 = not taking part); first_total, called with the
    // total weight of the first histogram, may set s_need.
    auto lds_select = [&](const unsigned* keys, int n, auto&& wgt, auto&& first_total) __attribute__((always_inline)) {
        if (tid == 0) { s_prefix = 0u; s_mask = 0u; }
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) { s_hist[tid] = 0ull; s_cnt[tid] = 0u; }
            __syncthreads();
            const unsigned prefix = s_prefix, mask = s_mask;
            for (int i = tid; i < n; i += kWarpWG) {
                const unsigned key = keys[i];
                if ((key & mask) == prefix) {
                    const unsigned long long w = wgt(key_value(key), key);
                    if (w) {
                        const int bin = static_cast<int>((key >> shift) & 255u);
                        atomicAdd(&s_hist[bin], w);
                        atomicAdd(&s_cnt[bin], 1u);
                    }
                }
            }
            if (shift == 24) pick_from_top(shift, first_total);
            else pick_from_top(shift, [](unsigned long long) {});
        }
    };
    // The same select over the whole row (the general path): every digit is a pass over the row
    // until the entries that still share the prefix fit the list; then they are gathered there and
    // the remaining digits come from the list.  track_max: the first pass also finds the row's maximum.
    auto row_select = [&](auto&& wgt, auto&& first_total, bool track_max) __attribute__((always_inline)) {
        if (tid == 0) { s_prefix = 0u; s_mask = 0u; }
        bool listed = false;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) { s_hist[tid] = 0ull; s_cnt[tid] = 0u; }
            __syncthreads();
            const unsigned prefix = s_prefix, mask = s_mask;
            if (listed) {
                const int nl = s_nlist;
                for (int i = tid; i < nl; i += kWarpWG) {
                    const unsigned key = s_lkey[i];
                    if ((key & mask) == prefix) {
                        const unsigned long long w = wgt(key_value(key), key);
                        if (w) {
                            const int bin = static_cast<int>((key >> shift) & 255u);
                            atomicAdd(&s_hist[bin], w);
                            atomicAdd(&s_cnt[bin], 1u);
                        }
                    }
                }
            } else {
                Run run{0, 0u, 0ull};
                float m = neg_inf();
                const bool tm = track_max && shift == 24;
                for_each([&](float sv, unsigned key) {
                    if (tm) m = fmaxf(m, sv);
                    if ((key & mask) == prefix) {
                        const unsigned long long w = wgt(sv, key);
                        if (w) run_add(run, static_cast<int>((key >> shift) & 255u), w);
                    }
                });
                run_flush(run);
                if (tm) block_max(m);
            }
            if (shift == 24) pick_from_top(shift, first_total);
            else pick_from_top(shift, [](unsigned long long) {});
            if (!listed && shift >= 16 && s_match <= static_cast<unsigned>(kWarpList)) {
                if (tid == 0) s_nlist = 0;
                __syncthreads();
                const unsigned prefix2 = s_prefix, mask2 = s_mask;
                for_each([&](float sv, unsigned key) {
                    if ((key & mask2) == prefix2 && wgt(sv, key)) {
                        const int at = atomicAdd(&s_nlist, 1);
                        if (at < kWarpList) s_lkey[at] = key;
                    }
                });
                __syncthreads();
                listed = true;
            }
        }
    };

    const bool want_k = P.top_k > 0 && P.top_k < P.V, want_p = P.top_p < 1.0f;
    bool done_k = !want_k, done_p = !want_p, have_max = false;
    float t_k = neg_inf(), t_p = neg_inf();
    float cmax = 0.0f;   // the row's maximum times log2 e, once it is known
    auto one = [&](float, unsigned) __attribute__((always_inline)) -> unsigned long long { return 1ull; };
    // e^(s - max) in 2^-40 units; entries at -inf or below the top-k cut weigh nothing
    auto weight = [&](float sv, unsigned) __attribute__((always_inline)) -> unsigned long long {
        if (!(sv >= t_k)) return 0ull;
        const float w = hw_exp2(fmaf(sv, kLog2e, -cmax));
        return static_cast<unsigned long long>(static_cast<double>(w) * 1099511627776.0 + 0.5);
    };
    auto nucleus_need = [&](unsigned long long Z) __attribute__((always_inline)) -> unsigned long long {
        double need = static_cast<double>(P.top_p) * static_cast<double>(Z);
        unsigned long long n = static_cast<unsigned long long>(need);
        if (static_cast<double>(n) < need) ++n;
        return n ? n : 1ull;
    };

    // ---- the short way, for the usual settings.  Every thread notes the largest entry it sees; the
    // kk-th largest of these 1024 maxima, L, has at least kk entries of the row at or above it, so
    // the k-th largest entry (k <= kk) is one of the entries >= L, and there are few of those (the
    // entries are dealt to the threads without regard to their values): they are gathered in one
    // more pass and everything else happens in LDS.  Two cheap passes instead of one costly pass per
    // digit.  If the list overflows (many equal entries), or a nucleus does not fit in it, the
    // general path below takes over.
    if (want_k ? (P.top_k <= kWarpFastK) : want_p) {
        float m = neg_inf();
        for_each([&](float sv, unsigned) { m = fmaxf(m, sv); });
        s_tmax[tid] = ordered_key(m);
        block_max(m);
        have_max = true;
        cmax = s_max * kLog2e;
        const int kk = want_k ? P.top_k : kWarpFastK;
        if (tid == 0) s_need = static_cast<unsigned long long>(kk);
        __syncthreads();
        lds_select(s_tmax, kWarpWG, one, [](unsigned long long) {});
        const unsigned low = s_prefix;   // key of L
        if (tid == 0) s_nlist = 0;
        __syncthreads();
        unsigned long long zt = 0ull;    // top-p alone: the normaliser runs over the whole row
        for_each([&](float sv, unsigned key) {
            if (!want_k) zt += weight(sv, key);
            if (key >= low) {
                const int at = atomicAdd(&s_nlist, 1);
                if (at < kWarpList) s_lkey[at] = key;
            }
        });
        __syncthreads();
        const int nl = s_nlist;
        if (nl <= kWarpList) {
            if (want_k) {
                if (tid == 0) s_need = static_cast<unsigned long long>(P.top_k);
                __syncthreads();
                lds_select(s_lkey, nl, one, [](unsigned long long) {});
                t_k = key_value(s_prefix);
                done_k = true;
                __syncthreads();
                if (want_p) {   // everything top-k kept is in the list
                    lds_select(s_lkey, nl, weight, [&](unsigned long long Z) { s_need = nucleus_need(Z); });
                    t_p = key_value(s_prefix);
                    done_p = true;
                }
            } else {
                // the row's total weight, then: does the nucleus end inside the list?
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) zt += __shfl_xor(zt, o);
                if (lane == 0) s_wsum[wave] = zt;
                __syncthreads();
                if (tid == 0) {
                    unsigned long long Z = 0;
                    for (int w = 0; w < kWarpWG / 64; ++w) Z += s_wsum[w];
                    s_need = nucleus_need(Z);
                    s_fits = 0;
                }
                __syncthreads();
                lds_select(s_lkey, nl, weight, [&](unsigned long long inlist) { s_fits = (inlist >= s_need) ? 1 : 0; });
                if (s_fits) {
                    t_p = key_value(s_prefix);
                    done_p = true;
                }
            }
        }
        __syncthreads();
    }

    // ---- the general path
    if (!done_k) {
        if (tid == 0) s_need = static_cast<unsigned long long>(P.top_k);
        __syncthreads();
        row_select(one, [](unsigned long long) {}, !have_max);
        have_max = true;
        cmax = s_max * kLog2e;
        t_k = key_value(s_prefix);
        __syncthreads();
    }
    if (!done_p) {
        if (!have_max) {
            float m = neg_inf();
            for_each([&](float sv, unsigned) { m = fmaxf(m, sv); });
            block_max(m);
            cmax = s_max * kLog2e;
        }
        __syncthreads();
        row_select(weight, [&](unsigned long long Z) { s_need = nucleus_need(Z); }, false);
        t_p = key_value(s_prefix);
    }
    if (tid == 0) P.thr[b] = fmaxf(t_k, t_p);
}

}  // namespace

#endif  // FSD_CSRC_WARP_SELECT_H_
