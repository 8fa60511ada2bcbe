// The vocabulary-reduction kernel (softmax normalisers and divergence of every row pair).
// Part of libfsd (gfx950); included by fsd_kernels.hip, which holds the host side and the C ABI.
#ifndef FSD_CSRC_PAIR_KERNEL_H_
#define FSD_CSRC_PAIR_KERNEL_H_

#include "device_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// kernel 1: vocabulary reduction over row pairs
//
// One (target row, draft row) pair is split over a team of GW wavefronts.  Every wavefront loads
// its slice of both rows ONCE into registers (NV 16-byte slots of each row per lane) and works on
// its own: there is no barrier and no shared memory, the wavefronts of a team only meet through
// 64-bit words in the workspace.
//
//   phase 1   maximum of the slice (DPP reduction), integer reference exponent k = ceil(max log2e),
//             e = 2^(z log2e - k) for every entry, their sums; posted as exchange words (two-phase
//             modes: the two exponents in one word, the two sums as binary32 in another).
//   exchange  (two-phase divergences) every wavefront reads the whole team's words and merges them
//             into row-wide normalisers.
//   phase 2   from the kept exponentials: p = e_t f_t, q = e_d f_d, the divergence's terms, one
//             (TV: two) word(s) of partial sums posted.
//   finish    the team's wavefronts take turns as finisher of a pair: it adds the posted partial
//             sums in member order (fixed order: results are bit-identical run to run) and writes
//             divergence and status.
//
// The kernel is persistent and software-pipelined: in a step a wavefront runs phase 1 of pair j
// and then phase 2 of pair j - LAG from an older set of kept exponentials (LAG = 1, or 2 where
// the registers allow a third set).  Memory operations return in the order they were issued,
// which fixes the order of the requests in a step (see `step`): small exchange words first, the
// next pair's logits as soon as phase 1 has consumed the registers (a whole step ahead where a
// second set of logit registers fits), and nothing after that waits on memory unless a team
// member is late.  The bfloat16 two-phase kernels (two wavefronts per SIMD) are bound by
// vector-ALU issue; the binary32 ones (one wavefront per SIMD) by the exposed latencies, which the
// longer lag and the earlier prefetch hide.  The single-pass modes (bfloat16 KL, the normalisers
// of strict SD) have no phase 2.  Waiting is bounded (spin_limit polls, then FSD_ROW_INTERNAL),
// so every wavefront reaches the end of the kernel whatever happens; all team members are
// resident by construction (the grid never exceeds what fits on the device at once).

// The exchange words are only ever touched with device-scope atomic loads and stores, which are
// performed at the memory side: no cache write-back or invalidate is needed to see them.  They are
// cleared before the kernel starts and a posted word is never zero (+0.0 is posted as -0.0), so
// each word says by itself whether it has arrived: no counter or fence sits between a post and
// its use.
__device__ __forceinline__ void post64(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, AGENT);
}
__device__ __forceinline__ unsigned long long read64(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, AGENT);
}
__device__ __forceinline__ unsigned long long dbits(double x) {   // never 0
    const unsigned long long u = static_cast<unsigned long long>(__double_as_longlong(x));
    return u ? u : 0x8000000000000000ull;
}
__device__ __forceinline__ double bitsd(unsigned long long x) {
    return __longlong_as_double(static_cast<long long>(x));
}
__device__ __forceinline__ unsigned fbits(float x) {              // never 0
    const unsigned u = __float_as_uint(x);
    return u ? u : 0x80000000u;
}

// Reference exponents are integers (k = ceil(max * log2e)), so moving a sum from one reference
// to another is an exact scaling by a power of two.
__device__ __forceinline__ int kdiff(float k, float M) { return static_cast<int>(k - M); }

// two binary32 values in one exchange word (never 0: +0.0 in the low half is posted as -0.0)
__device__ __forceinline__ unsigned long long pack2(float lo, float hi) {
    return static_cast<unsigned long long>(fbits(lo)) | (static_cast<unsigned long long>(__float_as_uint(hi)) << 32);
}
__device__ __forceinline__ float lo_f(unsigned long long w) { return __uint_as_float(static_cast<unsigned>(w)); }
__device__ __forceinline__ float hi_f(unsigned long long w) { return __uint_as_float(static_cast<unsigned>(w >> 32)); }

// A pair owns N GW words of an exchange array, N per member (what the mode uses): word k of member
// m sits at [m N + k], so that a member's post is one contiguous store and the 64 lanes of a
// request touch consecutive words.  Lane l reads the N words of member (base + l); lanes beyond
// the team re-read the last member's (no branch around the loads, see load_item).  Nothing looks at the values here, so the loads stay in flight until they are
// awaited.  With spread == false every lane reads member 0 (a request whose result is not needed
// costs one cache line).
// word i of a pair's words: a 32-bit byte offset added to a pointer that stays scalar
__device__ __forceinline__ unsigned long long* word_at(unsigned long long* p, unsigned i) {
    return reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(p) + i * 8u);
}
__device__ __forceinline__ const unsigned long long* word_at(const unsigned long long* p, unsigned i) {
    return reinterpret_cast<const unsigned long long*>(reinterpret_cast<const char*>(p) + i * 8u);
}
template <int N>
__device__ __forceinline__ void request_n(const unsigned long long* p, int GW, int base, unsigned long long (&w)[N],
                                          bool spread = true) {
    const int m = base + static_cast<int>(threadIdx.x & 63);
    const int mm = spread ? ((m < GW) ? m : GW - 1) : 0;
    const unsigned long long* const mine = word_at(p, static_cast<unsigned>(mm * N));
#pragma unroll
    for (int k = 0; k < N; ++k) w[k] = read64(mine + k);
}
// The words are normally there when they are looked at.  Everything that loops over memory (asking
// again, further rounds of 64 members) lives in functions that are NOT inlined: the compiler's
// bookkeeping of outstanding memory operations stays exact in the caller, which then never waits
// for the logits it has just requested for the next pair.
template <int N> struct WordsN { unsigned long long w[N]; bool ok; };

template <int N>
__device__ __noinline__ WordsN<N> repoll_n(const unsigned long long* p, int GW, int base, unsigned limit) {
    WordsN<N> r;
    r.ok = true;
    unsigned polls = 0;
    for (;;) {
        request_n<N>(p, GW, base, r.w);
        bool missing = false;   // duplicates included: harmless
#pragma unroll
        for (int k = 0; k < N; ++k) missing |= (r.w[k] == 0);
        if (!__any(missing)) break;
        if (polls++ >= limit) { r.ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
    }
    return r;
}
template <int N>
__device__ __forceinline__ bool await_n(const unsigned long long* p, int GW, int base, unsigned limit,
                                        unsigned long long (&w)[N]) {
    bool missing = false;
#pragma unroll
    for (int k = 0; k < N; ++k) missing |= (w[k] == 0);
    if (!__any(missing)) return true;
    const WordsN<N> r = repoll_n<N>(p, GW, base, limit);
#pragma unroll
    for (int k = 0; k < N; ++k) w[k] = r.w[k];
    return r.ok;
}

// binary32 merge of one round of team words (two-phase format: word 0 = the two reference
// exponents, word 1 = the two sums) into sums relative to the fixed references (n.Kt, n.Kd): the
// reading wavefront's own exponents.  Exact power-of-two rescaling; a member far above the reader
// makes the sum overflow to +inf, the reader's factor 1/sum is then 0, and so are its p and q:
// they are below 2^-127 of the row's mass.
struct TeamNorm { float Kt, Kd, zt, zd; bool ok; };

// one member's sums moved to the references (0 for a lane beyond the team; NaN stays NaN)
__device__ __forceinline__ void member_terms(const unsigned long long (&w)[2], bool in, const TeamNorm& n, float& at, float& ad) {
    // (a zero stays zero and a NaN stays NaN under the scaling: no case distinction is needed)
    at = ldexpf(in ? lo_f(w[1]) : 0.0f, kdiff(lo_f(w[0]), n.Kt));
    ad = ldexpf(in ? hi_f(w[1]) : 0.0f, kdiff(hi_f(w[0]), n.Kd));
}
__device__ __forceinline__ void merge_round(const unsigned long long (&w)[2], bool in, TeamNorm& n) {
    float at, ad;
    member_terms(w, in, n, at, ad);
    wave_sumf2(at, ad);
    n.zt += at;
    n.zd += ad;
}
// teams of more than 64 wavefronts: the members beyond the first round
__device__ __noinline__ TeamNorm merge_more_rounds(const unsigned long long* p1, int GW, unsigned limit, TeamNorm n) {
    for (int base = 128; base < GW; base += 64) {
        const WordsN<2> r = repoll_n<2>(p1, GW, base, limit);
        if (!r.ok) n.ok = false;
        merge_round(r.w, base + static_cast<int>(threadIdx.x & 63) < GW, n);
    }
    return n;
}
// the divergence words of the members beyond the first round, added in member order (each word
// holds two binary32 partial sums)
template <int N> struct Sums { double lo[N], hi[N]; bool ok; };

template <int N>
__device__ __noinline__ Sums<N> sum_more_rounds(const unsigned long long* p2, int GW, unsigned limit, Sums<N> s) {
    for (int base = 64; base < GW; base += 64) {
        const WordsN<N> r = repoll_n<N>(p2, GW, base, limit);
        if (!r.ok) s.ok = false;
        const bool in = base + static_cast<int>(threadIdx.x & 63) < GW;
#pragma unroll
        for (int k = 0; k < N; ++k) {
            s.lo[k] += wave_sum(in ? static_cast<double>(lo_f(r.w[k])) : 0.0);
            s.hi[k] += wave_sum(in ? static_cast<double>(hi_f(r.w[k])) : 0.0);
        }
    }
    return s;
}

// ------------------------------------------------------------------------------------------
// JS in entropy form (MODE_JSE, bfloat16 logits).  With p, q the two softmaxes and s = p + q,
//
//     JS = ln2 + (1/2) [ sum p ln p + sum q ln q - sum s ln s ]        (App. C.2, rearranged)
//
// Phase 1 keeps e = 2^x per entry (x = z log2e - k) and adds up S = sum e and A = sum e x, one fused
// multiply-add per logit more than the normalisers need.  Phase 2 knows the row sums, hence the
// member's factors f_t, f_d and c = f_d/f_t, forms u = e_t + c e_d = s/f_t and adds up U = sum u log2 u:
// one logarithm per entry where the pointwise form p ln(2p/s) + q ln(2q/s) needs a reciprocal and
// two.  With W = S_t + c S_d the mass of u, a member's share of 2 JS/ln2 is then
//
//     C = f_t [ A_t + c A_d - U + W + c S_d log2 c ]
//
// (write every logarithm as log2 f + log2 e: the terms in log2 f_t cancel because W is the mass of
// u, and log2 of 2 gives the W).  All five sums run over the same entries, so a lane combines its
// own five first (its part of the bracket is the sum of its entries' pointwise terms: small, where
// the separate sums are of the size of the entropies and cancel), one reduction over the wavefront
// follows, and C is posted as one word; the pair's finisher only adds the team's C.
// This removes a third of the kernel's instructions.  The price is what is left of the
// cancellation: the result carries an ABSOLUTE error that does not shrink with it (measured over
// vocabularies of 32 000 to 256 000: at most 1.4e-7 for results below 0.05, up to 1e-6 for results
// of order 0.5, which is 2e-6 of them).  Results below P.js_floor are therefore evaluated a
// second time in the pointwise form, by the same team, after its last pair (bit-identical rows give
// exactly 0 that way).
//
// Exchange words of this mode (zero = not posted yet):
//   part1 [pair][member][2]   (kt, kd) reference exponents | (St, Sd) sums of exponentials
//                             -- second evaluation: word 1 becomes (partial, -1); a sum is never -1
//   part2 [pair][member]      C as float64 bits
//   state [pair]              all ones = finished; else (L_t, L_d), the rows' log2-sum-exp2: evaluate again
constexpr unsigned long long kJsDone = ~0ull;
constexpr unsigned kJsFill = 0xF149F149u; // two bfloat16 of about -1e30: an entry no lane owns (exponential 0, e x = 0)

// The rows' log2-sum-exp2 from a pair's phase-1 words, merged in float64 over rounds of 64 members
// (exact rescaling between reference exponents).  Not inlined: used where a pair is evaluated a
// second time, which is rare.
struct RowNorms { double lse2_t, lse2_d; bool ok, usable; };
__device__ __noinline__ RowNorms row_norms(const unsigned long long* p1, int GW, unsigned limit) {
    const int lane = threadIdx.x & 63;
    float Kt = neg_inf(), Kd = neg_inf();
    double Zt = 0.0, Zd = 0.0;
    RowNorms r;
    r.ok = true;
    bool bad = false;
    for (int base = 0; base < GW; base += 64) {
        const WordsN<2> q = repoll_n<2>(p1, GW, base, limit);
        r.ok &= q.ok;
        const bool in = base + lane < GW;
        const float kt = lo_f(q.w[0]), kd = hi_f(q.w[0]);
        const double St = in ? static_cast<double>(lo_f(q.w[1])) : 0.0, Sd = in ? static_cast<double>(hi_f(q.w[1])) : 0.0;
        bad |= __any(!(St >= 0.0 && St < __builtin_inf() && Sd >= 0.0 && Sd < __builtin_inf())) != 0;
        const float nKt = fmaxf(Kt, wave_max((St > 0.0) ? kt : neg_inf()));
        const float nKd = fmaxf(Kd, wave_max((Sd > 0.0) ? kd : neg_inf()));
        Zt = ((Zt > 0.0) ? ldexp(Zt, kdiff(Kt, nKt)) : Zt) + wave_sum((St > 0.0) ? ldexp(St, kdiff(kt, nKt)) : 0.0);
        Zd = ((Zd > 0.0) ? ldexp(Zd, kdiff(Kd, nKd)) : Zd) + wave_sum((Sd > 0.0) ? ldexp(Sd, kdiff(kd, nKd)) : 0.0);
        Kt = nKt;
        Kd = nKd;
    }
    r.usable = !bad && Zt > 0.0 && Zd > 0.0 && Zt < __builtin_inf() && Zd < __builtin_inf() && Kt < __builtin_inff() &&
               Kd < __builtin_inff();
    r.lse2_t = static_cast<double>(Kt) + log2(Zt);
    r.lse2_d = static_cast<double>(Kd) + log2(Zd);
    return r;
}

// further rounds of 64 members of a sum of float64 words (teams of more than 64)
struct SumMore { double sum; bool ok; };
__device__ __noinline__ SumMore sum_f64_more_rounds(const unsigned long long* p2, int GW, unsigned limit, double sum) {
    const int lane = threadIdx.x & 63;
    SumMore r{sum, true};
    for (int base = 64; base < GW; base += 64) {
        const WordsN<1> q = repoll_n<1>(p2, GW, base, limit);
        r.ok &= q.ok;
        r.sum += wave_sum((base + lane < GW) ? __longlong_as_double(static_cast<long long>(q.w[0])) : 0.0);
    }
    return r;
}

// The pointwise form of App. C.2 over this wavefront's slice of one pair, from the rows' log2-sum-exp2:
// p = 2^(a log2e - L_t), q likewise, sum of p log2(2p/s) + q log2(2q/s).  Not pipelined: used for the
// few pairs whose entropy-form result is below the floor.
template <int NV, bool ALIGNED>
__device__ __noinline__ float js_pointwise_slice(const char* tptr, const char* dptr, long V, int sl0, int sl_end,
                                                 int sl_last, float Lt, float Ld) {
    float acc = 0.0f;
#pragma unroll 1
    for (int k = 0; k < NV; ++k) {
        const int sk = sl0 + 64 * k;
        const bool own = sk < sl_end;
        const long sl = own ? sk : sl_last;
        uint4 ra = load_slot<true, ALIGNED, false>(tptr, sl, V);
        uint4 rb = load_slot<true, ALIGNED, false>(dptr, sl, V);
        if (!own) { ra = slot_neg_inf<true>(); rb = slot_neg_inf<true>(); }
        float a[8], c[8];
        unpack<true>(ra, a);
        unpack<true>(rb, c);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = hw_exp2(fmaf(a[e], kLog2e, -Lt));
            const float q = hw_exp2(fmaf(c[e], kLog2e, -Ld));
            const float d = p - q, sum = p + q;
            // p = q = 0: 0 * inf = NaN, which max() drops (u = tiny, v = 2, both weights zero)
            const float inv = __builtin_amdgcn_rcpf(sum);
            const float u = fmaxf(fmaf(d, inv, 1.0f), 2e-38f), v = fmaxf(2.0f - u, 2e-38f);
            acc = fmaf(p, hw_log2(u), acc);
            acc = fmaf(q, hw_log2(v), acc);
        }
    }
    return wave_sumf(acc);
}

template <int I> struct SetId { static constexpr int value = I; };
template <bool B> struct BoolTag { static constexpr bool value = B; };

// wavefronts per SIMD the register allocation has to leave room for
constexpr int pair_kernel_waves(bool bf16, int nv, int mode) {
    return (bf16 && (((nv == 5 || nv == 6) && (mode == MODE_JS || mode == MODE_TV)) || mode == MODE_JSE)) ? 2 : 1;
}

// TSHARED: target rows are shared between pairs (a tree) and are loaded to stay cached (a template
// parameter, not a run-time decision: see load_item).
// ---- a call without a clearing kernel ---------------------------------------------------------
// Every kernel in a stream costs 4-5 us before its first instruction, whatever it does, so the plain
// calls do not launch one to clear the exchange words: the reduction's own wavefronts do it.  A
// wavefront clears its share of the words of its team's pairs (below) and a slice of what no team
// owns (the sampler's shares and counters, which the sampler only touches after this kernel has
// ended), waits until those stores have been performed, and writes the call's number into its slot
// of `arrive`.  Nobody reads or, after its first step, writes a word of a pair but the members of
// the pair's team, so a wavefront that has seen the call's number in the slots of all members of
// its team, which it waits for at the end of its first step, can take any word of theirs that is
// not zero as posted, and post to any word of the team's later pairs.  The
// slots are never cleared before a call: what an earlier call or the allocation left there is not
// this call's number.  (A captured call is replayed with the same number: the sampler, which follows
// in every call, clears the slots again.)
template <int N1, int PW, bool TWO_PHASE, bool JSE>
__device__ __noinline__ void clear_own_words(unsigned long long* part1, unsigned long long* part2, unsigned long long* state,
                                             uint4* clear_a, long a16, uint4* clear_b, long b16, int gwave, int nwaves,
                                             int member, int GW, int pair0, int pstep, int n_mine) {
    const int lane = threadIdx.x & 63;
    if (n_mine > 0) {
        // The team's first pair: every member its own words, because it posts them in its first step, before
        // it knows that the others have started.
        const size_t pr = static_cast<size_t>(pair0);
        if (lane < N1) post64(part1 + (pr * GW + member) * N1 + lane, 0ull);
        if constexpr (TWO_PHASE) {
            if (lane < PW) post64(part2 + (pr * GW + member) * PW + lane, 0ull);
        }
    }
    // The later pairs are posted to after the first step, when the whole team has announced itself: their
    // words are dealt to the members pair by pair, all members' words of a pair in one run of stores
    // (a member clearing its own word of every pair would write 8 bytes per memory line: +24 us at
    // 4096 pairs of 76 members).
    for (int idx = 1 + member; idx < n_mine; idx += GW) {
        const size_t pr = static_cast<size_t>(pair0) + static_cast<size_t>(idx) * pstep;
        unsigned long long* const w1 = part1 + pr * GW * N1;
        for (int w = lane; w < GW * N1; w += 64) post64(w1 + w, 0ull);
        if constexpr (TWO_PHASE) {
            unsigned long long* const w2 = part2 + pr * GW * PW;
            for (int w = lane; w < GW * PW; w += 64) post64(w2 + w, 0ull);
        }
    }
    if constexpr (JSE) {   // (a state word is posted by its pair's finisher, steps after the pair's phase 1)
        for (int idx = member * 64 + lane; idx < n_mine; idx += GW * 64)
            post64(state + static_cast<size_t>(pair0) + static_cast<size_t>(idx) * pstep, 0ull);
    }
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    for (long i = static_cast<long>(gwave) * 64 + lane; i < a16; i += static_cast<long>(nwaves) * 64) clear_a[i] = zero;
    for (long i = static_cast<long>(gwave) * 64 + lane; i < b16; i += static_cast<long>(nwaves) * 64) clear_b[i] = zero;
    // (the stores are still on their way when this returns: see where the wavefront announces itself)
}
// all members of the team have announced themselves (bounded wait)
__device__ __noinline__ bool team_arrived(const unsigned long long* slots, int GW, unsigned long long nonce, unsigned limit) {
    const int lane = threadIdx.x & 63;
    for (int base = 0; base < GW; base += 64) {
        const int m = base + lane;
        const unsigned long long* const p = slots + ((m < GW) ? m : GW - 1);
        unsigned polls = 0;
        for (;;) {
            const unsigned long long v = read64(p);
            if (!__any(v != nonce)) break;
            if (polls++ >= limit) return false;
            __builtin_amdgcn_s_sleep(1);
        }
    }
    return true;
}

template <bool BF16, int NV, int MODE, bool ALIGNED, bool TSHARED = false>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(pair_kernel_waves(BF16, NV, MODE))))
void pair_kernel(PairParams P) {
    constexpr int VE = Slot<BF16>::VE;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr bool TWO_PHASE = (MODE == MODE_JS || MODE == MODE_TV || MODE == MODE_KLP || MODE == MODE_JSE);
    constexpr bool JSE = (MODE == MODE_JSE);   // bfloat16 only (the host sends binary32 JS to MODE_JS)
    constexpr bool RECOMPUTE_SLOTS = JSE && TSHARED;   // (the tree variant of the entropy form is the one short of registers)
    constexpr bool SHARE = JSE && TSHARED;     // consecutive pairs with one target row share its phase 1 (see step)
    constexpr int NE = TWO_PHASE ? NV * VE : 1;   // exponentials kept per row and lane
    constexpr int PW = (MODE == MODE_TV || MODE == MODE_KLP) ? 2 : 1;   // divergence words a member posts (two sums each)
    constexpr int FW = TWO_PHASE ? PW : 4;          // words per member the finisher reads
    constexpr int N1 = TWO_PHASE ? 2 : 4;           // phase-1 words a member posts; both exchange arrays are
                                                    // dense, [pair][member][word]: only what a mode uses is cleared
    // binary32 logits: the two-phase kernels hold 8 slots of each row per lane and one wavefront per
    // SIMD anyway, which leaves registers for a second set of logits
    constexpr bool DEEP = !BF16 && TWO_PHASE && NV == 8;
    // Phase 2 of a pair runs LAG steps after its phase 1.  With one step, a wavefront's own chain
    // from one phase 1 to the next still holds the whole latency of the exchange (post, then the
    // slowest member's words), which only another wavefront on the same SIMD can fill; with two,
    // every member's words have long been posted when they are looked at.  That takes a third set
    // of kept exponentials: the binary32 kernels with 8 slots per lane run one wavefront per SIMD
    // and have the registers.  (The bfloat16 kernels run two per SIMD and are bound by vector-ALU
    // issue: a third set kept in LDS removed their waits and left their time unchanged, for the
    // pointwise kernels and again for the entropy-form one at 4 slots per lane, also with the team's
    // words requested a whole step before they are used.)
    constexpr int LAG = (TWO_PHASE && !BF16 && NV == 8) ? 2 : 1;
    constexpr int NB = LAG + 1;                      // sets of kept exponentials
    constexpr int NC = (NE + 3) / 4;                 // chunks of four per row
    constexpr float kTiny = 2e-38f;   // floor of u and v under the logarithm (their weights are then zero or negligible),
                                      // and of p and q where both are normalised (KL)
    constexpr int kWavesPerWG = kWG / 64;

    // the wavefront's number as a scalar: everything derived from it (member, slot range, exchange
    // addresses) then lives in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    // NB sets of kept exponentials, named by SetId<> so that every index is a constant and the
    // arrays stay in registers; accessed four at a time
    float et[NB][NE], ed[NB][NE];
    // The last NL chunks of each set live in LDS instead of registers (each lane reads back only what it
    // wrote itself: no barrier; LDS traffic is counted apart from the loads of the logits, so waiting for it
    // does not wait for the prefetch as a spill would).  The bfloat16 two-phase kernels keep 5 of their 12
    // chunks there: that is what lets them hold 6 slots per lane (96 logits a step) in 256 registers,
    // and with two workgroups of 80 KB it takes all of a compute unit's LDS.  (TV at 5 slots per lane,
    // a shape of the tuning hook, keeps one.)
    constexpr int NL = (JSE || (BF16 && NV == 6 && TWO_PHASE)) ? 5 : (BF16 && NV == 5 && MODE == MODE_TV) ? 1 : 0;   // (the least that leaves no register spilled, per variant)
    __shared__ float4 lds_keep[NL ? NB * NL * 2 * kWG : 1];
    auto put4 = [&](auto S, int c, const float (&t4)[4], const float (&d4)[4]) __attribute__((always_inline)) {
        constexpr int s_ = decltype(S)::value;
        if (NL > 0 && c >= NC - NL) {
            float4* const at = lds_keep + ((s_ * NL + (c - (NC - NL))) * 2) * kWG + threadIdx.x;
            at[0] = make_float4(t4[0], t4[1], t4[2], t4[3]);
            at[kWG] = make_float4(d4[0], d4[1], d4[2], d4[3]);
            return;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) { et[s_][4 * c + i] = t4[i]; ed[s_][4 * c + i] = d4[i]; }
    };
    auto get4 = [&](auto S, int c, float (&t4)[4], float (&d4)[4]) __attribute__((always_inline)) {
        constexpr int s_ = decltype(S)::value;
        if (NL > 0 && c >= NC - NL) {
            const float4* const at = lds_keep + ((s_ * NL + (c - (NC - NL))) * 2) * kWG + threadIdx.x;
            const float4 a = at[0], b = at[kWG];
            t4[0] = a.x; t4[1] = a.y; t4[2] = a.z; t4[3] = a.w;
            d4[0] = b.x; d4[1] = b.y; d4[2] = b.z; d4[3] = b.w;
            return;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) { t4[i] = et[s_][4 * c + i]; d4[i] = ed[s_][4 * c + i]; }
    };
    const int GW = P.G;                                   // wavefronts per pair
    // first exchange word of a pair in an array of n words per member
    auto words_at = [&](int pr, int n) __attribute__((always_inline)) -> size_t {
        return static_cast<size_t>(pr) * static_cast<size_t>(GW * n);
    };
    // A team is a run of GW consecutive wavefronts of the grid (workgroup boundaries do not matter: the
    // wavefronts of a workgroup share nothing), which the dispatcher spreads over the XCDs.  (Two
    // other deals were measured at C2 and dropped: teams whose workgroups all sit on one XCD ran a
    // third slower, and teams made half of early and half of late arrivals on the compute units
    // ended together but no sooner.)  The grid is rounded up to whole workgroups: the wavefronts
    // beyond the last team leave at once.
    const int nteams = P.nteams;
    const int gwave = static_cast<int>(blockIdx.x) * kWavesPerWG + wave;
    const int team = gwave / GW;
    if (team >= nteams) return;
    // Which pairs a team takes.  A chain: every nteams-th pair.  A tree: a run of consecutive pairs,
    // because the children of a node are numbered in a row and share their target row: the second
    // child's loads then find it in the cache its first child's loads filled one step earlier.
    const bool runs = (P.parent != nullptr);
    const int per_team = (P.npairs + nteams - 1) / nteams;
    const int pstep = runs ? 1 : nteams;
    const int pair0 = runs ? team * per_team : team;
    const int pair_end = runs ? ((pair0 + per_team < P.npairs) ? pair0 + per_team : P.npairs) : P.npairs;
    const int member = gwave - team * GW;
    const long s0 = static_cast<long>(member) * P.spm;
    const long s1 = (s0 + P.spm < P.nslots) ? s0 + P.spm : P.nslots;
    unsigned long long* const part1 = P.ws.part1;
    unsigned long long* const part2 = reinterpret_cast<unsigned long long*>(P.ws.part2);
    // the words the finisher of a pair reads: divergence sums (two-phase) or phase-1 words
    unsigned long long* const finw = TWO_PHASE ? part2 : part1;
#ifdef FSD_PHASE_TIMING
    unsigned long long pt_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const unsigned long long pt_wall = wall_clock64();
    const unsigned long long pt_first = __builtin_readcyclecounter();
    unsigned long long pt_last = pt_first;
#endif

    // the rows of pair (sequence b, position or node j)
    auto row_ptrs_bj = [&](int pair, int b, int j, const char*& tptr, const char*& dptr) __attribute__((always_inline)) {
        int trow = j;
        if (P.parent) {
            // an input nobody writes, read at an address all lanes share: through the constant address
            // space it is a scalar load, which is not counted with the vector loads (waiting for a vector
            // load here would wait for every request in flight, and make every later wait conservative)
            typedef const int __attribute__((address_space(4))) * ConstInts;
            const int par = ((ConstInts)(P.parent))[pair];
            trow = (par >= -1 && par < j) ? par + 1 : 0;   // invalid parents are reported by the next kernel
        }
        tptr = P.target + (static_cast<size_t>(b) * (P.rows + 1) + trow) * static_cast<size_t>(P.V) * ES;
        dptr = P.draft + static_cast<size_t>(pair) * static_cast<size_t>(P.V) * ES;
    };
    auto row_ptrs = [&](int pair, const char*& tptr, const char*& dptr) __attribute__((always_inline)) {
        const int b = pair / P.rows;
        row_ptrs_bj(pair, b, pair - b * P.rows, tptr, dptr);
    };
    // (sequence, row) of the pair whose logits are requested next: the pairs of a team are an arithmetic
    // sequence, so these advance by a fixed amount and no step pays for a division
    const int step_b = pstep / P.rows, step_j = pstep - step_b * P.rows;
    int load_pair = pair0, load_b = pair0 / P.rows, load_j = pair0 - load_b * P.rows;
    // ---- the only HBM reads of the reduction: NV slots of each row per lane
    // Every lane always loads (a lane without a slot of its own re-reads a valid one and the value is
    // replaced by -inf afterwards): loads that sit inside branches would make the compiler wait for
    // all outstanding memory operations at every later use, and the prefetch would no longer overlap.
    // Slot k of this lane is sl0 + 64 k; it is the lane's own while below s1 (computed where needed:
    // kept per slot, these would cost registers the two-phase kernels do not have).
    const int sl0 = static_cast<int>(s0) + lane;
    const int sl_last = (s1 > s0) ? static_cast<int>(s1) - 1 : 0;
    const int sl_end = static_cast<int>(s1);
    const bool fill_needed = s0 + NV * 64 > s1;   // wavefront-uniform: some lane lacks a slot
    // target rows of the pair in work, of the one before it and of the one requested last (entropy-form JS on
    // a tree: a pair whose target row is its predecessor's takes over that row's exponentials and sums)
    const char *tp_prev = nullptr, *tp_cur = nullptr, *tp_next = nullptr;
    auto load_item = [&](uint4 (&ra)[NV], uint4 (&rb)[NV], int pair, bool wanted = true) __attribute__((always_inline)) {
        const char *tptr, *dptr;
        // the requests come in the order of the team's pairs (the last one may be repeated)
        while (load_pair < pair) {
            load_pair += pstep;
            load_j += step_j;
            load_b += step_b;
            if (load_j >= P.rows) { load_j -= P.rows; ++load_b; }
        }
        row_ptrs_bj(pair, load_b, load_j, tptr, dptr);
        tp_next = tptr;
        // A draft row is read once.  So is a target row of a chain (but for the one the token is drawn
        // from); in a tree the children of a node share their parent's target row, which should stay
        // cached (TSHARED).  One copy of these loads, whatever the input: with two, in the arms of a
        // run-time branch, the compiler's count of requests in flight is no longer exact after the join,
        // and every later wait for an exchange word also waits for most of this prefetch.
        // (where registers are short the lane's slots are formed again at every request instead of
        // being kept: hidden from the hoisting of loop invariants)
        int first = sl0;
        if constexpr (RECOMPUTE_SLOTS) asm volatile("" : "+v"(first));
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int sk = first + 64 * k;
            const long sl = wanted ? (sk < sl_end ? sk : sl_last) : 0;   // not wanted: one cached slot for all lanes
            ra[k] = load_slot<BF16, ALIGNED, !TSHARED>(tptr, sl, P.V);
            rb[k] = load_slot<BF16, ALIGNED, true>(dptr, sl, P.V);
        }
    };
    auto fill_unowned = [&](uint4 (&ra)[NV], uint4 (&rb)[NV]) __attribute__((always_inline)) {
        if (fill_needed) {
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                // first the question that has one answer for the whole wavefront (does slot k reach past
                // the slice at all?): a scalar branch skips the full slots, and only the one or two at the
                // end of the slice go through the per-lane selection
                if (s0 + 64 * (k + 1) > s1) {
                    if constexpr (JSE) {
                        // (a finite logit far below everything: exponential 0 and e x = 0, where -inf gives NaN)
                        asm volatile("");   // stays a branch: only a team's last member with slots has such lanes
                        if (sl0 + 64 * k >= sl_end) {
                            ra[k] = make_uint4(kJsFill, kJsFill, kJsFill, kJsFill);
                            rb[k] = make_uint4(kJsFill, kJsFill, kJsFill, kJsFill);
                        }
                    } else {
                        if (sl0 + 64 * k >= sl_end) { ra[k] = slot_neg_inf<BF16>(); rb[k] = slot_neg_inf<BF16>(); }
                    }
                }
            }
        }
    };

    // strict SD's ln p(x) - ln q(x) at the candidate token (Sec. 3, eq. 1) from the rows' log2-sum-exp2;
    // lane 0 only.  Returns the status bits it adds.
    auto write_ratio = [&](int pair, double lse2_t, double lse2_d, int status, float* user) __attribute__((always_inline)) -> int {
        const int x = P.cand[pair];
        double ratio = __builtin_nan("");
        int add = 0;
        if (x < 0 || x >= P.V) {
            add = FSD_ROW_BAD_TOKEN;
        } else if (!(status & FSD_ROW_NONFINITE)) {
            const char *tptr, *dptr;
            row_ptrs(pair, tptr, dptr);
            const double lp = static_cast<double>(load_elem<BF16>(tptr, x)) - lse2_t * kLn2;
            const double lq = static_cast<double>(load_elem<BF16>(dptr, x)) - lse2_d * kLn2;
            ratio = (lp == -__builtin_inf()) ? -__builtin_inf() : lp - lq;
        }
        P.ws.lr[pair] = ratio;
        if (user) user[pair] = static_cast<float>(ratio);
        return add;
    };

    // ---- finishing a pair: add what the team posted for it, in member order.  fw holds the words of
    // the first 64 members, requested earlier.
    auto finish_two_phase = [&](int pair, unsigned long long (&fw)[FW]) __attribute__((always_inline)) {
        const unsigned long long* p2 = part2 + words_at(pair, PW);
        unsigned long long f[PW];
#pragma unroll
        for (int k = 0; k < PW; ++k) f[k] = fw[k % FW];
        Sums<PW> s;
        s.ok = await_n<PW>(p2, GW, 0, P.spin_limit, f);
#pragma unroll
        for (int k = 0; k < PW; ++k) {
            s.lo[k] = wave_sum((lane < GW) ? static_cast<double>(lo_f(f[k])) : 0.0);
            s.hi[k] = wave_sum((lane < GW) ? static_cast<double>(hi_f(f[k])) : 0.0);
        }
        if (GW > 64) s = sum_more_rounds<PW>(p2, GW, P.spin_limit, s);
        double value;
        if constexpr (MODE == MODE_TV) {
            // the sums of (p - q)+ and of (q - p)+ are the same number; the side that avoids the
            // heavy entries (smaller sum of p + q over its entries) carries the smaller rounding
            // error, which matters for nearly one-hot rows
            // (the two rows' masses add up to 2, so the side of (p - q)+ is the lighter one when the
            // p + q it covers is at most 1)
            const double A = s.lo[0], Bn = s.hi[0], MA = s.lo[1];
            value = (MA != MA) ? __builtin_nan("") : (MA <= 1.0 ? A : Bn);
        } else {
            value = 0.5 * kLn2 * s.lo[0];
        }
        bool log_domain = false;
        if constexpr (MODE == MODE_KLP) log_domain = s.lo[1] > 0.0 && value < __builtin_inf();   // some term saturated
        int status = 0;
        if (value != value) status |= FSD_ROW_NONFINITE;   // NaN / +inf logits, or a row without mass
        if (!s.ok) status |= FSD_ROW_INTERNAL;
        if (value < 0.0) value = 0.0;
        if (status) value = __builtin_nan("");
        double lse2_t = 0.0, lse2_d = 0.0;
        if (P.want_ratio || log_domain) {
            // reducible FSD also needs the rows' normalisers: the team's phase-1 words once more, this
            // time merged in float64 (they were all posted before the divergence words read above)
            const unsigned long long* p1 = part1 + words_at(pair, N1);
            float Kt = neg_inf(), Kd = neg_inf();
            double Zt = 0.0, Zd = 0.0;
            bool ok = true;
            for (int base = 0; base < GW; base += 64) {
                const WordsN<2> r = repoll_n<2>(p1, GW, base, P.spin_limit);
                ok &= r.ok;
                const bool in = base + lane < GW;
                const float kt = lo_f(r.w[0]), kd = hi_f(r.w[0]);
                const double St = in ? static_cast<double>(lo_f(r.w[1])) : 0.0, Sd = in ? static_cast<double>(hi_f(r.w[1])) : 0.0;
                const float nKt = fmaxf(Kt, wave_max((St > 0.0) ? kt : neg_inf()));
                const float nKd = fmaxf(Kd, wave_max((Sd > 0.0) ? kd : neg_inf()));
                Zt = ((Zt > 0.0) ? ldexp(Zt, kdiff(Kt, nKt)) : Zt) + wave_sum((St > 0.0) ? ldexp(St, kdiff(kt, nKt)) : 0.0);
                Zd = ((Zd > 0.0) ? ldexp(Zd, kdiff(Kd, nKd)) : Zd) + wave_sum((Sd > 0.0) ? ldexp(Sd, kdiff(kd, nKd)) : 0.0);
                Kt = nKt;
                Kd = nKd;
            }
            if (!ok) status |= FSD_ROW_INTERNAL;
            lse2_t = static_cast<double>(Kt) + log2(Zt);
            lse2_d = static_cast<double>(Kd) + log2(Zd);
            if constexpr (MODE == MODE_KLP) {
                if (log_domain && !status) {
                    // the saturated form is a lower bound; the log-domain value replaces it where it is
                    // larger by more than its own rounding can explain
                    const double dl = (lse2_t - lse2_d) * kLn2;
                    const double v = s.hi[0] - dl;
                    if (v == v && v - value > 4e-7 * (fabs(s.hi[0]) + fabs(dl))) value = v;
                }
            }
        }
        if (lane == 0) {
            if (P.want_ratio) status |= write_ratio(pair, lse2_t, lse2_d, status, P.user_ratio);
            P.ws.div[pair] = static_cast<float>(value);
            P.ws.lse2[2 * pair] = lse2_t;
            P.ws.lse2[2 * pair + 1] = lse2_d;
            if (P.user_div) P.user_div[pair] = static_cast<float>(value);
            P.ws.pst[pair] = status;
        }
    };
    auto finish_single_pass = [&](int pair, unsigned long long (&fw)[FW]) __attribute__((always_inline)) {
        const unsigned long long* p1 = part1 + words_at(pair, N1);
        // online merge over rounds of 64 members, float64, exact rescaling between references
        float Kt = neg_inf(), Kd = neg_inf();
        double Zt = 0.0, Zd = 0.0, Wt = 0.0;
        bool ok = true, winf = false;
        for (int base = 0; base < GW; base += 64) {
            unsigned long long w[4];
            if (base == 0) {
#pragma unroll
                for (int k = 0; k < 4; ++k) w[k] = fw[k % FW];
                ok &= await_n<4>(p1, GW, 0, P.spin_limit, w);
            } else {
                const WordsN<4> r = repoll_n<4>(p1, GW, base, P.spin_limit);
                ok &= r.ok;
#pragma unroll
                for (int k = 0; k < 4; ++k) w[k] = r.w[k];
            }
            const bool in = base + lane < GW;
            const float kt = lo_f(w[0]), kd = hi_f(w[0]);
            const double St = in ? bitsd(w[1]) : 0.0, Sd = in ? bitsd(w[2]) : 0.0, W = in ? bitsd(w[3]) : 0.0;
            const float nKt = fmaxf(Kt, wave_max((St > 0.0) ? kt : neg_inf()));
            const float nKd = fmaxf(Kd, wave_max((Sd > 0.0) ? kd : neg_inf()));
            Zt = ((Zt > 0.0) ? ldexp(Zt, kdiff(Kt, nKt)) : Zt) +
                 wave_sum((St > 0.0) ? ldexp(St, kdiff(kt, nKt)) : (St != St ? St : 0.0));
            Zd = ((Zd > 0.0) ? ldexp(Zd, kdiff(Kd, nKd)) : Zd) +
                 wave_sum((Sd > 0.0) ? ldexp(Sd, kdiff(kd, nKd)) : (Sd != Sd ? Sd : 0.0));
            if constexpr (MODE == MODE_KL) {
                winf |= __any(in && W == __builtin_inf()) != 0;
                Wt = ((Kt > neg_inf()) ? ldexp(Wt, kdiff(Kt, nKt)) : Wt) +
                     wave_sum((St > 0.0 && W == W && W != __builtin_inf()) ? ldexp(W, kdiff(kt, nKt)) : 0.0);
            }
            Kt = nKt;
            Kd = nKd;
        }
        int status = 0;
        const bool bad = !(Zt > 0.0) || !(Zd > 0.0) || !(Zt < __builtin_inf()) || !(Zd < __builtin_inf()) ||
                         !(Kt < __builtin_inff()) || !(Kd < __builtin_inff());
        if (bad) status |= FSD_ROW_NONFINITE;
        if (!ok) status |= FSD_ROW_INTERNAL;
        const double lse2_t = static_cast<double>(Kt) + log2(Zt), lse2_d = static_cast<double>(Kd) + log2(Zd);
        double value = 0.0;
        if constexpr (MODE == MODE_KL) {
            // KL = sum_v p_v (a_v - b_v) - (lse_t - lse_d), p_v = 2^(a log2e - Kt) / Zt
            value = winf ? __builtin_inf() : Wt / Zt - (lse2_t - lse2_d) * kLn2;
        }
        if (value < 0.0) value = 0.0;
        if (status) value = __builtin_nan("");
        if (lane == 0) {
            P.ws.div[pair] = static_cast<float>(value);
            P.ws.lse2[2 * pair] = lse2_t;
            P.ws.lse2[2 * pair + 1] = lse2_d;
            if (P.user_div) P.user_div[pair] = static_cast<float>(value);
            if constexpr (MODE == MODE_LSE) {
                status |= write_ratio(pair, lse2_t, lse2_d, status, P.user_div);
            } else {
                if (P.want_ratio) status |= write_ratio(pair, lse2_t, lse2_d, status, P.user_ratio);
            }
            P.ws.pst[pair] = status;
        }
    };
    auto finish_jse = [&](int pair, unsigned long long (&fw)[FW]) __attribute__((always_inline)) {
        const unsigned long long* p2 = part2 + words_at(pair, 1);
        unsigned long long f[1] = {fw[0]};
        bool ok = await_n<1>(p2, GW, 0, P.spin_limit, f);
        double sum = wave_sum((lane < GW) ? __longlong_as_double(static_cast<long long>(f[0])) : 0.0);
        if (GW > 64) {
            const SumMore m = sum_f64_more_rounds(p2, GW, P.spin_limit, sum);
            sum = m.sum;
            ok &= m.ok;
        }
        double value = 0.5 * kLn2 * sum;
        int status = ok ? 0 : FSD_ROW_INTERNAL;
        unsigned long long state = kJsDone;
        // below the floor (cancellation), or anything but a plain number (unusable rows, or sums the
        // masked entries of usable rows have spoilt): the pointwise form decides, if the rows are usable
        // (the floor is read where it is used: as a double kept across the loop it would be spilled)
        float floor_here = P.js_floor;
        asm volatile("" : "+v"(floor_here));
        if (ok && (!(value >= static_cast<double>(floor_here)) || !(value < 1.0))) {
            asm volatile("");   // stays a branch
            const RowNorms n = row_norms(part1 + words_at(pair, N1), GW, P.spin_limit);
            if (!n.ok) status |= FSD_ROW_INTERNAL;
            else if (!n.usable) status |= FSD_ROW_NONFINITE;
            else state = pack2(static_cast<float>(n.lse2_t), static_cast<float>(n.lse2_d));
        }
        if (value < 0.0) value = 0.0;
        if (status) value = __builtin_nan("");
        if (lane == 0) {
            double zero = 0.0;   // (made here, for the same reason)
            asm volatile("" : "+v"(zero));
            P.ws.lse2[2 * pair] = zero;
            P.ws.lse2[2 * pair + 1] = zero;
            if (state == kJsDone) {
                P.ws.div[pair] = static_cast<float>(value);
                if (P.user_div) P.user_div[pair] = static_cast<float>(value);
                P.ws.pst[pair] = status;
                if (status & FSD_ROW_INTERNAL) flag_failure(P.ws);
            }
            // the word every member of the team looks at before it leaves
            post64(P.ws.state + pair, state);
        }
    };
    auto finish = [&](int pair, unsigned long long (&fw)[FW]) __attribute__((always_inline)) {
        if constexpr (JSE) finish_jse(pair, fw);
        else if constexpr (TWO_PHASE) finish_two_phase(pair, fw);
        else finish_single_pass(pair, fw);
    };

    // ---- state of the previous pair, whose phase 2 is still to come (two-phase modes)
    // wsum, dmax: pointwise KL; entropy-form JS: this lane's A_t + S_t and A_d, and sd is this lane's S_d
    struct Pend { int pair; float kt, kd; bool mass_t, mass_d, mask; float wsum, dmax, st, sd; };
    Pend pend[LAG];   // [0] the last step's pair ... [LAG-1] the one whose phase 2 is due
#pragma unroll
    for (int i = 0; i < LAG; ++i) pend[i] = Pend{-1, 0.0f, 0.0f, false, false, false, 0.0f, 0.0f, 0.0f, 0.0f};
    bool js_clamp2 = false;   // entropy-form JS: phase 2 keeps u above the smallest normal number (see phase2)
    // pairs this wavefront has to finish: fin[0] now, fin[i] i steps from now.  A two-phase pair
    // is finished NF steps after its phase 1.  Whoever starts step n has merged the team words of
    // step n - 1, so every member has ended step n - 2 - LAG and with it phase 2 of the pair of step
    // n - 2 - 2 LAG: the finisher's words are there when it asks, however far the team has spread.
    constexpr int NF = TWO_PHASE ? 2 * LAG + 2 : 1;
    int fin[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) fin[i] = -1;
    int iter = 0;

    // the previous pair's row-wide normalisers from the team's words (w holds the first 64 members'):
    // factors ft, fd with p = e_t ft, q = e_d fd
    auto merge_team = [&](const Pend& pp, unsigned long long (&w)[2], unsigned long long (&w2)[2], float& ft, float& fd) __attribute__((always_inline)) -> bool {
        const unsigned long long* p1 = part1 + words_at(pp.pair, N1);
        // binary32 is enough: the normalisers enter p and q as common factors
        TeamNorm n{pp.kt, pp.kd, 0.0f, 0.0f, true};
        n.ok = await_n<2>(p1, GW, 0, P.spin_limit, w);
        if (GW > 64) {
            // members 64..127 were requested with the first 64: a lane adds its two members before the
            // one reduction over the wavefront; larger teams ask for the rest afterwards
            if (!await_n<2>(p1, GW, 64, P.spin_limit, w2)) n.ok = false;
            float at, ad, at2, ad2;
            member_terms(w, lane < GW, n, at, ad);
            member_terms(w2, 64 + lane < GW, n, at2, ad2);
            at += at2;
            ad += ad2;
            wave_sumf2(at, ad);
            n.zt += at;
            n.zd += ad;
            if (GW > 128) n = merge_more_rounds(p1, GW, P.spin_limit, n);
        } else {
            merge_round(w, lane < GW, n);
        }
        const bool ok = n.ok;
        // the row's sum relative to this wavefront's own reference exponent: p = e / sum.  The
        // hardware reciprocal (1 ulp) is as good as a division here: the factor is common to a row.
        // inf for a row without mass, NaN for a bad one
        const float rzt = __builtin_amdgcn_rcpf(n.zt), rzd = __builtin_amdgcn_rcpf(n.zd);
        // A wavefront without mass has only zeros in e; its factor is 0 (NaN if the row is unusable).
        ft = pp.mass_t ? rzt : rzt * 0.0f;
        fd = pp.mass_d ? rzd : rzd * 0.0f;
        return ok;
    };

    // phase 2 of the previous pair from its kept exponentials
    auto phase2 = [&](const Pend& pp, auto S, float ft, float fd, bool ok) __attribute__((always_inline)) {
        // Only relative errors enter p and q, and the divergences below are functions of (p, q)
        // alone, second order in r = (p - q)/(p + q): the result is the divergence of a slightly
        // perturbed input.  u = 1 + r = 2p/s and v = 2 - u = 2q/s (exact subtraction).
        //
        // JS and TV are homogeneous of degree one in (p, q) and bounded, so only one side is scaled entry by
        // entry: with c = fd/ft the pair (e_t, e_d c) = (p, q)/ft, and the wavefront's sum takes the
        // factor ft once.  Factors below 2^-80 (a wavefront whose share of the row is that small) are
        // raised to it, which moves the result by less than 1e-20; equal factors give c = 1 exactly,
        // so equal rows still give p == q entry by entry.  The exponentials are zero or normal numbers
        // (the hardware exponential flushes), hence so is a positive p - q and its p + q.
        const float ftc = fmaxf(ft, 0x1p-80f), fdc = fmaxf(fd, 0x1p-80f);   // max() drops NaN: see below
        const float cq = (ftc == fdc) ? 1.0f : fdc * __builtin_amdgcn_rcpf(ftc);
        unsigned long long word[PW];
        if constexpr (JSE) {
            // U = sum u log2 u with u = e_t + c e_d = (p + q)/ft
            float acc = 0.0f;
            if (!js_clamp2) {
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    float t4[4], d4[4];
                    get4(S, c, t4, d4);
                    // (the four logarithms first: a logarithm's result cannot be used by the very next instruction)
                    float u[4], l[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) u[i] = fmaf(d4[i], cq, t4[i]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) l[i] = hw_log2(u[i]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc = fmaf(u[i], l[i], acc);
                }
                // an entry without mass in either row (both exponentials flushed to zero, or masked) gives
                // 0 log 0 = NaN: from then on this wavefront keeps u above the smallest normal number, whose
                // term is nothing, at one more instruction per entry (the kept exponentials are still there,
                // so this pair is done again right away)
                if (__any(acc != acc)) js_clamp2 = true;
            }
            if (js_clamp2) {
                acc = 0.0f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    float t4[4], d4[4];
                    get4(S, c, t4, d4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float u = fmaxf(fmaf(d4[i], cq, t4[i]), 0x1p-126f);
                        acc = fmaf(u, hw_log2(u), acc);
                    }
                }
            }
            // the member's share C = f_t [A_t + c A_d - U + W + c S_d log2 c] with W = S_t + c S_d.  Every sum
            // in it runs over the same entries, so a lane forms its own part first, from its own sums
            // (pp.wsum = A_t + S_t, pp.dmax = A_d, pp.sd = S_d of this lane), and one reduction over the
            // wavefront follows: a lane's part is its entries' pointwise terms, small and not negative up to
            // rounding, where the separate sums are large and cancel.  1 + log2 c = exponent + (1 + log2 of
            // the mantissa in [1/2, 1)); c = 1 gives exactly 1.
            const float g = static_cast<float>(__builtin_amdgcn_frexp_expf(cq)) + (1.0f + hw_log2(__builtin_amdgcn_frexp_mantf(cq)));
            const float part = fmaf(cq, fmaf(pp.sd, g, pp.dmax), pp.wsum) - acc;
            double share = static_cast<double>(wave_sumf(part)) * static_cast<double>(ftc);
            if (ft != ft || fd != fd) share = static_cast<double>(ft + fd);   // an unusable row stays NaN (max() drops it above)
            if (!ok) share = __builtin_nan("");
            word[0] = dbits(share);
        } else if constexpr (MODE == MODE_TV) {
            float A = 0.0f, Bn = 0.0f, MA = 0.0f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                float t4[4], d4[4];
                get4(S, c, t4, d4);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = t4[i], q = d4[i] * cq;
                    const float d = p - q, sum = p + q;
                    A += fmaxf(d, 0.0f);
                    Bn += fmaxf(-d, 0.0f);
                    MA += (d > 0.0f) ? sum : 0.0f;   // the other side's mass is what is left of 2
                }
            }
            // max() drops NaN: an unusable row (NaN factor) is made to reach the side selection
            wave_sumf2(A, Bn);
            MA = wave_sumf(MA);
            A *= ftc; Bn *= ftc; MA *= ftc;
            if (ft != ft || fd != fd) { A = ft + fd; Bn = A; MA = A; }
            if (!ok) { A = __builtin_nanf(""); MA = A; }
            word[0] = pack2(A, Bn);
            word[1] = pack2(MA, 0.0f);
        } else {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
              float t4[4], d4[4];
              get4(S, c, t4, d4);
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                // KL is not bounded: where q/p leaves binary32's range its terms saturate (ln of the range),
                // and raised factors would lower that point from 87 to 55; it keeps both factors, and a
                // floor under p and q instead
                const float p = (MODE == MODE_KLP) ? fmaf(t4[i], ft, kTiny) : t4[i];
                const float q = (MODE == MODE_KLP) ? fmaf(d4[i], fd, kTiny) : d4[i] * cq;
                const float d = p - q, sum = p + q;
                // (JS) p = q = 0: 0 * inf = NaN, which max() drops (u = kTiny, v = 2, both weights zero)
                const float inv = __builtin_amdgcn_rcpf(sum);
                float u = fmaxf(fmaf(d, inv, 1.0f), kTiny), v = fmaxf(2.0f - u, kTiny);
                if constexpr (MODE == MODE_KLP) {
                    // u = 1 + r and v = 2 - u carry an absolute error of 2^-23: harmless for JS, where a
                    // small u or v comes with a small weight, but KL weighs ln(u/v) with the larger of the
                    // two.  Far from p = q the smaller one is taken from its own quotient instead (a
                    // relative error); near p = q the exact complement is what keeps the first-order
                    // terms cancelling.
                    const float inv2 = inv + inv;
                    if (u < 0.5f) u = fmaxf(p * inv2, kTiny);
                    if (v < 0.5f) v = fmaxf(q * inv2, kTiny);
                }
                if constexpr (MODE == MODE_JS) {
                    // p ln(2p/s) + q ln(2q/s) = ln2 (p log2 u + q log2 v); the rounding of u = 1 + r
                    // cancels between the two terms because p/u = q/v
                    acc = fmaf(p, hw_log2(u), acc);
                    acc = fmaf(q, hw_log2(v), acc);
                } else {
                    // p ln(p/q) + q - p = (s/2) [u ln(u/v) + v - u] >= 0 entry by entry (the added q - p
                    // sums to zero).  Written in (u, v) only, the rounding of u cancels between the
                    // two parts; p ln(u/v) - (p - q) would keep it to first order.
                    acc = fmaf(sum, fmaf(u, hw_log2(u) - hw_log2(v), (v - u) * kLog2e), acc);
                }
              }
            }
            acc = wave_sumf(acc);
            if constexpr (MODE != MODE_KLP) acc *= ftc;
            if (ft != ft || fd != fd) acc = ft + fd;   // an unusable row stays NaN
            if constexpr (MODE == MODE_KLP) {
                if (__any(pp.mask)) acc += __builtin_inff();   // draft masks an entry the target keeps; NaN stays NaN
            }
            if (!ok) acc = __builtin_nanf("");
            if constexpr (MODE == MODE_KLP) {
                // Where q/p leaves binary32's range the terms above saturate.  Beside them goes this
                // wavefront's share of sum p (a - b), from which the finisher can form the log-domain
                // value sum p (a - b) - (lse_t - lse_d), and a mark that says it should look: an entry
                // whose ln(p/q) = (a - b) - (lse_t - lse_d) passes 80 (or a draft side without any mass
                // here).  log2 f = k - lse2 for both factors.  (The entry may carry no weight; the
                // finisher compares the two values.)
                const float dl = ((pp.kt - hw_log2(ft)) - (pp.kd - hw_log2(fd))) * static_cast<float>(kLn2);
                const bool sat = (ft > 0.0f) && pp.dmax > neg_inf() && (fd == 0.0f || pp.dmax - dl > 80.0f);
                word[0] = pack2(acc, pp.wsum * ft);
                word[1] = pack2(sat ? 1.0f : 0.0f, 0.0f);
            } else {
                word[0] = pack2(acc, 0.0f);
            }
        }
        if (!ok && lane == 0) flag_failure(P.ws);
        if (lane < PW) {
            unsigned long long mine = word[0];
#pragma unroll
            for (int k = 1; k < PW; ++k) mine = (lane == k) ? word[k] : mine;
            // the lane's offset is recomputed here (hidden from loop-invariant hoisting): kept across
            // the loop it would be spilled, and the reload would wait for every load in flight
            int l = lane;
            asm volatile("" : "+v"(l));
            post64(word_at(part2 + words_at(pp.pair, PW), static_cast<unsigned>(member * PW + l)), mine);
        }
    };

    auto finish_now = [&](int pair) __attribute__((always_inline)) {
        unsigned long long fw[FW];
        request_n<FW>(finw + words_at(pair, FW), GW, 0, fw);
        finish(pair, fw);
    };
    // Single-pass modes: nothing makes the members of a team wait for each other, so they drift
    // apart, and a finisher that looked for the words one step after its own post would wait for
    // the slowest member (measured: a third of the kernel's time was this tail).  The finisher of
    // a pair therefore looks kSpDelay steps later, or after its last step, whichever comes first:
    // by then the words are there, and what little waiting is left falls where the kernel has to
    // wait for its slowest wavefront anyway.  A member is named every GW steps, so one pending
    // pair is all there is to remember.
    const int sp_delay = (GW - 1 < 16) ? GW - 1 : 16;
    int sp_pair = -1, sp_due = 0;

    // One step: phase 1 of `pair` into (ect, ecd), then phase 2 of the previous pair from (ept, epd).
    // Memory operations return in the order they were issued, so the order of the requests decides
    // what can overlap: the small exchange words (the previous pair's team words, and the words of a
    // pair this wavefront has to finish) are requested first, at the top of the step, where they sit
    // behind the logits that are about to be used anyway; the logits of the next pair are requested
    // once phase 1 has consumed the registers (in the two-phase modes after this wavefront's sums are
    // posted: the team's next step waits for every member's post, so nothing that can wait comes
    // before it); and nothing after that waits on memory unless a team member is late (then the
    // words are asked for again, behind the prefetch).
    // (ra, rb) hold the logits of `pair`, the next pair's go to (rna, rnb).  Where registers allow
    // (DEEP) these are different sets and the next pair is requested at the top of the step, a whole
    // step ahead; otherwise both names are the same set and the request follows phase 1.
    // SC names the set that takes this pair's exponentials, SP the one written LAG steps ago.
    auto step = [&](auto SC, auto SP, uint4 (&ra)[NV], uint4 (&rb)[NV], uint4 (&rna)[NV], uint4 (&rnb)[NV], int pair)
                    __attribute__((always_inline)) {
        unsigned long long w[2] = {1, 1}, w2[2] = {1, 1};
        unsigned long long fw[FW];
        const int fpair = TWO_PHASE ? fin[0] : ((sp_pair >= 0 && iter >= sp_due) ? sp_pair : -1);
        const Pend due = pend[LAG - 1];
        // Phase 1 and the post of this wavefront's sums are what the whole team waits for: they run at
        // raised priority (and the request for the next pair's logits right behind them); what follows
        // overlaps with the memory latency and does not need it.
        __builtin_amdgcn_s_setprio(3);
        asm volatile("" ::: "memory");
        if constexpr (TWO_PHASE)
        {
            const unsigned long long* const p1 = part1 + words_at(due.pair >= 0 ? due.pair : pair, N1);
            request_n<2>(p1, GW, 0, w);
            request_n<2>(p1, GW, 64, w2, GW > 64);
        }
        request_n<FW>(finw + words_at(fpair >= 0 ? fpair : pair, FW), GW, 0, fw, fpair >= 0);
        if constexpr (DEEP) {
            // this pair's logits arrived in (ra, rb) during the last step; ask for the next pair's now
            const bool more = pair + pstep < pair_end;
            load_item(rna, rnb, more ? pair + pstep : pair, more);
        }
        asm volatile("" ::: "memory");
        fill_unowned(ra, rb);
        // ---- phase 1: maximum, then sums of 2^(z log2e - k) with k = ceil(max log2e)
        // SHARE (entropy-form JS on a tree): the children of a node come one after the other and share their
        // target row.  A pair whose target row is the previous pair's takes that row's exponentials from
        // the previous step's set, and its reference exponent and sums from that step's record: half of
        // phase 1 is not computed again (the loads are still made: they hit the cache, and a request that
        // is only made sometimes would make the count of requests in flight inexact).
        tp_prev = tp_cur;
        tp_cur = tp_next;
        const bool same_target = SHARE && iter > 0 && tp_cur == tp_prev;
        float kt, kd, st = 0.0f, sd = 0.0f, wacc = 0.0f, dmax = JSE ? 0.0f : neg_inf();
        auto phase1 = [&](auto SAME_T) __attribute__((always_inline)) {
            constexpr bool SAME = decltype(SAME_T)::value;
            float mt = neg_inf(), md = neg_inf();
            if constexpr (BF16) {
                // A 32-bit word holds two bfloat16 logits.  Read as binary32 it is its upper logit plus a
                // perturbation below that logit's last place, so the maximum over the words as they are has
                // the largest upper logit in its upper half: only the lower logits need a shift.  (A word
                // whose upper logit is +-inf or NaN reads as NaN and is dropped: a masked entry is never
                // the maximum, and the exponential pass still sees the +inf or NaN that spoils a row.)
                float th = neg_inf(), tl = neg_inf(), dh = neg_inf(), dl = neg_inf();
#pragma unroll
                for (int k = 0; k < NV; ++k) {
                    if constexpr (!SAME) {
                        th = fmaxf(fmaxf(th, __uint_as_float(ra[k].x)), __uint_as_float(ra[k].y));
                        th = fmaxf(fmaxf(th, __uint_as_float(ra[k].z)), __uint_as_float(ra[k].w));
                        tl = fmaxf(fmaxf(tl, __uint_as_float(ra[k].x << 16)), __uint_as_float(ra[k].y << 16));
                        tl = fmaxf(fmaxf(tl, __uint_as_float(ra[k].z << 16)), __uint_as_float(ra[k].w << 16));
                    }
                    dh = fmaxf(fmaxf(dh, __uint_as_float(rb[k].x)), __uint_as_float(rb[k].y));
                    dh = fmaxf(fmaxf(dh, __uint_as_float(rb[k].z)), __uint_as_float(rb[k].w));
                    dl = fmaxf(fmaxf(dl, __uint_as_float(rb[k].x << 16)), __uint_as_float(rb[k].y << 16));
                    dl = fmaxf(fmaxf(dl, __uint_as_float(rb[k].z << 16)), __uint_as_float(rb[k].w << 16));
                }
                if constexpr (!SAME) mt = fmaxf(__uint_as_float(__float_as_uint(th) & 0xFFFF0000u), tl);
                md = fmaxf(__uint_as_float(__float_as_uint(dh) & 0xFFFF0000u), dl);
            } else {
#pragma unroll
                for (int k = 0; k < NV; ++k) {
                    float a[VE], c[VE];
                    if constexpr (!SAME) unpack<BF16>(ra[k], a);
                    unpack<BF16>(rb[k], c);
#pragma unroll
                    for (int e = 0; e < VE; e += 2) {
                        if constexpr (!SAME) mt = fmaxf(fmaxf(mt, a[e]), a[e + 1]);
                        md = fmaxf(fmaxf(md, c[e]), c[e + 1]);
                    }
                }
            }
            PT(0);   // load wait + max pass
            if constexpr (SAME) md = wave_max(md); else wave_max2(mt, md);
            kt = SAME ? due.kt : ((mt == neg_inf()) ? 0.0f : ceilf(mt * kLog2e));
            kd = (md == neg_inf()) ? 0.0f : ceilf(md * kLog2e);
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                float a[VE], c[VE];
                if constexpr (!SAME) unpack<BF16>(ra[k], a);
                unpack<BF16>(rb[k], c);
                float xa_[VE], xb_[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    const float yb = fmaf(c[e], kLog2e, -kd);
                    const float xb = hw_exp2(yb);
                    xb_[e] = xb;
                    sd += xb;
                    float ya = 0.0f, xa = 0.0f;
                    if constexpr (!SAME) {
                        ya = fmaf(a[e], kLog2e, -kt);
                        xa = hw_exp2(ya);
                        xa_[e] = xa;
                        st += xa;
                    }
                    if constexpr (JSE) {   // the entropies' sums of e x (wacc: target, dmax: draft)
                        if constexpr (!SAME) wacc = fmaf(xa, ya, wacc);
                        dmax = fmaf(xb, yb, dmax);
                    }
                    if constexpr (MODE == MODE_KL || MODE == MODE_KLP) {
                        const float diff = a[e] - c[e];
                        dmax = fmaxf(dmax, diff);   // +inf iff the draft masks an entry the target does not
                        if constexpr (MODE == MODE_KL) {
                            wacc = fmaf(xa, fminf(fmaxf(diff, -FLT_MAX), FLT_MAX), wacc);
                        } else {
                            // only used where the pointwise terms saturate, and checked there: the median
                            // instruction clamps in one operation (a NaN difference, -inf on both sides,
                            // has the weight 0 either way)
                            wacc = fmaf(xa, __builtin_amdgcn_fmed3f(diff, -FLT_MAX, FLT_MAX), wacc);
                        }
                    }
                }
                if constexpr (TWO_PHASE) {
#pragma unroll
                    for (int h = 0; h < VE / 4; ++h) {
                        float t4[4], d4[4];
                        if constexpr (SAME) {
                            get4(SP, k * (VE / 4) + h, t4, d4);   // the previous pair's target exponentials
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i) t4[i] = xa_[4 * h + i];
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) d4[i] = xb_[4 * h + i];
                        put4(SC, k * (VE / 4) + h, t4, d4);
                    }
                }
            }
        };
        if constexpr (SHARE) {
            if (same_target) {
                asm volatile("");
                phase1(BoolTag<true>{});
            } else {
                phase1(BoolTag<false>{});
            }
        } else {
            phase1(BoolTag<false>{});
        }
        if constexpr (JSE) {
            // A -inf logit is legal (a masked entry) and has the exponential 0, but its 0 * x is NaN: the sums
            // of e x are then formed once more from the kept exponentials, as e log2 e with 0 log 0 = 0 (the
            // logits' registers are free by now; the hardware logarithm of e is x to 1e-7)
            if (__any((wacc != wacc) || (dmax != dmax))) {
                asm volatile("");   // keeps this a branch (as straight-line code with selections it would run every step)
                wacc = 0.0f;
                dmax = 0.0f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    float t4[4], d4[4];
                    get4(SC, c, t4, d4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        wacc = fmaf(t4[i], hw_log2((t4[i] == 0.0f) ? 1.0f : t4[i]), wacc);   // NaN stays NaN
                        dmax = fmaf(d4[i], hw_log2((d4[i] == 0.0f) ? 1.0f : d4[i]), dmax);
                    }
                }
            }
        }
        PT(1);   // reductions + exp pass
        asm volatile("" ::: "memory");
        // ---- the registers that held the logits are free: fetch the next pair (the request is
        // unconditional: the last step asks for one slot of its own pair, which the caches hold).  In the
        // two-phase modes only after the post below: every member's post is what the whole team's next
        // step waits for (bfloat16 JS: C2 -2 %, C4 -4 % against the request first).
        if constexpr (!DEEP && !TWO_PHASE) {
            const bool more = pair + pstep < pair_end;
            load_item(rna, rnb, more ? pair + pstep : pair, more);
            __builtin_amdgcn_s_setprio(0);
        }
        asm volatile("" ::: "memory");
        // ---- post this wavefront's partial.  The two-phase modes need the normalisers to a relative
        // 1e-7 only (common factors of p and q); the single-pass modes take them through a logarithm.
        const unsigned long long w0 = pack2(kt, kd);
        unsigned long long mine;
        [[maybe_unused]] const float st_lane = st, sd_lane = sd;
        if constexpr (TWO_PHASE) {
            wave_sumf2(st, sd);
            if constexpr (MODE == MODE_KLP) { wacc = wave_sumf(wacc); dmax = wave_max(dmax); }
            if constexpr (SHARE) {
                if (same_target) st = due.st;   // the target row's sum, as the previous step formed it
            }
            mine = (lane == 0) ? w0 : pack2(st, sd);
        } else {
            const double pst_ = wave_sum(static_cast<double>(st));
            const double psd_ = wave_sum(static_cast<double>(sd));
            double pw_ = 0.0;
            if constexpr (MODE == MODE_KL) {
                pw_ = wave_sum(static_cast<double>(wacc));
                if (wave_max(dmax) == __builtin_inff()) pw_ = __builtin_inf();
            }
            mine = (lane == 0) ? w0 : (lane == 1) ? dbits(pst_) : (lane == 2) ? dbits(psd_) : dbits(pw_);
        }
        // (the lane's word is addressed by a 32-bit offset from the pair's scalar pointer, formed here)
        int pl = lane;
        asm volatile("" : "+v"(pl));
        unsigned long long* const post_at = word_at(part1 + words_at(pair, N1), static_cast<unsigned>(member * N1 + (pl & 3)));
        if (pl < N1) post64(post_at, mine);
        asm volatile("" ::: "memory");
        if constexpr (TWO_PHASE) {
            if constexpr (!DEEP) {
                const bool more = pair + pstep < pair_end;
                load_item(rna, rnb, more ? pair + pstep : pair, more);
            }
            __builtin_amdgcn_s_setprio(0);   // only now does the priority drop
        }
        asm volatile("" ::: "memory");
        if constexpr (JSE) wacc += st_lane;   // the lane's A_t + S_t (phase 2 of a later step combines the lanes' sums)
        if constexpr (SHARE) {
            if (same_target) wacc = due.wsum;
        }
        PT(3);   // wave sums, prefetch issue, post
        if constexpr (TWO_PHASE) {
            // ---- the previous pair's normalisers, then its phase 2
            float ft = 0.0f, fd = 0.0f;
            bool ok2 = false;
            if (due.pair >= 0) ok2 = merge_team(due, w, w2, ft, fd);
            PT(2);   // team merge (wait for the team's words)
            if (due.pair >= 0) phase2(due, SP, ft, fd, ok2);
            PT(4);   // phase 2
            // the posted value and its address stay in their registers until here: reusing them
            // earlier would make phase 2 wait for the store, and with it for the prefetch
            asm volatile("" ::"v"(mine), "v"(post_at));
#pragma unroll
            for (int i = LAG - 1; i > 0; --i) pend[i] = pend[i - 1];
            pend[0] = Pend{pair, kt, kd, (st > 0.0f) || (st != st), (sd > 0.0f) || (sd != sd), dmax == __builtin_inff(), wacc, dmax, st, JSE ? sd_lane : sd};
        }
        // ---- finishing duties: the pair whose turn has come, then note this pair if it is ours
        if (fpair >= 0) finish(fpair, fw);
        if constexpr (TWO_PHASE) {
#pragma unroll
            for (int i = 0; i + 1 < NF; ++i) fin[i] = fin[i + 1];
            fin[NF - 1] = (iter % GW == member) ? pair : -1;   // the members take turns
        } else {
            if (fpair >= 0) sp_pair = -1;
            if (iter % GW == member) { sp_pair = pair; sp_due = iter + sp_delay; }
        }
        PT(5);   // finishing duty
        if (iter == 0 && P.self_clear) {
            // A call without a clearing kernel: nothing of the team's has been read so far; from the next
            // step on it is, so every member must have cleared its words by now.  (Not at the start of the
            // kernel: the workgroups of a team start microseconds apart, and this step's work is what
            // absorbs that.)
            asm volatile("");   // stays a branch
            if (!team_arrived(P.ws.arrive + team * GW, GW, P.ws.nonce, P.spin_limit)) flag_failure(P.ws);
        }
        ++iter;
    };

    // DEEP: three sets of logit registers that rotate with the three sets of exponentials (two are in
    // use at any time; the third saves copying 64 registers a step)
    static_assert(!DEEP || NB == 3, "the logit sets rotate with the sets of exponentials");
    constexpr int NR = DEEP ? 3 : 1;
    uint4 rta[NR][NV], rtb[NR][NV];
    int pair = pair0;
    if (P.self_clear) {
        const int n_mine = (pair_end > pair0) ? (pair_end - pair0 + pstep - 1) / pstep : 0;
        clear_own_words<N1, PW, TWO_PHASE, JSE>(part1, part2, P.ws.state, P.clear_a, P.clear_a16, P.clear_b, P.clear_b16,
                                                gwave, nteams * GW, member, GW, pair0, pstep, n_mine);
    }
    // (a team without pairs, which a tree's last teams can be, posts nothing and nobody waits for it)
    if (pair >= pair_end) return;
    asm volatile("" ::: "memory");
    load_item(rta[0], rtb[0], pair);
    {
        // The first pair's logits are requested before the clearing stores are waited for.  Vector memory
        // operations complete in the order they were issued, so once all but the 2 NV requests above have
        // completed the stores have been performed (the exchange words are cleared with the device-scope
        // stores they are always written with, which are performed at the memory side: no write-back of
        // the cache is needed, and a release fence here would write back all of it from every wavefront,
        // +25 us at C2; the sampler's words are cleared with ordinary stores, which the end of the kernel
        // publishes).  Then lane 0 announces the wavefront.
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NV) : "memory");
        if (P.self_clear && lane == 0) post64(P.ws.arrive + gwave, P.ws.nonce);
        asm volatile("" ::: "memory");
    }
    auto one_step = [&](auto SC, auto SP, int pr) __attribute__((always_inline)) {
        constexpr int c = decltype(SC)::value % NR, n = (decltype(SC)::value + 1) % NR;
        step(SC, SP, rta[c], rtb[c], rta[n], rtb[n], pr);
    };
    if constexpr (TWO_PHASE) {
        // step i keeps its exponentials in set i % NB and reads the set written LAG steps earlier
        bool live = pair < pair_end;
        while (live) {
            one_step(SetId<0>{}, SetId<1 % NB>{}, pair);
            pair += pstep;
            live = pair < pair_end;
            if (live) {
                one_step(SetId<1>{}, SetId<2 % NB>{}, pair);
                pair += pstep;
                live = pair < pair_end;
            }
            if constexpr (NB == 3) {
                if (live) {
                    one_step(SetId<2>{}, SetId<0>{}, pair);
                    pair += pstep;
                    live = pair < pair_end;
                }
            }
        }
        // ---- drain: phase 2 of the pairs still pending, oldest first, then the finishes still owed
#pragma unroll
        for (int d = LAG; d >= 1; --d) {
            const Pend pp = pend[d - 1];
            if (pp.pair >= 0) {
                unsigned long long w[2], w2[2];
                float ft, fd;
                request_n<2>(part1 + words_at(pp.pair, N1), GW, 0, w);
                request_n<2>(part1 + words_at(pp.pair, N1), GW, 64, w2, GW > 64);
                const bool ok2 = merge_team(pp, w, w2, ft, fd);
                const int b = (iter + NB - d) % NB;   // written at step iter - d
                if (b == 0) phase2(pp, SetId<0>{}, ft, fd, ok2);
                else if (b == 1) phase2(pp, SetId<1>{}, ft, fd, ok2);
                else phase2(pp, SetId<NB - 1>{}, ft, fd, ok2);
            }
        }
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            if (fin[i] >= 0) finish_now(fin[i]);
        }
    } else {
        for (; pair < pair_end; pair += pstep) one_step(SetId<0>{}, SetId<1>{}, pair);
        if (sp_pair >= 0) finish_now(sp_pair);
    }
    PT(6);   // drain
    if constexpr (JSE) {
        // ---- the team's pairs whose entropy-form result was below the floor, once more in the pointwise
        // form.  Every member walks the team's pairs in the same order and waits (bounded) for each pair's
        // state word; member (index mod GW) adds the team's partial sums in member order.
        const int n_mine = (pair_end > pair0) ? (pair_end - pair0 + pstep - 1) / pstep : 0;
        for (int base = 0; base < n_mine; base += 64) {
            const int idx = base + lane;
            const bool valid = idx < n_mine;
            const unsigned long long* sp = P.ws.state + (valid ? pair0 + idx * pstep : pair0);
            unsigned long long sw = read64(sp);
            unsigned polls = 0;
            while (__any(valid && sw == 0)) {
                if (polls++ >= P.spin_limit) break;
                __builtin_amdgcn_s_sleep(2);
                sw = read64(sp);
            }
            if (__any(valid && sw == 0)) {
                if (lane == 0) flag_failure(P.ws);   // a finisher never came: the call reports it
            }
            unsigned long long todo = __ballot(valid && sw != 0 && sw != kJsDone);
            while (todo) {
                const int i = __builtin_ctzll(todo);
                todo &= todo - 1;
                const int rp = pair0 + (base + i) * pstep;
                const unsigned lo = __builtin_amdgcn_readlane(static_cast<unsigned>(sw), i);
                const unsigned hi = __builtin_amdgcn_readlane(static_cast<unsigned>(sw >> 32), i);
                const char *tptr, *dptr;
                row_ptrs(rp, tptr, dptr);
                const float part = js_pointwise_slice<NV, ALIGNED>(tptr, dptr, P.V, sl0, sl_end, sl_last, __uint_as_float(lo),
                                                                   __uint_as_float(hi));
                // the partial replaces this member's sums of exponentials, which nobody reads any more once the
                // pair's state word is out (a sum is never -1)
                unsigned long long* const p2 = part1 + words_at(rp, N1) + 1;
                if (lane == 0) post64(p2 + member * N1, pack2(part, -1.0f));
                if ((base + i) % GW == member) {
                    double sum = 0.0;
                    bool ok = true;
                    for (int mb = 0; mb < GW; mb += 64) {
                        const int m = mb + lane;
                        const bool in = m < GW;
                        const unsigned long long* wp = p2 + (in ? m : GW - 1) * N1;
                        unsigned long long v = read64(wp);
                        unsigned tries = 0;
                        while (__any(hi_f(v) != -1.0f)) {
                            if (tries++ >= P.spin_limit) { ok = false; break; }
                            __builtin_amdgcn_s_sleep(2);
                            v = read64(wp);
                        }
                        sum += wave_sum(in ? static_cast<double>(lo_f(v)) : 0.0);
                    }
                    double value = 0.5 * kLn2 * sum;
                    int status = 0;
                    if (value != value) status |= FSD_ROW_NONFINITE;
                    if (!ok) status |= FSD_ROW_INTERNAL;
                    if (value < 0.0) value = 0.0;
                    if (status) value = __builtin_nan("");
                    if (lane == 0) {
                        P.ws.div[rp] = static_cast<float>(value);
                        if (P.user_div) P.user_div[rp] = static_cast<float>(value);
                        P.ws.pst[rp] = status;
                        if (!ok) flag_failure(P.ws);
                    }
                }
            }
        }
    }
#ifdef FSD_PHASE_TIMING
    PT(7);   // second evaluations (entropy-form JS)
    if (P.dbg && lane == 0) {
        unsigned long long* o = P.dbg + (static_cast<size_t>(blockIdx.x) * kWavesPerWG + wave) * 10;
        for (int i = 0; i < 8; ++i) o[i] = pt_acc[i];
        o[8] = pt_wall;
        o[9] = pt_last - pt_first;
    }
#endif
}

}  // namespace

#endif  // FSD_CSRC_PAIR_KERNEL_H_
