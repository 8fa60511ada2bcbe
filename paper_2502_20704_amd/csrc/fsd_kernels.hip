// HIP kernels and C ABI of the FSD candidate-verification step for gfx950 (MI355X).
//
// Three launches per call:
//   zero_counters   clears the counters and exchange words the next two kernels use
//   pair_kernel     the vocabulary reduction: one (target row, draft row) pair is split over a
//                   team of G wavefronts; every wavefront loads its slice of both rows ONCE into
//                   registers with 128-bit loads, the team exchanges the softmax normalisers
//                   through 64-bit words in the workspace, and the divergence (paper App. C.1-C.3)
//                   is accumulated from the registers.  One member per pair (they take turns) adds
//                   the team's partial sums in a fixed order, so results are run-to-run identical.
//   accept_sample   per sequence: the accepted prefix (Sec. 4, eq. 4) or accepted tree path
//                   (Sec. 6.4) or the strict-SD acceptance (Sec. 3, eq. 1-2), then the extra token
//                   by Gumbel-max over the vocabulary of one target row, split over GS workgroups.
//
// Nothing here is shared with the CPU oracle: Philox4x32-10 and the exact-operation logarithm
// are implemented a second time from their published / stated definitions.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <float.h>
#include <math.h>

#include "fsd.h"

namespace {

constexpr int kWG = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int kMaxRows = 2048;    // K or N
constexpr int kWalkShare = 8;     // workgroups that share a sequence's passes in the tree walk (at most)
constexpr float kLog2e = 1.44269504088896340736f;
constexpr double kLn2 = 0.69314718055994530942;
constexpr double kLog2eD = 1.44269504088896340736;

// MODE_KL: single-pass KL (absolute error ~1e-7, enough for bfloat16 inputs); MODE_KLP: two-phase,
// pointwise non-negative KL for binary32 inputs; MODE_LSE: normalisers only (strict SD)
enum { MODE_KL = 0, MODE_JS = 1, MODE_TV = 2, MODE_LSE = 3, MODE_KLP = 4 };
enum { KIND_CHAIN = 0, KIND_TREE = 1, KIND_SD = 2, KIND_RFSD = 3, KIND_TREESD = 4 };

#define AGENT __HIP_MEMORY_SCOPE_AGENT

// Optional phase timing of pair_kernel (development builds only: -DFSD_PHASE_TIMING).
#ifdef FSD_PHASE_TIMING
#define PT(i) do { const unsigned long long pt_now = __builtin_readcyclecounter(); pt_acc[i] += pt_now - pt_last; pt_last = pt_now; } while (0)
#else
#define PT(i) do { } while (0)
#endif

// ------------------------------------------------------------------------------------------
// small device helpers

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float hw_log2(float x) { return __builtin_amdgcn_logf(x); }

// Wavefront reductions on the data-parallel-primitive path (no LDS traffic): four steps reduce
// each row of 16 lanes (quad swaps, then mirrors), the four row totals are read back as scalars.
// Every lane gets the result; the order of the additions is fixed.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
    const int lo = dpp_i<CTRL>(__double2loint(v)), hi = dpp_i<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}
constexpr int kDppSwap1 = 0xB1, kDppSwap2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;   // last lane of a row to the next row(s)

__device__ __forceinline__ float lane_f(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ double lane_d(double v, int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l),
                            __builtin_amdgcn_readlane(__double2loint(v), l));
}
// the other rows' partial, or the neutral element 0 in rows the broadcast does not reach
template <int CTRL, int ROWS>
__device__ __forceinline__ double bcast_d(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROWS, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROWS, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Maximum over the wavefront, NaN ignored.  The compiler's own lowering of fmaxf() around a DPP
// move costs four instructions a step (it has to quieten a possible signalling NaN); the max
// instruction with a DPP operand does the same in one.  Each step waits two states for the
// previous write of its operand, as DPP reads require.
__device__ __forceinline__ float wave_max(float v) {
    asm("s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return lane_f(v, 63);
}
// Sums over the wavefront in a fixed order: within rows of 16 lanes, then row 0 into row 1 and
// row 2 into row 3, then rows 0-1 into rows 2-3; lane 63 holds the total.
__device__ __forceinline__ float wave_sumf(float v) {
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return lane_f(v, 63);
}
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_d<kDppSwap1>(v);
    v += dpp_d<kDppSwap2>(v);
    v += dpp_d<kDppHalfMirror>(v);
    v += dpp_d<kDppMirror>(v);
    v += bcast_d<kDppBcast15, 0xA>(v);
    v += bcast_d<kDppBcast31, 0xC>(v);
    return lane_d(v, 63);
}

// One 16-byte slot of a logits row: 8 bfloat16 or 4 binary32 values.
template <bool BF16> struct Slot { static constexpr int VE = BF16 ? 8 : 4; };

template <bool BF16>
__device__ __forceinline__ uint4 slot_neg_inf() {
    const unsigned w = BF16 ? 0xFF80FF80u : 0xFF800000u;
    return make_uint4(w, w, w, w);
}

// ALIGNED: rows start on 16-byte boundaries and V is a multiple of the slot width.
// Otherwise elements are fetched one by one and the ragged tail is padded with -inf.
template <bool BF16, bool ALIGNED>
__device__ __forceinline__ uint4 load_slot(const char* row, long slot, long V) {
    if constexpr (ALIGNED) {
        // a 32-bit offset from the row (rows are at most 2 MiB): the row pointer stays scalar
        return *reinterpret_cast<const uint4*>(row + static_cast<size_t>(static_cast<unsigned>(slot) * 16u));
    } else if constexpr (BF16) {
        const unsigned short* p = reinterpret_cast<const unsigned short*>(row);
        unsigned w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const long e = slot * 8 + 2 * d;
            const unsigned lo = (e < V) ? p[e] : 0xFF80u;
            const unsigned hi = (e + 1 < V) ? p[e + 1] : 0xFF80u;
            w[d] = lo | (hi << 16);
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    } else {
        const unsigned* p = reinterpret_cast<const unsigned*>(row);
        unsigned w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const long e = slot * 4 + d;
            w[d] = (e < V) ? p[e] : 0xFF800000u;
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <bool BF16>
__device__ __forceinline__ void unpack(const uint4& r, float* x) {
    if constexpr (BF16) {
        x[0] = __uint_as_float(r.x << 16); x[1] = __uint_as_float(r.x & 0xFFFF0000u);
        x[2] = __uint_as_float(r.y << 16); x[3] = __uint_as_float(r.y & 0xFFFF0000u);
        x[4] = __uint_as_float(r.z << 16); x[5] = __uint_as_float(r.z & 0xFFFF0000u);
        x[6] = __uint_as_float(r.w << 16); x[7] = __uint_as_float(r.w & 0xFFFF0000u);
    } else {
        x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
    }
}

template <bool BF16>
__device__ __forceinline__ float load_elem(const char* row, long e) {
    if constexpr (BF16)
        return __uint_as_float(static_cast<unsigned>(reinterpret_cast<const unsigned short*>(row)[e]) << 16);
    else
        return reinterpret_cast<const float*>(row)[e];
}

// ------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11) and the exact-operation Gumbel transform

struct U4 { unsigned x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0,
                                            unsigned k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32 x 32 -> 64 bit multiply gives both halves
        const unsigned long long p0 = static_cast<unsigned long long>(0xD2511F53u) * c0;
        const unsigned long long p1 = static_cast<unsigned long long>(0xCD9E8D57u) * c2;
        const unsigned hi0 = static_cast<unsigned>(p0 >> 32), lo0 = static_cast<unsigned>(p0);
        const unsigned hi1 = static_cast<unsigned>(p1 >> 32), lo1 = static_cast<unsigned>(p1);
        const unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

// (2*(w>>9)+1) * 2^-24: an odd 24-bit integer scaled, exact in binary32, inside (0,1)
__device__ __forceinline__ float word_to_uniform(unsigned w) {
    return __fmul_rn(static_cast<float>(((w >> 9) << 1) | 1u), 0x1p-24f);
}

// ln x for positive normal x using only correctly rounded operations:
// x = 2^e m, m in [sqrt(1/2), sqrt(2)); ln m = 2 atanh((m-1)/(m+1)), series to s^11.
__device__ __forceinline__ float flog32(float x) {
    const unsigned bits = __float_as_uint(x);
    int e = static_cast<int>(bits >> 23) - 127;
    float m = __uint_as_float((bits & 0x007FFFFFu) | 0x3F800000u);
    if (m >= 0x1.6a09e6p+0f) { m = __fmul_rn(m, 0.5f); e += 1; }
    const float s = __fdiv_rn(__fsub_rn(m, 1.0f), __fadd_rn(m, 1.0f));
    const float s2 = __fmul_rn(s, s);
    float poly = 0x1.745d18p-4f;
    poly = __fmaf_rn(poly, s2, 0x1.c71c72p-4f);
    poly = __fmaf_rn(poly, s2, 0x1.24924ap-3f);
    poly = __fmaf_rn(poly, s2, 0x1.99999ap-3f);
    poly = __fmaf_rn(poly, s2, 0x1.555556p-2f);
    poly = __fmaf_rn(poly, s2, 1.0f);
    const float lnm = __fmul_rn(__fmul_rn(2.0f, s), poly);
    return __fmaf_rn(static_cast<float>(e), 0x1.62e43p-1f, lnm);
}

__device__ __forceinline__ float gumbel(unsigned w) {
    const float t = -flog32(word_to_uniform(w));
    return -flog32(t);
}

// ------------------------------------------------------------------------------------------
// workspace view

struct Ws {
    unsigned* counters;  // 64 words ([1]: a bounded wait expired), then sdone[B]
    unsigned* sdone;     // [B] sampler workgroups that posted
    unsigned long long* part1;  // [R][G][4]: (kt,kd) | St | Sd | W
    double* part2;       // [R][G][4] divergence words (one used, four for TV)
    float* div;          // [R]
    int* pst;            // [R] status bits per pair
    double* lse2;        // [R][2] log2-sum-exp2 of the target / draft row of the pair
    double* lr;          // [R] strict SD: ln p(x) - ln q(x)
    unsigned long long* spart;  // [B][GS][4]
    float* thr;          // [B] warpers: smallest kept scaled logit of the sampled row
    int* tsd;            // [B][4 + rows] strict SD on a tree, from the walk to the sampler: status, depth,
                         // last node (-1 = root), length of the residual chain, then the chain's nodes
    float* tsd_invz;     // [B][rows] 1 / normaliser of the chain's residuals (all but the last)
    unsigned long long* wz;     // [B][rows][kWalkShare] the walk's partial normalisers, one round per rejection
};

struct PairParams {
    const char* target;
    const char* draft;
    const int32_t* parent;  // tree only
    const int32_t* cand;    // strict SD only
    int rows;               // K or N
    int npairs;             // B * rows
    long V;
    long nslots;
    int spm;                // slots per team member
    int G;
    unsigned spin_limit;
#ifdef FSD_PHASE_TIMING
    unsigned long long* dbg;   // [grid][4 wavefronts][10]
#endif
    float* user_div;        // optional [R]
    float* user_ratio;      // optional [R], reducible FSD only
    int want_ratio;         // 1: the finisher also writes ln p(x) - ln q(x) at the candidate token (reducible FSD)
    Ws ws;
};

// ------------------------------------------------------------------------------------------
// kernel 0: clear the counters and the exchange words (a zero word means "not posted yet")

__global__ void zero_counters(uint4* p, long n16) {
    const long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

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

// A pair owns 4 GW words of an exchange array, of which a mode uses N per member: word k of member
// m sits at [m N + k], so that a member's post is one contiguous store and the 64 lanes of a
// request touch consecutive words.  Lane l reads the N words of member (base + l); lanes beyond
// the team re-read the last member's (no branch around the loads, see load_item).  Nothing looks at the values here, so the loads stay in flight until they are
// awaited.  With spread == false every lane reads member 0 (a request whose result is not needed
// costs one cache line).
template <int N>
__device__ __forceinline__ void request_n(const unsigned long long* p, int GW, int base, unsigned long long (&w)[N],
                                          bool spread = true) {
    const int m = base + static_cast<int>(threadIdx.x & 63);
    const int mm = spread ? ((m < GW) ? m : GW - 1) : 0;
#pragma unroll
    for (int k = 0; k < N; ++k) w[k] = read64(p + mm * N + k);
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

__device__ __forceinline__ void merge_round(const unsigned long long (&w)[2], bool in, TeamNorm& n) {
    const float tk_t = lo_f(w[0]), tk_d = hi_f(w[0]);
    const float tSt = in ? lo_f(w[1]) : 0.0f, tSd = in ? hi_f(w[1]) : 0.0f;
    n.zt += wave_sumf((tSt > 0.0f) ? ldexpf(tSt, kdiff(tk_t, n.Kt)) : (tSt != tSt ? tSt : 0.0f));
    n.zd += wave_sumf((tSd > 0.0f) ? ldexpf(tSd, kdiff(tk_d, n.Kd)) : (tSd != tSd ? tSd : 0.0f));
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

template <int I> struct SetId { static constexpr int value = I; };

// wavefronts per SIMD the register allocation has to leave room for
constexpr int pair_kernel_waves(bool bf16, int nv, int mode) {
    return (bf16 && nv == 5 && (mode == MODE_JS || mode == MODE_TV)) ? 2 : 1;
}

template <bool BF16, int NV, int MODE, bool ALIGNED>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(pair_kernel_waves(BF16, NV, MODE))))
void pair_kernel(PairParams P) {
    constexpr int VE = Slot<BF16>::VE;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr bool TWO_PHASE = (MODE == MODE_JS || MODE == MODE_TV || MODE == MODE_KLP);
    constexpr int NE = TWO_PHASE ? NV * VE : 1;   // exponentials kept per row and lane
    constexpr int PW = (MODE == MODE_TV) ? 2 : 1;   // divergence words a member posts (two sums each)
    constexpr int FW = TWO_PHASE ? PW : 4;          // words per member the finisher reads
    // binary32 logits: the two-phase kernels hold 8 slots of each row per lane and one wavefront per
    // SIMD anyway, which leaves registers for a second set of logits
    constexpr bool DEEP = !BF16 && TWO_PHASE && NV == 8;
    // Phase 2 of a pair runs LAG steps after its phase 1.  With one step, a wavefront's own chain
    // from one phase 1 to the next still holds the whole latency of the exchange (post, then the
    // slowest member's words), which only another wavefront on the same SIMD can fill; with two,
    // every member's words have long been posted when they are looked at.  That takes a third set
    // of kept exponentials: the binary32 kernels with 8 slots per lane run one wavefront per SIMD
    // and have the registers.  (The bfloat16 kernels run two per SIMD and are bound by vector-ALU
    // issue: a third set kept in LDS removed their waits and left their time unchanged.)
    constexpr int LAG = (TWO_PHASE && !BF16 && NV == 8) ? 2 : 1;
    constexpr int NB = LAG + 1;                      // sets of kept exponentials
    constexpr int NC = (NE + 3) / 4;                 // chunks of four per row
    constexpr float kTiny = 2e-38f;   // keeps p + q > 0 without changing any result
    constexpr int kWavesPerWG = kWG / 64;

    // the wavefront's number as a scalar: everything derived from it (member, slot range, exchange
    // addresses) then lives in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    // NB sets of kept exponentials, named by SetId<> so that every index is a constant and the
    // arrays stay in registers; accessed four at a time
    float et[NB][NE], ed[NB][NE];
    auto put4 = [&](auto S, int c, const float (&t4)[4], const float (&d4)[4]) __attribute__((always_inline)) {
        constexpr int s_ = decltype(S)::value;
#pragma unroll
        for (int i = 0; i < 4; ++i) { et[s_][4 * c + i] = t4[i]; ed[s_][4 * c + i] = d4[i]; }
    };
    auto get4 = [&](auto S, int c, float (&t4)[4], float (&d4)[4]) __attribute__((always_inline)) {
        constexpr int s_ = decltype(S)::value;
#pragma unroll
        for (int i = 0; i < 4; ++i) { t4[i] = et[s_][4 * c + i]; d4[i] = ed[s_][4 * c + i]; }
    };
    const int GW = P.G;                                   // wavefronts per pair
    const int wgs_per_team = GW / kWavesPerWG;
    // A team is a run of consecutive workgroups, which the dispatcher spreads over the XCDs.  (Two
    // other deals were measured at C2 and dropped: teams whose workgroups all sit on one XCD ran a
    // third slower, and teams made half of early and half of late arrivals on the compute units
    // ended together but no sooner: the kernel is bound by vector-ALU issue either way.)
    const int nteams = static_cast<int>(gridDim.x) / wgs_per_team;
    const int team = static_cast<int>(blockIdx.x) / wgs_per_team;
    const int wg_in_team = static_cast<int>(blockIdx.x) % wgs_per_team;
    const int member = wg_in_team * kWavesPerWG + wave;
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

    auto row_ptrs = [&](int pair, const char*& tptr, const char*& dptr) __attribute__((always_inline)) {
        const int b = pair / P.rows;
        const int j = pair - b * P.rows;
        int trow = j;
        if (P.parent) {
            const int par = P.parent[pair];
            trow = (par >= -1 && par < j) ? par + 1 : 0;   // invalid parents are reported by the next kernel
        }
        tptr = P.target + (static_cast<size_t>(b) * (P.rows + 1) + trow) * static_cast<size_t>(P.V) * ES;
        dptr = P.draft + static_cast<size_t>(pair) * static_cast<size_t>(P.V) * ES;
    };
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
    auto load_item = [&](uint4 (&ra)[NV], uint4 (&rb)[NV], int pair, bool wanted = true) __attribute__((always_inline)) {
        const char *tptr, *dptr;
        row_ptrs(pair, tptr, dptr);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int sk = sl0 + 64 * k;
            const long sl = wanted ? (sk < sl_end ? sk : sl_last) : 0;   // not wanted: one cached slot for all lanes
            ra[k] = load_slot<BF16, ALIGNED>(tptr, sl, P.V);
            rb[k] = load_slot<BF16, ALIGNED>(dptr, sl, P.V);
        }
    };
    auto fill_unowned = [&](uint4 (&ra)[NV], uint4 (&rb)[NV]) __attribute__((always_inline)) {
        if (fill_needed) {
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                if (sl0 + 64 * k >= sl_end) { ra[k] = slot_neg_inf<BF16>(); rb[k] = slot_neg_inf<BF16>(); }
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
        const unsigned long long* p2 = part2 + static_cast<size_t>(pair) * GW * 4;
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
            const double A = s.lo[0], Bn = s.hi[0], MA = s.lo[1], MB = s.hi[1];
            value = (MA != MA || MB != MB) ? __builtin_nan("") : (MA <= MB ? A : Bn);
        } else {
            value = 0.5 * kLn2 * s.lo[0];
        }
        int status = 0;
        if (value != value) status |= FSD_ROW_NONFINITE;   // NaN / +inf logits, or a row without mass
        if (!s.ok) status |= FSD_ROW_INTERNAL;
        if (value < 0.0) value = 0.0;
        if (status) value = __builtin_nan("");
        double lse2_t = 0.0, lse2_d = 0.0;
        if (P.want_ratio) {
            // reducible FSD also needs the rows' normalisers: the team's phase-1 words once more, this
            // time merged in float64 (they were all posted before the divergence words read above)
            const unsigned long long* p1 = part1 + static_cast<size_t>(pair) * GW * 4;
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
        const unsigned long long* p1 = part1 + static_cast<size_t>(pair) * GW * 4;
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
    auto finish = [&](int pair, unsigned long long (&fw)[FW]) __attribute__((always_inline)) {
        if constexpr (TWO_PHASE) finish_two_phase(pair, fw); else finish_single_pass(pair, fw);
    };

    // ---- state of the previous pair, whose phase 2 is still to come (two-phase modes)
    struct Pend { int pair; float kt, kd; bool mass_t, mass_d, mask; };
    Pend pend[LAG];   // [0] the last step's pair ... [LAG-1] the one whose phase 2 is due
#pragma unroll
    for (int i = 0; i < LAG; ++i) pend[i] = Pend{-1, 0.0f, 0.0f, false, false, false};
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
        const unsigned long long* p1 = part1 + static_cast<size_t>(pp.pair) * GW * 4;
        // binary32 is enough: the normalisers enter p and q as common factors
        TeamNorm n{pp.kt, pp.kd, 0.0f, 0.0f, true};
        n.ok = await_n<2>(p1, GW, 0, P.spin_limit, w);
        merge_round(w, lane < GW, n);
        if (GW > 64) {
            // members 64..127 were requested with the first 64; larger teams ask for the rest here
            if (!await_n<2>(p1, GW, 64, P.spin_limit, w2)) n.ok = false;
            merge_round(w2, 64 + lane < GW, n);
            if (GW > 128) n = merge_more_rounds(p1, GW, P.spin_limit, n);
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
        unsigned long long word[PW];
        if constexpr (MODE == MODE_TV) {
            float A = 0.0f, Bn = 0.0f, MA = 0.0f, MB = 0.0f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                float t4[4], d4[4];
                get4(S, c, t4, d4);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = t4[i] * ft, q = d4[i] * fd;   // separately rounded: p == q for equal rows
                    const float d = p - q, sum = p + q;
                    A += fmaxf(d, 0.0f);
                    Bn += fmaxf(-d, 0.0f);
                    MA += (d > 0.0f) ? sum : 0.0f;
                    MB += (d < 0.0f) ? sum : 0.0f;
                }
            }
            // max() drops NaN: an unusable row (NaN factor) is made to reach the side selection
            if (ft != ft || fd != fd) { A = ft + fd; Bn = A; MA = A; MB = A; }
            A = wave_sumf(A);
            Bn = wave_sumf(Bn);
            MA = wave_sumf(MA);
            MB = wave_sumf(MB);
            if (!ok) { A = __builtin_nanf(""); MA = A; }
            word[0] = pack2(A, Bn);
            word[1] = pack2(MA, MB);
        } else {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
              float t4[4], d4[4];
              get4(S, c, t4, d4);
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const float p = fmaf(t4[i], ft, kTiny), q = fmaf(d4[i], fd, kTiny);
                const float d = p - q, sum = p + q;
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
            if constexpr (MODE == MODE_KLP) {
                if (__any(pp.mask)) acc += __builtin_inff();   // draft masks an entry the target keeps; NaN stays NaN
            }
            if (!ok) acc = __builtin_nanf("");
            word[0] = pack2(acc, 0.0f);
        }
        if (!ok && lane == 0) atomicOr(P.ws.counters + 1, 1u);
        if (lane < PW) {
            unsigned long long mine = word[0];
#pragma unroll
            for (int k = 1; k < PW; ++k) mine = (lane == k) ? word[k] : mine;
            // the lane's offset is recomputed here (hidden from loop-invariant hoisting): kept across
            // the loop it would be spilled, and the reload would wait for every load in flight
            int l = lane;
            asm volatile("" : "+v"(l));
            post64(part2 + static_cast<size_t>(pp.pair) * GW * 4 + member * PW + l, mine);
        }
    };

    auto finish_now = [&](int pair) __attribute__((always_inline)) {
        unsigned long long fw[FW];
        request_n<FW>(finw + static_cast<size_t>(pair) * GW * 4, GW, 0, fw);
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
    // as soon as phase 1 has consumed the registers; and nothing after that waits on memory unless a
    // team member is late (then the words are asked for again, behind the prefetch).
    // (ra, rb) hold the logits of `pair`, the next pair's go to (rna, rnb).  Where registers allow
    // (DEEP) these are two sets and the next pair is requested at the top of the step, a whole step
    // ahead; otherwise both names are the same set and the request follows phase 1.
    // SC names the set that takes this pair's exponentials, SP the one written LAG steps ago.
    auto step = [&](auto SC, auto SP, uint4 (&ra)[NV], uint4 (&rb)[NV], uint4 (&rna)[NV], uint4 (&rnb)[NV], int pair)
                    __attribute__((always_inline)) {
        unsigned long long w[2] = {1, 1}, w2[2] = {1, 1};
        unsigned long long fw[FW];
        const int fpair = TWO_PHASE ? fin[0] : ((sp_pair >= 0 && iter >= sp_due) ? sp_pair : -1);
        const Pend due = pend[LAG - 1];
        // Phase 1 and the request for the next pair's logits are what the whole team waits for: they
        // run at raised priority; what follows overlaps with the memory latency and does not need it.
        __builtin_amdgcn_s_setprio(3);
        asm volatile("" ::: "memory");
        if constexpr (TWO_PHASE)
        {
            const unsigned long long* const p1 = part1 + static_cast<size_t>(due.pair >= 0 ? due.pair : pair) * GW * 4;
            request_n<2>(p1, GW, 0, w);
            request_n<2>(p1, GW, 64, w2, GW > 64);
        }
        request_n<FW>(finw + static_cast<size_t>(fpair >= 0 ? fpair : pair) * GW * 4, GW, 0, fw, fpair >= 0);
        if constexpr (DEEP) {
            // this pair's logits arrived in the second set a step ago; move them and ask for the next pair's
#pragma unroll
            for (int k = 0; k < NV; ++k) { ra[k] = rna[k]; rb[k] = rnb[k]; }
            asm volatile("" ::: "memory");
            const bool more = pair + nteams < P.npairs;
            load_item(rna, rnb, more ? pair + nteams : pair, more);
        }
        asm volatile("" ::: "memory");
        fill_unowned(ra, rb);
        // ---- phase 1: maximum, then sums of 2^(z log2e - k) with k = ceil(max log2e)
        float mt = neg_inf(), md = neg_inf();
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            float a[VE], c[VE];
            unpack<BF16>(ra[k], a);
            unpack<BF16>(rb[k], c);
#pragma unroll
            for (int e = 0; e < VE; e += 2) { mt = fmaxf(fmaxf(mt, a[e]), a[e + 1]); md = fmaxf(fmaxf(md, c[e]), c[e + 1]); }
        }
        PT(0);   // load wait + max pass
        mt = wave_max(mt);
        md = wave_max(md);
        const float kt = (mt == neg_inf()) ? 0.0f : ceilf(mt * kLog2e);
        const float kd = (md == neg_inf()) ? 0.0f : ceilf(md * kLog2e);
        float st = 0.0f, sd = 0.0f, wacc = 0.0f, dmax = neg_inf();
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            float a[VE], c[VE];
            unpack<BF16>(ra[k], a);
            unpack<BF16>(rb[k], c);
            float xa_[VE], xb_[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                const float xa = hw_exp2(fmaf(a[e], kLog2e, -kt));
                const float xb = hw_exp2(fmaf(c[e], kLog2e, -kd));
                xa_[e] = xa;
                xb_[e] = xb;
                st += xa;
                sd += xb;
                if constexpr (MODE == MODE_KL || MODE == MODE_KLP) {
                    const float diff = a[e] - c[e];
                    dmax = fmaxf(dmax, diff);   // +inf iff the draft masks an entry the target does not
                    if constexpr (MODE == MODE_KL) wacc = fmaf(xa, fminf(fmaxf(diff, -FLT_MAX), FLT_MAX), wacc);
                }
            }
            if constexpr (TWO_PHASE) {
#pragma unroll
                for (int h = 0; h < VE / 4; ++h) {
                    const float t4[4] = {xa_[4 * h], xa_[4 * h + 1], xa_[4 * h + 2], xa_[4 * h + 3]};
                    const float d4[4] = {xb_[4 * h], xb_[4 * h + 1], xb_[4 * h + 2], xb_[4 * h + 3]};
                    put4(SC, k * (VE / 4) + h, t4, d4);
                }
            }
        }
        PT(1);   // reductions + exp pass
        // ---- the registers that held the logits are free: fetch the next pair (the request is
        // unconditional: the last step asks for one slot of its own pair, which the caches hold)
        asm volatile("" ::: "memory");
        if constexpr (!DEEP) {
            const bool more = pair + nteams < P.npairs;
            load_item(rna, rnb, more ? pair + nteams : pair, more);
        }
        __builtin_amdgcn_s_setprio(0);
        asm volatile("" ::: "memory");
        // ---- post this wavefront's partial.  The two-phase modes need the normalisers to a relative
        // 1e-7 only (common factors of p and q); the single-pass modes take them through a logarithm.
        const unsigned long long w0 = pack2(kt, kd);
        unsigned long long mine;
        if constexpr (TWO_PHASE) {
            st = wave_sumf(st);
            sd = wave_sumf(sd);
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
        constexpr int kPosted = TWO_PHASE ? 2 : 4;
        unsigned long long* const post_at = part1 + static_cast<size_t>(pair) * GW * 4 + member * kPosted + (lane & 3);
        if (lane < kPosted) post64(post_at, mine);
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
            pend[0] = Pend{pair, kt, kd, (st > 0.0f) || (st != st), (sd > 0.0f) || (sd != sd), dmax == __builtin_inff()};
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
        ++iter;
    };

    uint4 r0a[NV], r0b[NV], r1a[DEEP ? NV : 1], r1b[DEEP ? NV : 1];
    int pair = team;
    if (pair < P.npairs) {
        if constexpr (DEEP) load_item(r1a, r1b, pair); else load_item(r0a, r0b, pair);
    }
    auto one_step = [&](auto SC, auto SP, int pr) __attribute__((always_inline)) {
        if constexpr (DEEP) step(SC, SP, r0a, r0b, r1a, r1b, pr);
        else step(SC, SP, r0a, r0b, r0a, r0b, pr);
    };
    if constexpr (TWO_PHASE) {
        // step i keeps its exponentials in set i % NB and reads the set written LAG steps earlier
        bool live = pair < P.npairs;
        while (live) {
            one_step(SetId<0>{}, SetId<1 % NB>{}, pair);
            pair += nteams;
            live = pair < P.npairs;
            if (live) {
                one_step(SetId<1>{}, SetId<2 % NB>{}, pair);
                pair += nteams;
                live = pair < P.npairs;
            }
            if constexpr (NB == 3) {
                if (live) {
                    one_step(SetId<2>{}, SetId<0>{}, pair);
                    pair += nteams;
                    live = pair < P.npairs;
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
                request_n<2>(part1 + static_cast<size_t>(pp.pair) * GW * 4, GW, 0, w);
                request_n<2>(part1 + static_cast<size_t>(pp.pair) * GW * 4, GW, 64, w2, GW > 64);
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
        for (; pair < P.npairs; pair += nteams) one_step(SetId<0>{}, SetId<1>{}, pair);
        if (sp_pair >= 0) finish_now(sp_pair);
    }
#ifdef FSD_PHASE_TIMING
    PT(6);   // drain
    if (P.dbg && lane == 0) {
        unsigned long long* o = P.dbg + (static_cast<size_t>(blockIdx.x) * kWavesPerWG + wave) * 10;
        for (int i = 0; i < 8; ++i) o[i] = pt_acc[i];
        o[8] = pt_wall;
        o[9] = pt_last - pt_first;
    }
#endif
}

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
            if constexpr (KIND == KIND_SD || KIND == KIND_RFSD) {   // reducible FSD (Sec. 4.2): either rule accepts
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
        const bool gave_up = P.ws.counters[1] != 0;
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
    if (P.ws.counters[1]) status |= FSD_ROW_INTERNAL;   // a bounded wait of the reduction kernel expired

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
        // Scores already seen anywhere in the wavefront: an entry whose score cannot reach them cannot
        // be the argmax, and its Gumbel variate (two logarithms) is not evaluated.  The bound:
        // G = -ln(-ln u) <= -ln(1 - u), and 1 - u = m 2^-24 with the integer m below, so
        // G <= ln2 (24 - floor(log2 m)) = ln2 (clz(m) - 7); 1e-3 covers the rounding of the
        // logarithm routine by a wide margin.
        float thr = neg_inf(), rthr = neg_inf();
        const float thr_b = P.thr ? P.thr[b] : neg_inf();
        // the trip count is the same for every lane: the thresholds are wavefront reductions
        for (long sb = s0; sb < s1; sb += kWG) {
            const long s = sb + tid;
            const bool live = s < s1;
            float z[VE], zd[VE];
            const uint4 raw = load_slot<BF16, ALIGNED>(trow, live ? s : s1 - 1, P.V);
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
            if (P.mode == FSD_SAMPLE) {
                // No variate is below -ln(24 ln 2) = -2.8116 (u >= 2^-24), so the largest logit seen minus
                // 2.82 is already a score the winner must reach: most entries are ruled out before any
                // variate has been evaluated at all.
                float zm = neg_inf();
#pragma unroll
                for (int e = 0; e < VE; ++e) zm = fmaxf(zm, z[e]);
                thr = fmaxf(thr, wave_max(live ? zm : neg_inf()) - 2.82f);
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
#pragma unroll
            for (int blk = 0; blk < VE / 4; ++blk) {
                const long e0 = s * VE + blk * 4;
                unsigned w4[4] = {0u, 0u, 0u, 0u};
                if (P.mode == FSD_SAMPLE) {
                    const U4 r = philox4x32_10(static_cast<unsigned>(e0 >> 2), static_cast<unsigned>(b), P.off_lo,
                                               P.off_hi, P.seed_lo, P.seed_hi);
                    w4[0] = r.x; w4[1] = r.y; w4[2] = r.z; w4[3] = r.w;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float zz = z[blk * 4 + q];
                    const int idx = static_cast<int>(e0 + q);
                    bad |= !(zz < __builtin_inff());
                    float lnr = neg_inf();
                    if (residual) {
                        float r;
                        if constexpr (KIND == KIND_TREESD) {
                            r = rres[blk * 4 + q];
                        } else {
                            const float p = hw_exp2(fmaf(zz, kLog2e, -lt));
                            const float qq = hw_exp2(fmaf(zd[blk * 4 + q], kLog2e, -ld));
                            r = p - qq;
                        }
                        if (r > 0.0f) lnr = hw_log2(r) * static_cast<float>(kLn2);
                    }
                    if (P.mode == FSD_SAMPLE) {
                        const unsigned m = 0x00FFFFFFu ^ ((w4[q] >> 9) << 1);   // (1 - u) 2^24, odd, >= 1
                        const float gb = fmaf(static_cast<float>(__clz(static_cast<int>(m)) - 7), 0.693148f, 1e-3f);
                        const bool may = !(__fadd_rn(zz, gb) < thr) || (residual && !(__fadd_rn(lnr, gb) < rthr));
                        if (may) {
                            const float g = gumbel(w4[q]);
                            const float score = __fadd_rn(zz, g);
                            if (score > best.score) best = Best{score, idx};
                            if (lnr > neg_inf()) {
                                const float rs = __fadd_rn(lnr, g);
                                if (rs > rbest.score) rbest = Best{rs, idx};
                            }
                        }
                    } else {
                        if (zz > best.score) best = Best{zz, idx};
                        if (lnr > rbest.score) rbest = Best{lnr, idx};
                    }
                }
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
        unsigned long long* slot = P.ws.spart + (static_cast<size_t>(b) * P.GS + gs) * 4;
        __hip_atomic_store(slot + 0, (static_cast<unsigned long long>(__float_as_uint(m.score)) << 32) | static_cast<unsigned>(m.idx), __ATOMIC_RELAXED, AGENT);
        __hip_atomic_store(slot + 1, (static_cast<unsigned long long>(__float_as_uint(r.score)) << 32) | static_cast<unsigned>(r.idx), __ATOMIC_RELAXED, AGENT);
        __hip_atomic_store(slot + 2, static_cast<unsigned long long>(bd), __ATOMIC_RELAXED, AGENT);
        // The three words above are device-scope atomic stores, performed at the memory side; the
        // wait for their completion orders them before the count (a device-scope release would also
        // write the whole L2 back, which costs far more than the kernel's arithmetic).  The reader
        // uses device-scope atomic loads, so it needs no invalidate either.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        const unsigned prev = __hip_atomic_fetch_add(P.ws.sdone + b, 1u, __ATOMIC_RELAXED, AGENT);
        s_last = (prev == static_cast<unsigned>(P.GS) - 1u) ? 1 : 0;
    }
    __syncthreads();
    if (!s_last) return;

    // ---- the last workgroup of the sequence merges the shares and writes the outputs
    if (tid == 0) {
        Best m{neg_inf(), 0x7FFFFFFF}, r{neg_inf(), 0x7FFFFFFF};
        int bd = 0;
        for (int k = 0; k < P.GS; ++k) {
            const unsigned long long* slot = P.ws.spart + (static_cast<size_t>(b) * P.GS + k) * 4;
            const unsigned long long w0 = __hip_atomic_load(slot + 0, __ATOMIC_RELAXED, AGENT);
            const unsigned long long w1 = __hip_atomic_load(slot + 1, __ATOMIC_RELAXED, AGENT);
            bd |= static_cast<int>(__hip_atomic_load(slot + 2, __ATOMIC_RELAXED, AGENT));
            m = better(m, Best{__uint_as_float(static_cast<unsigned>(w0 >> 32)), static_cast<int>(static_cast<unsigned>(w0))});
            r = better(r, Best{__uint_as_float(static_cast<unsigned>(w1 >> 32)), static_cast<int>(static_cast<unsigned>(w1))});
        }
        int st = status;
        if (!st && (bd || m.idx == 0x7FFFFFFF)) st |= FSD_ROW_NONFINITE;
        const int tok = (residual && r.idx != 0x7FFFFFFF) ? r.idx : m.idx;
        s_st = st;
        s_key = tok;
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
    }
}

// ------------------------------------------------------------------------------------------
// strict SD over a token tree: the walk
//
// The tree analogue of strict SD's acceptance (Sec. 3, eq. 1-3, applied child by child as in the
// tree-verification methods Sec. 2 cites).  At the current context with target distribution p the
// children are tried in index order: child j is accepted iff min(1, p(x_j)/q_j(x_j)) > y_j; after a
// rejection p becomes the normalised positive part of p - q_j.  One workgroup per sequence walks
// the tree.  The first child of a context is tested against the log-ratio the reduction kernel has
// stored; a later child needs p after the rejections so far, evaluated at its token through the
// chain of rejected draft rows, and every rejection that is followed by another sibling costs one
// pass over the vocabulary for its normaliser.  The token itself is drawn by accept_sample from
// what this kernel leaves in the workspace.
//
// gridDim.x workgroups share a sequence (all of them resident at once, which the host checks):
// every one walks the same tree and takes the same decisions, a pass is split between them, and
// the partial sums meet through 64-bit words in the workspace that are zero until posted, one
// round of words per pass.  Every workgroup adds the partials in the same order, so all see the
// same normaliser.  Waiting is bounded: a workgroup that gives up sets the call's internal-error
// flag and leaves.  Workgroup 0 of a sequence writes the outputs.
struct WalkParams {
    const char* target;
    const char* draft;
    const int32_t* tokens;    // [B,N]
    const int32_t* parent;    // [B,N]
    int rows;                 // N
    int max_depth;
    long V;
    long nslots;
    unsigned seed_lo, seed_hi, off_lo, off_hi;
    int32_t* path_nodes;      // [B,max_depth]
    int32_t* out_tokens;      // [B,max_depth+1]
    float* user_ratio;        // optional [B,N]
    unsigned spin_limit;
    Ws ws;
};

constexpr int kWalkWG = 1024;

template <bool BF16, bool ALIGNED>
__global__ __launch_bounds__(kWalkWG) void tree_sd_walk(WalkParams P) {
    constexpr int VE = Slot<BF16>::VE;
    constexpr int ES = BF16 ? 2 : 4;
    extern __shared__ int s_walk[];   // par[N], dep[N], chain[N], then Z[N] (float64)
    __shared__ double s_red[kWalkWG / 64];
    __shared__ int s_st;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y, N = P.rows;
    const int g = blockIdx.x, GSW = gridDim.x;
    const bool writer = (g == 0);
    int* par = s_walk;
    int* dep = s_walk + N;
    int* chain = s_walk + 2 * N;
    float* s_invz = reinterpret_cast<float*>(s_walk + 3 * N);
    double* Zs = reinterpret_cast<double*>(s_walk + 4 * N);
    const double* lr_of = P.ws.lr + static_cast<size_t>(b) * N;
    const double* lse_of = P.ws.lse2 + 2 * static_cast<size_t>(b) * N;
    int* hdr = P.ws.tsd + static_cast<size_t>(b) * (4 + N);
    float* invz = P.ws.tsd_invz + static_cast<size_t>(b) * N;
    int32_t* pn = P.path_nodes + static_cast<size_t>(b) * P.max_depth;
    int32_t* out = P.out_tokens + static_cast<size_t>(b) * (P.max_depth + 1);
    const int32_t* tok = P.tokens + static_cast<size_t>(b) * N;

    if (tid == 0) s_st = 0;
    __syncthreads();
    for (int j = tid; j < N; j += kWalkWG) {
        const size_t pr = static_cast<size_t>(b) * N + j;
        int p = P.parent[pr];
        if (p < -1 || p >= j) { atomicOr(&s_st, FSD_ROW_BAD_PARENT); p = -1; }
        const int st = P.ws.pst[pr];
        if (st) atomicOr(&s_st, st);
        par[j] = p;
        if (writer && P.user_ratio) P.user_ratio[pr] = __builtin_nanf("");
    }
    if (writer) {
        for (int i = tid; i < P.max_depth; i += kWalkWG) pn[i] = -1;
        for (int i = tid; i <= P.max_depth; i += kWalkWG) out[i] = -1;
    }
    __syncthreads();
    if (tid == 0) {
        for (int j = 0; j < N; ++j) {   // parents come first, so one sweep gives the depths
            dep[j] = par[j] < 0 ? 1 : dep[par[j]] + 1;
            if (dep[j] > P.max_depth) s_st |= FSD_ROW_TOO_DEEP;
        }
    }
    __syncthreads();
    int status = s_st;
    if (status & FSD_ROW_BAD_PARENT) status &= ~FSD_ROW_TOO_DEEP;
    if (P.ws.counters[1]) status |= FSD_ROW_INTERNAL;
    if (status) {
        if (writer && tid == 0) { hdr[0] = status; hdr[1] = 0; hdr[2] = -1; hdr[3] = 0; }
        return;
    }
    // this workgroup's share of a pass
    const long share = (P.nslots + GSW - 1) / GSW;
    const long sl_lo = static_cast<long>(g) * share;
    const long sl_hi = (sl_lo + share < P.nslots) ? sl_lo + share : P.nslots;
    int round = 0;   // passes so far in this sequence

    const size_t rowb = static_cast<size_t>(P.V) * ES;
    int cur = -1, n = 0, nrej = 0, last_j = -1, before_last = 0;
    for (;;) {   // every value below is the same in all threads
        const char* trow = P.target + (static_cast<size_t>(b) * (N + 1) + (cur + 1)) * rowb;
        nrej = 0; last_j = -1; before_last = 0;
        int next = -1;
        for (int j = cur + 1; j < N; ++j) {
            if (par[j] != cur) continue;
            const size_t pr = static_cast<size_t>(b) * N + j;
            const char* drow = P.draft + pr * rowb;
            const int x = tok[j];
            const double lt2 = lse_of[2 * j], ld2 = lse_of[2 * j + 1];
            double ratio;
            if (nrej == 0) {
                ratio = lr_of[j];
            } else {
                double r = exp2(static_cast<double>(load_elem<BF16>(trow, x)) * kLog2eD - lt2);
                for (int m = 0; m < nrej; ++m) {
                    const size_t pc = static_cast<size_t>(b) * N + chain[m];
                    const double q = exp2(static_cast<double>(load_elem<BF16>(P.draft + pc * rowb, x)) * kLog2eD - lse_of[2 * chain[m] + 1]);
                    r = fmax(r - q, 0.0) / Zs[m];
                }
                const double lq = (static_cast<double>(load_elem<BF16>(drow, x)) * kLog2eD - ld2) * kLn2;
                ratio = (r > 0.0) ? log(r) - lq : -__builtin_inf();
            }
            // Sec. 3 eq. 1-2 in the log domain, with the uniform number of index j
            const U4 rw = philox4x32_10((static_cast<unsigned>(j) >> 2) | (1u << 30), static_cast<unsigned>(b), P.off_lo,
                                        P.off_hi, P.seed_lo, P.seed_hi);
            const unsigned wsel = (j & 3) == 0 ? rw.x : (j & 3) == 1 ? rw.y : (j & 3) == 2 ? rw.z : rw.w;
            const double u = static_cast<double>(word_to_uniform(wsel));
            const double thr = ratio < 0.0 ? ratio : 0.0;
            if (writer && tid == 0 && P.user_ratio) P.user_ratio[pr] = static_cast<float>(ratio);
            if (thr - log(u) > 0.0) { next = j; break; }
            last_j = j;
            before_last = nrej;
            bool more = false;
            for (int j2 = j + 1; j2 < N; ++j2) more |= (par[j2] == cur);
            if (!more) break;
            // ---- the normaliser of the positive part of p - q_j, p being the distribution in force
            const float ltf = static_cast<float>(lt2), ldf = static_cast<float>(ld2);
            // CH slots per thread at a time, row by row: the CH loads of a row are in flight together
            // (one slot at a time, each load waited for the one before it)
            constexpr int CH = BF16 ? 4 : 8;
            double acc = 0.0;
            for (long base = sl_lo; base < sl_hi; base += static_cast<long>(kWalkWG) * CH) {
                float pv[CH][VE];
                uint4 raw[CH];
                long slc[CH];
                bool in[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const long sl = base + static_cast<long>(c) * kWalkWG + tid;
                    in[c] = sl < sl_hi;
                    slc[c] = in[c] ? sl : P.nslots - 1;
                    raw[c] = load_slot<BF16, ALIGNED>(trow, slc[c], P.V);
                }
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    float z[VE];
                    unpack<BF16>(raw[c], z);
#pragma unroll
                    for (int e = 0; e < VE; ++e) pv[c][e] = in[c] ? hw_exp2(fmaf(z[e], kLog2e, -ltf)) : 0.0f;
                }
                for (int m = 0; m < nrej; ++m) {
                    const size_t pc = static_cast<size_t>(b) * N + chain[m];
                    const char* cr = P.draft + pc * rowb;
#pragma unroll
                    for (int c = 0; c < CH; ++c) raw[c] = load_slot<BF16, ALIGNED>(cr, slc[c], P.V);
                    const float ldm = static_cast<float>(lse_of[2 * chain[m] + 1]), izm = s_invz[m];
#pragma unroll
                    for (int c = 0; c < CH; ++c) {
                        float zd[VE];
                        unpack<BF16>(raw[c], zd);
#pragma unroll
                        for (int e = 0; e < VE; ++e)
                            pv[c][e] = fmaxf(pv[c][e] - hw_exp2(fmaf(zd[e], kLog2e, -ldm)), 0.0f) * izm;
                    }
                }
#pragma unroll
                for (int c = 0; c < CH; ++c) raw[c] = load_slot<BF16, ALIGNED>(drow, slc[c], P.V);
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    float zd[VE];
                    unpack<BF16>(raw[c], zd);
                    float part = 0.0f;
#pragma unroll
                    for (int e = 0; e < VE; ++e) part += fmaxf(pv[c][e] - hw_exp2(fmaf(zd[e], kLog2e, -ldf)), 0.0f);
                    acc += static_cast<double>(part);
                }
            }
            acc = wave_sum(acc);
            __syncthreads();   // the previous round's readers are done with s_red
            if (lane == 0) s_red[wave] = acc;
            __syncthreads();
            double Z = 0.0;
            for (int w = 0; w < kWalkWG / 64; ++w) Z += s_red[w];   // same order in every thread
            if (GSW > 1) {
                // ---- meet the other workgroups of the sequence: post this share, read all of them
                unsigned long long* const words = P.ws.wz + (static_cast<size_t>(b) * N + round) * kWalkShare;
                if (tid == 0) post64(words + g, dbits(Z));
                __syncthreads();   // everyone has read s_red
                if (tid < GSW) {
                    unsigned long long v = 0;
                    unsigned polls = 0;
                    for (;;) {
                        v = read64(words + tid);
                        if (v != 0 || polls++ >= P.spin_limit) break;
                        __builtin_amdgcn_s_sleep(2);
                    }
                    s_red[tid] = (v != 0) ? bitsd(v) : __builtin_nan("");
                }
                __syncthreads();
                Z = 0.0;
                for (int w = 0; w < GSW; ++w) Z += s_red[w];
                if (Z != Z) {   // a workgroup of this sequence never posted: give up, the call reports it
                    if (tid == 0) atomicOr(P.ws.counters + 1, 1u);
                    return;
                }
            }
            ++round;
            if (Z > 0.0) {
                if (tid == 0) {
                    chain[nrej] = j; Zs[nrej] = Z; s_invz[nrej] = static_cast<float>(1.0 / Z);
                    if (writer) invz[nrej] = static_cast<float>(1.0 / Z);
                }
                __syncthreads();
                ++nrej;
            }
        }
        if (next < 0) break;
        if (writer && tid == 0) { pn[n] = next; out[n] = tok[next]; }
        ++n;
        cur = next;
    }
    // ---- what the sampler needs: the residual chain ends with the last rejected child, whose
    // normaliser nobody needs
    if (writer && tid == 0) {
        hdr[0] = 0;
        hdr[1] = n;
        hdr[2] = cur;
        const int nchain = (last_j >= 0) ? before_last + 1 : 0;
        hdr[3] = nchain;
        for (int m = 0; m < before_last && m < nchain; ++m) hdr[4 + m] = chain[m];
        if (nchain > 0) hdr[4 + nchain - 1] = last_j;
    }
}

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
    int rows;             // K
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
    if (tid == 0) { s_n = P.rows; s_st = 0; }
    __syncthreads();
    for (int i = tid; i < P.rows; i += kWarpWG) {
        const int pr = b * P.rows + i;
        if (P.ws.pst[pr]) atomicOr(&s_st, 1);
        if (!(P.ws.div[pr] <= P.T)) atomicMin(&s_n, i);
    }
    __syncthreads();
    if (s_st || P.ws.counters[1]) {   // nothing will be drawn for this sequence
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

// ------------------------------------------------------------------------------------------
// threshold tuning on a dev set (Sec. 5.3, App. A): the smallest occurring T at which the chain rule
// accepts a given share of all candidate positions.  A position is accepted iff every divergence up
// to it is <= T, i.e. iff the running maximum of its sequence is: T is the ceil(fraction n)-th
// smallest running maximum.  Non-negative binary32 values order like their bit patterns, so the
// order statistic is found exactly by a radix select over four 8-bit digits.

struct CalibState { unsigned prefix, mask, rank, count_le; unsigned hist[256]; };
constexpr unsigned kCalibInf = 0x7F800000u, kCalibNever = 0x7FFFFFFFu;

__global__ void calib_keys(const float* div, int B, int K, unsigned* keys) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    float m = 0.0f;
    bool dead = false;
    for (int i = 0; i < K; ++i) {
        const float d = div[static_cast<size_t>(b) * K + i];
        // an unusable position (NaN) is never accepted, nor is anything after it: a key above +inf
        dead |= (d != d);
        m = fmaxf(m, d);
        keys[static_cast<size_t>(b) * K + i] = dead ? kCalibNever : __float_as_uint(m);
    }
}
__global__ void calib_init(CalibState* st, unsigned rank) {
    const int t = threadIdx.x;
    if (t == 0) { st->prefix = 0u; st->mask = 0u; st->rank = rank; st->count_le = 0u; }
    st->hist[t] = 0u;
}
__global__ void calib_hist(const unsigned* keys, long n, int shift, CalibState* st) {
    __shared__ unsigned h[256];
    h[threadIdx.x] = 0u;
    __syncthreads();
    const unsigned prefix = st->prefix, mask = st->mask;
    for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += static_cast<long>(gridDim.x) * blockDim.x) {
        const unsigned k = keys[i];
        if ((k & mask) == prefix) atomicAdd(&h[(k >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&st->hist[threadIdx.x], h[threadIdx.x]);
}
// one workgroup of 256: the digit whose cumulative count reaches the rank; clears the histogram
__global__ void calib_pick(CalibState* st, int shift) {
    __shared__ unsigned h[256];
    const int t = threadIdx.x;
    h[t] = st->hist[t];
    st->hist[t] = 0u;
    __syncthreads();
    if (t == 0) {
        unsigned rank = st->rank, below = 0u;
        int d = 0;
        for (; d < 255; ++d) {
            if (below + h[d] >= rank) break;
            below += h[d];
        }
        st->prefix |= static_cast<unsigned>(d) << shift;
        st->mask |= 255u << shift;
        st->rank = rank - below;
    }
}
__global__ void calib_count(const unsigned* keys, long n, CalibState* st) {
    __shared__ unsigned c;
    if (threadIdx.x == 0) c = 0u;
    __syncthreads();
    const unsigned key = st->prefix < kCalibInf ? st->prefix : kCalibInf;   // no threshold reaches the target: +inf
    unsigned mine = 0u;
    for (long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += static_cast<long>(gridDim.x) * blockDim.x)
        mine += (keys[i] <= key) ? 1u : 0u;
    if (mine) atomicAdd(&c, mine);
    __syncthreads();
    if (threadIdx.x == 0 && c) atomicAdd(&st->count_le, c);
}
__global__ void calib_result(const CalibState* st, long n, float* T_out, float* fraction_out) {
    *T_out = __uint_as_float(st->prefix < kCalibInf ? st->prefix : kCalibInf);
    if (fraction_out) *fraction_out = static_cast<float>(static_cast<double>(st->count_le) / static_cast<double>(n));
}

// ------------------------------------------------------------------------------------------
// host side: planning, workspace, launches

struct Plan {
    int VE, NV, G, spm, GS, sps;   // G = wavefronts per pair
    long nslots;
    size_t off_counters, n_counters, off_part1, off_part2, off_wz, zero_bytes, off_div, off_pst, off_lse2, off_lr, off_spart,
        off_thr, off_tsd, off_tsdz, bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kMaxTeam = 256;     // wavefronts per pair (merged in rounds of 64)
int g_shape_nv = 0;               // 0 = chosen by make_plan (see fsd_debug_set_shape)

// wavefronts per pair when every lane holds nv slots of each row: whole workgroups
long team_size(long nslots, int nv) {
    const long per_wave = 64L * nv;
    const long G = (nslots + per_wave - 1) / per_wave;
    return (G + 3) / 4 * 4;
}

bool make_plan(int B, int rows, long V, int dtype, Plan& p) {
    if (B < 1 || B > 65535 || rows < 1 || rows > kMaxRows || V < 1) return false;
    if (dtype != FSD_F32 && dtype != FSD_BF16) return false;
    if (static_cast<long>(B) * rows >= (1L << 24)) return false;
    if (V > fsd_max_vocab(dtype)) return false;
    p.VE = (dtype == FSD_BF16) ? 8 : 4;
    p.nslots = (V + p.VE - 1) / p.VE;
    // 32 vocabulary entries of each row per lane: 4 slots of bfloat16, 8 of binary32
    p.NV = (dtype == FSD_BF16) ? 4 : 8;
    if (g_shape_nv && !(dtype == FSD_BF16 && g_shape_nv > 5) && team_size(p.nslots, g_shape_nv) <= kMaxTeam) p.NV = g_shape_nv;
    const long G = team_size(p.nslots, p.NV);
    if (G > kMaxTeam) return false;
    p.G = static_cast<int>(G);
    p.spm = static_cast<int>((p.nslots + G - 1) / G);
    long GS = (1024 + B - 1) / B;
    const long maxgs = (p.nslots + kWG - 1) / kWG;
    if (GS > maxgs) GS = maxgs;
    if (GS > 64) GS = 64;
    if (GS < 1) GS = 1;
    p.GS = static_cast<int>(GS);
    p.sps = static_cast<int>((p.nslots + GS - 1) / GS);
    const size_t R = static_cast<size_t>(B) * rows;
    size_t o = 0;
    p.off_counters = o; p.n_counters = 64 + B; o = align_up(o + p.n_counters * 4, 256);
    p.off_part1 = o; o = align_up(o + R * p.G * 32, 256);
    p.off_part2 = o; o = align_up(o + R * p.G * 32, 256);
    p.off_wz = o; o = align_up(o + R * kWalkShare * 8, 256);
    p.zero_bytes = o;
    p.off_div = o; o = align_up(o + R * 4, 256);
    p.off_pst = o; o = align_up(o + R * 4, 256);
    p.off_lse2 = o; o = align_up(o + R * 16, 256);
    p.off_lr = o; o = align_up(o + R * 8, 256);
    p.off_spart = o; o = align_up(o + static_cast<size_t>(B) * p.GS * 32, 256);
    p.off_thr = o; o = align_up(o + static_cast<size_t>(B) * 4, 256);
    p.off_tsd = o; o = align_up(o + static_cast<size_t>(B) * (4 + rows) * 4, 256);
    p.off_tsdz = o; o = align_up(o + static_cast<size_t>(B) * rows * 4, 256);
    p.bytes = o;
    return true;
}

Ws carve(void* workspace, const Plan& p, int B, int rows) {
    char* base = static_cast<char*>(workspace);
    const size_t R = static_cast<size_t>(B) * rows;
    Ws w;
    w.counters = reinterpret_cast<unsigned*>(base + p.off_counters);
    w.sdone = w.counters + 64;
    w.part1 = reinterpret_cast<unsigned long long*>(base + p.off_part1);
    w.part2 = reinterpret_cast<double*>(base + p.off_part2);
    w.div = reinterpret_cast<float*>(base + p.off_div);
    w.pst = reinterpret_cast<int*>(base + p.off_pst);
    w.lse2 = reinterpret_cast<double*>(base + p.off_lse2);
    w.lr = reinterpret_cast<double*>(base + p.off_lr);
    w.spart = reinterpret_cast<unsigned long long*>(base + p.off_spart);
    w.thr = reinterpret_cast<float*>(base + p.off_thr);
    w.tsd = reinterpret_cast<int*>(base + p.off_tsd);
    w.tsd_invz = reinterpret_cast<float*>(base + p.off_tsdz);
    w.wz = reinterpret_cast<unsigned long long*>(base + p.off_wz);
    return w;
}

unsigned g_spin_limit = 1u << 22;
#ifdef FSD_PHASE_TIMING
unsigned long long* g_dbg = nullptr;
#endif

// ---- optional event timing of pair_kernel
constexpr int kMaxProf = 4096;
bool g_prof_on = false;
int g_prof_n = 0;
hipEvent_t g_prof_ev[2 * kMaxProf];
bool g_prof_made = false;

// How many workgroups of a kernel are resident at once on the current device, and how much unused
// dynamic LDS to ask for so that the hardware cannot place more than that number on any one CU.
// Without the padding a grid that does not fill every slot may be spread unevenly (some CUs full,
// others half empty), and the team members that share a pair then all run at the pace of the most
// crowded CU.  The padding leaves 8 KB of slack so that it can only lower the count it is checked
// against, never the number of workgroups that really fit.
struct Residency { int total; unsigned pad_lds; };

int g_last_grid = 0, g_last_total = 0;

template <typename Kernel>
Residency residency_of(Kernel kernel, int threads, Residency (&cache)[16]) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 16) dev = 0;
    if (cache[dev].total == 0) {
        int per_cu = 0, cus = 0, lds_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess) per_cu = 1;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 64;
        if (hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess) lds_cu = 0;
        if (per_cu < 1) per_cu = 1;
        if (cus < 1) cus = 1;
        unsigned pad = 0;
        hipFuncAttributes attr;
        if (lds_cu > 16384 && hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(kernel)) == hipSuccess) {
            const long stat = static_cast<long>(attr.sharedSizeBytes);
            const long want = ((static_cast<long>(lds_cu) - 8192) / per_cu - stat) / 1024 * 1024;
            if (want > 0 && (stat + want) * (per_cu + 1) > lds_cu) {
                bool ok = true;
                if (stat + want > 65536)
                    ok = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>(want)) == hipSuccess;
                int check = 0;
                if (ok && hipOccupancyMaxActiveBlocksPerMultiprocessor(&check, kernel, threads, static_cast<size_t>(want)) == hipSuccess &&
                    check == per_cu)
                    pad = static_cast<unsigned>(want);
            }
        }
        (void)hipGetLastError();
        cache[dev] = Residency{per_cu * cus, pad};
    }
    g_last_total = cache[dev].total;
    return cache[dev];
}

template <bool BF16, int NV, int MODE, bool ALIGNED>
void launch_pair_k(hipStream_t st, const PairParams& P) {
    // persistent grid: whole teams only, never more than fits on the device at once
    static Residency cache[16] = {};
    const Residency res = residency_of(pair_kernel<BF16, NV, MODE, ALIGNED>, kWG, cache);
    const long wgs_per_team = P.G / (kWG / 64);
    const long want = static_cast<long>(P.npairs) * wgs_per_team;
    long cap = res.total / wgs_per_team * wgs_per_team;
    if (cap < wgs_per_team) cap = wgs_per_team;
    const long grid = want < cap ? want : cap;
    g_last_grid = static_cast<int>(grid);
    hipLaunchKernelGGL((pair_kernel<BF16, NV, MODE, ALIGNED>), dim3(static_cast<unsigned>(grid)), dim3(kWG), res.pad_lds, st, P);
}
template <bool BF16, int NV, int MODE>
void launch_pair_a(bool aligned, hipStream_t st, const PairParams& P) {
    if (aligned) launch_pair_k<BF16, NV, MODE, true>(st, P);
    else launch_pair_k<BF16, NV, MODE, false>(st, P);
}
template <bool BF16, int NV>
void launch_pair_m(int mode, bool aligned, hipStream_t st, const PairParams& P) {
    switch (mode) {
        case MODE_KL: launch_pair_a<BF16, NV, MODE_KL>(aligned, st, P); break;
        case MODE_JS: launch_pair_a<BF16, NV, MODE_JS>(aligned, st, P); break;
        case MODE_TV: launch_pair_a<BF16, NV, MODE_TV>(aligned, st, P); break;
        case MODE_KLP: launch_pair_a<BF16, NV, MODE_KLP>(aligned, st, P); break;
        default: launch_pair_a<BF16, NV, MODE_LSE>(aligned, st, P); break;
    }
}
void launch_pair(int dtype, int NV, int mode, bool aligned, hipStream_t st, const PairParams& P) {
    const bool prof = g_prof_on && g_prof_n < kMaxProf;
    if (prof) {
        if (!g_prof_made) {
            for (int i = 0; i < 2 * kMaxProf; ++i) (void)hipEventCreate(&g_prof_ev[i]);
            g_prof_made = true;
        }
        (void)hipEventRecord(g_prof_ev[2 * g_prof_n], st);
    }
    if (dtype == FSD_BF16) {
        if (NV == 2) launch_pair_m<true, 2>(mode, aligned, st, P);
        else if (NV == 5) launch_pair_m<true, 5>(mode, aligned, st, P);
        else launch_pair_m<true, 4>(mode, aligned, st, P);
    } else {
        if (NV == 2) launch_pair_m<false, 2>(mode, aligned, st, P);
        else if (NV == 4) launch_pair_m<false, 4>(mode, aligned, st, P);
        else launch_pair_m<false, 8>(mode, aligned, st, P);
    }
    if (prof) {
        (void)hipEventRecord(g_prof_ev[2 * g_prof_n + 1], st);
        ++g_prof_n;
    }
}

template <bool BF16, bool ALIGNED>
void launch_sample_k(int kind, dim3 grid, size_t lds, hipStream_t st, const SampleParams& P) {
    switch (kind) {
        case KIND_CHAIN: hipLaunchKernelGGL((accept_sample<BF16, ALIGNED, KIND_CHAIN>), grid, dim3(kWG), lds, st, P); break;
        case KIND_TREE: hipLaunchKernelGGL((accept_sample<BF16, ALIGNED, KIND_TREE>), grid, dim3(kWG), lds, st, P); break;
        case KIND_RFSD: hipLaunchKernelGGL((accept_sample<BF16, ALIGNED, KIND_RFSD>), grid, dim3(kWG), lds, st, P); break;
        case KIND_TREESD: hipLaunchKernelGGL((accept_sample<BF16, ALIGNED, KIND_TREESD>), grid, dim3(kWG), lds, st, P); break;
        default: hipLaunchKernelGGL((accept_sample<BF16, ALIGNED, KIND_SD>), grid, dim3(kWG), lds, st, P); break;
    }
}
void launch_sample(int dtype, bool aligned, int kind, dim3 grid, size_t lds, hipStream_t st, const SampleParams& P) {
    if (dtype == FSD_BF16) {
        if (aligned) launch_sample_k<true, true>(kind, grid, lds, st, P);
        else launch_sample_k<true, false>(kind, grid, lds, st, P);
    } else {
        if (aligned) launch_sample_k<false, true>(kind, grid, lds, st, P);
        else launch_sample_k<false, false>(kind, grid, lds, st, P);
    }
}

// The workgroups that share a sequence wait for each other, so the whole grid has to be resident:
// as many per sequence as fit (at most kWalkShare, and no more than there are passes' worth of
// slots), a single one otherwise.
template <typename Kernel>
void launch_walk(Kernel kernel, int B, long nslots, size_t lds, hipStream_t st, const WalkParams& P) {
    int dev = 0, per_cu = 0, cus = 0;
    (void)hipGetDevice(&dev);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kWalkWG, lds) != hipSuccess) per_cu = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    (void)hipGetLastError();
    long gsw = (static_cast<long>(per_cu) * cus) / B;
    if (gsw > kWalkShare) gsw = kWalkShare;
    const long by_work = (nslots + kWalkWG - 1) / kWalkWG;
    if (gsw > by_work) gsw = by_work;
    if (gsw < 1) gsw = 1;
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(gsw), static_cast<unsigned>(B)), dim3(kWalkWG), lds, st, P);
}

bool is_aligned(const void* a, const void* b, long V, int VE) {
    return (V % VE == 0) && (reinterpret_cast<uintptr_t>(a) % 16 == 0) &&
           (b == nullptr || reinterpret_cast<uintptr_t>(b) % 16 == 0);
}

// the common body of the three entry points
int run(int kind, const void* target, const void* draft, const int32_t* tokens, const int32_t* parent, int B,
        int rows, int max_depth, int V, int dtype, int div, float T, int mode, uint64_t seed, uint64_t offset,
        int32_t* out_len, int32_t* path_nodes, int32_t* out_tokens, float* user_vals, float* user_ratio,
        int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream,
        float temperature = 1.0f, int top_k = 0, float top_p = 1.0f) {
    if (!target || !draft || !tokens || !out_len || !out_tokens) return FSD_ERR_NULL;
    const bool tree = (kind == KIND_TREE || kind == KIND_TREESD);
    if (tree && (!parent || !path_nodes)) return FSD_ERR_NULL;
    if (dtype != FSD_F32 && dtype != FSD_BF16) return FSD_ERR_DTYPE;
    if (kind != KIND_SD && kind != KIND_TREESD && (div < FSD_DIV_KL || div > FSD_DIV_TV)) return FSD_ERR_DIV;
    if (mode != FSD_SAMPLE && mode != FSD_GREEDY) return FSD_ERR_MODE;
    if (T != T) return FSD_ERR_SHAPE;
    if (tree && (max_depth < 1 || max_depth > kMaxRows)) return FSD_ERR_SHAPE;
    if (!(temperature >= 1e-3f && temperature <= 1e3f) || top_k < 0 || !(top_p > 0.0f && top_p <= 1.0f)) return FSD_ERR_SHAPE;
    Plan p;
    if (!make_plan(B, rows, V, dtype, p)) return FSD_ERR_SHAPE;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || workspace_bytes < p.bytes)
        return FSD_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Ws ws = carve(workspace, p, B, rows);
    const bool aligned = is_aligned(target, draft, V, p.VE);
    const int R = B * rows;

    const long n16 = static_cast<long>(p.zero_bytes / 16);
    hipLaunchKernelGGL(zero_counters, dim3(static_cast<unsigned>((n16 + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<uint4*>(ws.counters), n16);

    PairParams pp;
    pp.target = static_cast<const char*>(target);
    pp.draft = static_cast<const char*>(draft);
    pp.parent = tree ? parent : nullptr;
    pp.cand = tokens;
    pp.rows = rows;
    pp.npairs = R;
    pp.V = V;
    pp.nslots = p.nslots;
    pp.spm = p.spm;
    pp.G = p.G;
    pp.spin_limit = g_spin_limit;
#ifdef FSD_PHASE_TIMING
    pp.dbg = g_dbg;
#endif
    pp.user_div = user_vals;
    pp.user_ratio = user_ratio;
    pp.want_ratio = (kind == KIND_RFSD) ? 1 : 0;
    pp.ws = ws;
    int k1mode = (kind == KIND_SD || kind == KIND_TREESD) ? MODE_LSE : div;
    if (k1mode == MODE_KL && dtype == FSD_F32) k1mode = MODE_KLP;
    if (dtype == FSD_BF16 && !g_shape_nv && (k1mode == MODE_JS || k1mode == MODE_TV)) {
        // The bfloat16 two-phase kernels are bound by instruction issue, a third of it per step and not
        // per entry: 5 slots per lane instead of 4 is the most that fits two wavefronts per SIMD (256
        // registers).  The workspace is laid out for the larger team of the 4-slot shape.
        p.NV = 5;
        p.G = static_cast<int>(team_size(p.nslots, 5));
        p.spm = static_cast<int>((p.nslots + p.G - 1) / p.G);
        pp.spm = p.spm;
        pp.G = p.G;
    }
    launch_pair(dtype, p.NV, k1mode, aligned, st, pp);

    SampleParams sp;
    sp.target = static_cast<const char*>(target);
    sp.draft = static_cast<const char*>(draft);
    sp.tokens = tokens;
    sp.parent = parent;
    sp.rows = rows;
    sp.max_depth = max_depth;
    sp.V = V;
    sp.nslots = p.nslots;
    sp.sps = p.sps;
    sp.GS = p.GS;
    sp.T = T;
    sp.mode = mode;
    sp.seed_lo = static_cast<unsigned>(seed);
    sp.seed_hi = static_cast<unsigned>(seed >> 32);
    sp.off_lo = static_cast<unsigned>(offset);
    sp.off_hi = static_cast<unsigned>(offset >> 32);
    sp.out_len = out_len;
    sp.out_tokens = out_tokens;
    sp.path_nodes = path_nodes;
    sp.row_status = row_status;
    sp.ws = ws;
    sp.thr = nullptr;
    sp.inv_temp = 1.0f;
    const bool warped = (temperature != 1.0f) || (top_k > 0 && top_k < V) || (top_p < 1.0f);
    if (warped && mode == FSD_SAMPLE) {
        // warpers: one more kernel finds, per sequence, the smallest kept scaled logit
        WarpParams wp;
        wp.target = static_cast<const char*>(target);
        wp.rows = rows;
        wp.V = V;
        wp.nslots = p.nslots;
        wp.T = T;
        wp.inv_temp = static_cast<float>(1.0 / static_cast<double>(temperature));
        wp.top_k = top_k;
        wp.top_p = top_p;
        wp.thr = ws.thr;
        wp.ws = ws;
        const bool keep = dtype == FSD_BF16 && aligned && p.nslots <= static_cast<long>(kWarpKeep) * kWarpWG;
        if (dtype == FSD_BF16) {
            if (keep) hipLaunchKernelGGL((warp_select<true, true, true>), dim3(B), dim3(kWarpWG), 0, st, wp);
            else if (aligned) hipLaunchKernelGGL((warp_select<true, true, false>), dim3(B), dim3(kWarpWG), 0, st, wp);
            else hipLaunchKernelGGL((warp_select<true, false, false>), dim3(B), dim3(kWarpWG), 0, st, wp);
        } else {
            if (aligned) hipLaunchKernelGGL((warp_select<false, true, false>), dim3(B), dim3(kWarpWG), 0, st, wp);
            else hipLaunchKernelGGL((warp_select<false, false, false>), dim3(B), dim3(kWarpWG), 0, st, wp);
        }
        sp.thr = ws.thr;
        sp.inv_temp = wp.inv_temp;
    }
    if (kind == KIND_TREESD) {
        // strict SD on a tree: one workgroup per sequence walks the tree before the token is drawn
        WalkParams wk;
        wk.target = sp.target;
        wk.draft = sp.draft;
        wk.tokens = tokens;
        wk.parent = parent;
        wk.rows = rows;
        wk.max_depth = max_depth;
        wk.V = V;
        wk.nslots = p.nslots;
        wk.seed_lo = sp.seed_lo; wk.seed_hi = sp.seed_hi; wk.off_lo = sp.off_lo; wk.off_hi = sp.off_hi;
        wk.path_nodes = path_nodes;
        wk.out_tokens = out_tokens;
        wk.user_ratio = user_ratio;
        wk.ws = ws;
        wk.spin_limit = g_spin_limit;
        const size_t wlds = static_cast<size_t>(rows) * 24 + 16;
        if (dtype == FSD_BF16) {
            if (aligned) launch_walk(tree_sd_walk<true, true>, B, p.nslots, wlds, st, wk);
            else launch_walk(tree_sd_walk<true, false>, B, p.nslots, wlds, st, wk);
        } else {
            if (aligned) launch_walk(tree_sd_walk<false, true>, B, p.nslots, wlds, st, wk);
            else launch_walk(tree_sd_walk<false, false>, B, p.nslots, wlds, st, wk);
        }
    }
    const size_t lds = (kind == KIND_TREE) ? static_cast<size_t>(rows) * 16
                     : (kind == KIND_TREESD) ? static_cast<size_t>(rows) * 12 : 0;
    launch_sample(dtype, aligned, kind, dim3(p.GS, B), lds, st, sp);

    return (hipGetLastError() == hipSuccess) ? FSD_OK : FSD_ERR_LAUNCH;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// C ABI

extern "C" {

int64_t fsd_max_vocab(int dtype) {
    // 256 wavefronts per pair, 64 lanes, 32 entries of each row per lane
    if (dtype == FSD_BF16 || dtype == FSD_F32) return static_cast<int64_t>(kMaxTeam) * 64 * 32;
    return 0;
}

size_t fsd_workspace_bytes(int B, int rows_per_seq, int V, int dtype) {
    Plan p;
    if (!make_plan(B, rows_per_seq, V, dtype, p)) return 0;
    return p.bytes;
}

size_t fsd_calibrate_workspace_bytes(int B, int K) {
    if (B < 1 || K < 1 || K > kMaxRows || static_cast<long>(B) * K >= (1L << 24)) return 0;
    return align_up(sizeof(CalibState), 256) + align_up(static_cast<size_t>(B) * K * 4, 256);
}

int fsd_calibrate_threshold(const float* divergences, int B, int K, float target_fraction, float* T_out,
                            float* fraction_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!divergences || !T_out) return FSD_ERR_NULL;
    const size_t need = fsd_calibrate_workspace_bytes(B, K);
    if (need == 0 || !(target_fraction > 0.0f) || !(target_fraction <= 1.0f)) return FSD_ERR_SHAPE;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || workspace_bytes < need) return FSD_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    CalibState* state = static_cast<CalibState*>(workspace);
    unsigned* keys = reinterpret_cast<unsigned*>(static_cast<char*>(workspace) + align_up(sizeof(CalibState), 256));
    const long n = static_cast<long>(B) * K;
    // rank = ceil(fraction n), in exact arithmetic on the binary32 fraction
    const double want = static_cast<double>(target_fraction) * static_cast<double>(n);
    long rank = static_cast<long>(want);
    if (static_cast<double>(rank) < want) ++rank;
    if (rank < 1) rank = 1;
    if (rank > n) rank = n;
    const unsigned blocks = static_cast<unsigned>(n / 4096 + 1 > 1024 ? 1024 : n / 4096 + 1);
    hipLaunchKernelGGL(calib_keys, dim3((B + 255) / 256), dim3(256), 0, st, divergences, B, K, keys);
    hipLaunchKernelGGL(calib_init, dim3(1), dim3(256), 0, st, state, static_cast<unsigned>(rank));
    for (int shift = 24; shift >= 0; shift -= 8) {
        hipLaunchKernelGGL(calib_hist, dim3(blocks), dim3(256), 0, st, keys, n, shift, state);
        hipLaunchKernelGGL(calib_pick, dim3(1), dim3(256), 0, st, state, shift);
    }
    hipLaunchKernelGGL(calib_count, dim3(blocks), dim3(256), 0, st, keys, n, state);
    hipLaunchKernelGGL(calib_result, dim3(1), dim3(1), 0, st, state, n, T_out, fraction_out);
    return (hipGetLastError() == hipSuccess) ? FSD_OK : FSD_ERR_LAUNCH;
}

const char* fsd_status_string(int status) {
    switch (status) {
        case FSD_OK: return "ok";
        case FSD_ERR_NULL: return "a required pointer is NULL";
        case FSD_ERR_SHAPE: return "size out of range or T is NaN";
        case FSD_ERR_DTYPE: return "unknown dtype";
        case FSD_ERR_DIV: return "unknown divergence";
        case FSD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case FSD_ERR_MODE: return "unknown sampling mode";
        case FSD_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int fsd_verify_chain(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens, int B, int K,
                     int V, int dtype, int div, float T, int mode, uint64_t seed, uint64_t offset,
                     int32_t* accept_len, int32_t* out_tokens, float* divergences, int32_t* row_status,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(KIND_CHAIN, target_logits, draft_logits, cand_tokens, nullptr, B, K, 0, V, dtype, div, T, mode, seed,
               offset, accept_len, nullptr, out_tokens, divergences, nullptr, row_status, workspace, workspace_bytes,
               hip_stream);
}

int fsd_verify_tree(const void* target_logits, const void* draft_logits, const int32_t* node_tokens,
                    const int32_t* parent, int B, int N, int max_depth, int V, int dtype, int div, float T,
                    int mode, uint64_t seed, uint64_t offset, int32_t* path_len, int32_t* path_nodes,
                    int32_t* out_tokens, float* divergences, int32_t* row_status, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    return run(KIND_TREE, target_logits, draft_logits, node_tokens, parent, B, N, max_depth, V, dtype, div, T, mode,
               seed, offset, path_len, path_nodes, out_tokens, divergences, nullptr, row_status, workspace,
               workspace_bytes, hip_stream);
}

int sd_verify_chain(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens, int B, int K,
                    int V, int dtype, int mode, uint64_t seed, uint64_t offset, int32_t* accept_len,
                    int32_t* out_tokens, float* log_ratio, int32_t* row_status, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    return run(KIND_SD, target_logits, draft_logits, cand_tokens, nullptr, B, K, 0, V, dtype, FSD_DIV_KL, 0.0f, mode,
               seed, offset, accept_len, nullptr, out_tokens, log_ratio, nullptr, row_status, workspace, workspace_bytes,
               hip_stream);
}

int fsd_verify_chain_warped(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens, int B,
                            int K, int V, int dtype, int div, float T, int mode, uint64_t seed, uint64_t offset,
                            float temperature, int top_k, float top_p, int32_t* accept_len, int32_t* out_tokens,
                            float* divergences, int32_t* row_status, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    return run(KIND_CHAIN, target_logits, draft_logits, cand_tokens, nullptr, B, K, 0, V, dtype, div, T, mode, seed,
               offset, accept_len, nullptr, out_tokens, divergences, nullptr, row_status, workspace, workspace_bytes,
               hip_stream, temperature, top_k, top_p);
}

int sd_verify_tree(const void* target_logits, const void* draft_logits, const int32_t* node_tokens,
                   const int32_t* parent, int B, int N, int max_depth, int V, int dtype, int mode, uint64_t seed,
                   uint64_t offset, int32_t* path_len, int32_t* path_nodes, int32_t* out_tokens, float* log_ratio,
                   int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(KIND_TREESD, target_logits, draft_logits, node_tokens, parent, B, N, max_depth, V, dtype, FSD_DIV_KL,
               0.0f, mode, seed, offset, path_len, path_nodes, out_tokens, nullptr, log_ratio, row_status, workspace,
               workspace_bytes, hip_stream);
}

int rfsd_verify_chain(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens, int B, int K,
                      int V, int dtype, int div, float T, int mode, uint64_t seed, uint64_t offset,
                      int32_t* accept_len, int32_t* out_tokens, float* divergences, float* log_ratio,
                      int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(KIND_RFSD, target_logits, draft_logits, cand_tokens, nullptr, B, K, 0, V, dtype, div, T, mode, seed,
               offset, accept_len, nullptr, out_tokens, divergences, log_ratio, row_status, workspace,
               workspace_bytes, hip_stream);
}

int fsd_profile_enable(int on) {
    g_prof_on = (on != 0);
    return FSD_OK;
}

int fsd_profile_collect(float* mean_ms, float* min_ms) {
    const int n = g_prof_n;
    double sum = 0.0;
    float mn = 0.0f;
    for (int i = 0; i < n; ++i) {
        (void)hipEventSynchronize(g_prof_ev[2 * i + 1]);
        float ms = 0.0f;
        (void)hipEventElapsedTime(&ms, g_prof_ev[2 * i], g_prof_ev[2 * i + 1]);
        sum += ms;
        if (i == 0 || ms < mn) mn = ms;
    }
    if (mean_ms) *mean_ms = n ? static_cast<float>(sum / n) : 0.0f;
    if (min_ms) *min_ms = mn;
    g_prof_n = 0;
    return n;
}

int fsd_debug_set_shape(int wavefronts, int slots_per_thread) {
    const bool ok = (wavefronts == 0 || wavefronts == 4) &&
                    (slots_per_thread == 0 || slots_per_thread == 2 || slots_per_thread == 4 || slots_per_thread == 5 ||
                     slots_per_thread == 8);
    if (!ok) return FSD_ERR_SHAPE;
    g_shape_nv = slots_per_thread;
    return FSD_OK;
}

size_t fsd_debug_warp_threshold_offset(int B, int rows_per_seq, int V, int dtype) {
    Plan p;
    if (!make_plan(B, rows_per_seq, V, dtype, p)) return 0;
    return p.off_thr;
}

void fsd_debug_last_launch(int* grid, int* resident) {
    if (grid) *grid = g_last_grid;
    if (resident) *resident = g_last_total;
}

unsigned fsd_debug_set_spin_limit(unsigned polls) {
    const unsigned prev = g_spin_limit;
    g_spin_limit = polls;
    return prev;
}

#ifdef FSD_PHASE_TIMING
void fsd_debug_set_dbg(void* p) { g_dbg = static_cast<unsigned long long*>(p); }
#endif

}  // extern "C"
