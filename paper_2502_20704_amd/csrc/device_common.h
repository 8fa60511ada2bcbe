// Device helpers shared by every kernel of libfsd: constants, wavefront reductions, slot loads,
// Philox4x32-10 and the exact-operation logarithm, the workspace view, the clearing kernel.
// Part of libfsd (gfx950); included by fsd_kernels.hip, which holds the host side and the C ABI.
#ifndef FSD_CSRC_DEVICE_COMMON_H_
#define FSD_CSRC_DEVICE_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <float.h>
#include <math.h>

#include "fsd.h"

namespace {

constexpr int kWG = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int kMaxRows = 2048;    // K or N
constexpr int kSampleWGs = 1024;  // sampler workgroups aimed at per call (all sequences together): more cost
                                  // more in launch and posting than their parallelism returns
constexpr int kSdoneStride = 64;  // 32-bit words between the sampler's per-sequence counters: one 256-byte
                                  // line each, so that the counting atomics of different sequences do not
                                  // queue at one memory channel
constexpr int kWalkShare = 8;     // workgroups that share a sequence's passes in the tree walk (at most)
constexpr float kLog2e = 1.44269504088896340736f;
constexpr double kLn2 = 0.69314718055994530942;
constexpr double kLog2eD = 1.44269504088896340736;

// MODE_KL: single-pass KL (absolute error ~1e-7, enough for bfloat16 inputs); MODE_KLP: two-phase,
// pointwise non-negative KL for binary32 inputs; MODE_LSE: normalisers only (strict SD); MODE_JSE: JS in
// entropy form for bfloat16 inputs (one logarithm per entry; small results are evaluated again pointwise)
enum { MODE_KL = 0, MODE_JS = 1, MODE_TV = 2, MODE_LSE = 3, MODE_KLP = 4, MODE_JSE = 5 };
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
// Two reductions at once, interleaved: each one's step sits in the other's wait states.  Every value
// goes through the same operations in the same order as in the single forms: identical results.
__device__ __forceinline__ void wave_max2(float& a, float& b) {
    asm("s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 0"
        : "+v"(a), "+v"(b));
    a = lane_f(a, 63);
    b = lane_f(b, 63);
}
__device__ __forceinline__ void wave_sumf2(float& a, float& b) {
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_add_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_add_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_add_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 0"
        : "+v"(a), "+v"(b));
    a = lane_f(a, 63);
    b = lane_f(b, 63);
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
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <bool BF16, bool ALIGNED, bool STREAM = false>
__device__ __forceinline__ uint4 load_slot(const char* row, long slot, long V) {
    if constexpr (ALIGNED) {
        // a 32-bit offset from the row (rows are at most 2 MiB): the row pointer stays scalar
        const char* at = row + static_cast<size_t>(static_cast<unsigned>(slot) * 16u);
        if constexpr (STREAM) {
            // read once by this kernel: marked non-temporal
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(at));
            return make_uint4(v.x, v.y, v.z, v.w);
        } else {
            return *reinterpret_cast<const uint4*>(at);
        }
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
        // a three-input bitwise operation with the truth table of a ^ b ^ c (0x96): one instruction
        const unsigned n0 = __builtin_amdgcn_bitop3_b32(hi1, c1, k0, 0x96);
        const unsigned n2 = __builtin_amdgcn_bitop3_b32(hi0, c3, k1, 0x96);
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
    unsigned* counters;  // 64 words (words 2-3: the failure word, see flag_failure; word 4: sequences the sampler has finished), then sdone
    unsigned* sdone;     // [B][kSdoneStride], first word: sampler workgroups that posted
    unsigned long long* part1;  // [R][G][n1] phase-1 words, dense: (kt,kd) | (St,Sd) in the two-phase modes (n1 = 2),
                                // (kt,kd) | St | Sd | W in the single-pass ones (n1 = 4)
    double* part2;       // [R][G][n2] divergence words of the two-phase modes (n2 = 1, or 2 for TV and pointwise KL)
    unsigned long long* state;  // [R] entropy-form JS: 0 = pair not finished yet, all ones = done, else the rows'
                                // log2-sum-exp2 (two binary32) of a pair the team evaluates again pointwise
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
    unsigned long long* arrive; // [kMaxArrive] a call without a clearing kernel: wavefront i of the reduction kernel
                                // writes the call's number here once it has cleared its words (never cleared
                                // by a kernel before the reduction: only a word equal to the number counts)
    unsigned long long nonce;   // the call's number: never 0, different for every call of the process
};

constexpr int kMaxArrive = 16384;   // wavefronts of a reduction grid that can announce themselves

// "A bounded wait expired somewhere in this call": the failure word holds the call's own number.
// Whatever else it holds (zero, an earlier call's number, what the memory held before) says nothing,
// so the word needs no clearing and a flag raised early cannot be lost to a late clear.
__device__ __forceinline__ void flag_failure(const Ws& w) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(w.counters + 2), w.nonce, __ATOMIC_RELAXED, AGENT);
}
__device__ __forceinline__ bool failure_flagged(const Ws& w) {
    return __hip_atomic_load(reinterpret_cast<const unsigned long long*>(w.counters + 2), __ATOMIC_RELAXED, AGENT) == w.nonce;
}

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
    int nteams;             // teams of G consecutive wavefronts in the grid (set by the launch)
    unsigned spin_limit;
#ifdef FSD_PHASE_TIMING
    unsigned long long* dbg;   // [grid][4 wavefronts][10]
#endif
    float* user_div;        // optional [R]
    float* user_ratio;      // optional [R], reducible FSD only
    int want_ratio;         // 1: the finisher also writes ln p(x) - ln q(x) at the candidate token (reducible FSD)
    float js_floor;         // entropy-form JS: results below this (nats) are evaluated again in the pointwise form
    // A call without a clearing kernel of its own (see the start of pair_kernel): the wavefronts clear
    // what they and the sampler need, [clear_a, +clear_a16) and [clear_b, +clear_b16) in 16-byte units
    // being the parts no team owns.  0: a kernel before this one has cleared everything.
    int self_clear;
    uint4* clear_a;
    long clear_a16;
    uint4* clear_b;
    long clear_b16;
    Ws ws;
};

// ------------------------------------------------------------------------------------------
// kernel 0: clear the counters and the exchange words (a zero word means "not posted yet")

__global__ void zero_counters(uint4* p, long n16) {
    const long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace

#endif  // FSD_CSRC_DEVICE_COMMON_H_
