// The walk of strict SD over a token tree.
// Part of libfsd (gfx950); included by fsd_kernels.hip, which holds the host side and the C ABI.
#ifndef FSD_CSRC_TREE_SD_WALK_H_
#define FSD_CSRC_TREE_SD_WALK_H_

#include "device_common.h"
#include "accept_sample.h"

namespace {

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
    if (failure_flagged(P.ws)) status |= FSD_ROW_INTERNAL;
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
            // p and q of an entry: 2^(z log2e - lse2) with the argument formed in float64 and split into a
            // binary32 part for the hardware exponential and a remainder applied as 1 + ln2 * rest.  A
            // binary32 argument would carry the rounding of lse2 (about 1e-6 at |lse2| = 20) into every
            // entry of the row alike, and a later sibling's log-ratio multiplies such a common error by
            // p/(p - q); this way only the exponential's own rounding is left, which averages out in the sums.
            auto prob = [&](float z, double lse2) __attribute__((always_inline)) -> float {
                const double x = fma(static_cast<double>(z), kLog2eD, -lse2);
                const float xh = static_cast<float>(x);
                const float xl = static_cast<float>(x - static_cast<double>(xh));
                return hw_exp2(xh) * fmaf(xl, static_cast<float>(kLn2), 1.0f);
            };
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
                    for (int e = 0; e < VE; ++e) pv[c][e] = in[c] ? prob(z[e], lt2) : 0.0f;
                }
                for (int m = 0; m < nrej; ++m) {
                    const size_t pc = static_cast<size_t>(b) * N + chain[m];
                    const char* cr = P.draft + pc * rowb;
#pragma unroll
                    for (int c = 0; c < CH; ++c) raw[c] = load_slot<BF16, ALIGNED>(cr, slc[c], P.V);
                    const double ldm = lse_of[2 * chain[m] + 1];
                    const float izm = s_invz[m];
#pragma unroll
                    for (int c = 0; c < CH; ++c) {
                        float zd[VE];
                        unpack<BF16>(raw[c], zd);
#pragma unroll
                        for (int e = 0; e < VE; ++e)
                            pv[c][e] = fmaxf(pv[c][e] - prob(zd[e], ldm), 0.0f) * izm;
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
                    for (int e = 0; e < VE; ++e) part += fmaxf(pv[c][e] - prob(zd[e], ld2), 0.0f);
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
                    if (tid == 0) flag_failure(P.ws);
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

}  // namespace

#endif  // FSD_CSRC_TREE_SD_WALK_H_
