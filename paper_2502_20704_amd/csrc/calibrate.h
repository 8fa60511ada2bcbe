// Threshold tuning on a dev set: an exact order statistic of the running maxima.
// Part of libfsd (gfx950); included by fsd_kernels.hip, which holds the host side and the C ABI.
#ifndef FSD_CSRC_CALIBRATE_H_
#define FSD_CSRC_CALIBRATE_H_

#include "device_common.h"

namespace {

// ------------------------------------------------------------------------------------------
// threshold tuning on a dev set (Sec. 6.2, App. A): the smallest occurring T at which the chain rule
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

}  // namespace

#endif  // FSD_CSRC_CALIBRATE_H_
