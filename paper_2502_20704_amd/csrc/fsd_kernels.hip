// Host side and C ABI of libfsd, the FSD candidate-verification step for gfx950 (MI355X).
//
// A verify call launches
//   zero_counters   (device_common.h) clears the counters and exchange words of the call (only where there
//                   are more than 4 MB of them: otherwise the reduction kernel does it itself)
//   pair_kernel     (pair_kernel.h) the vocabulary reduction: one (target row, draft row) pair is
//                   split over a team of G wavefronts; every wavefront loads its slice of both rows
//                   ONCE into registers with 128-bit loads, the team exchanges the softmax
//                   normalisers through 64-bit words in the workspace, and the divergence (paper
//                   App. C.1-C.3) is accumulated from the registers.  One member per pair (they take
//                   turns) adds the team's partial sums in a fixed order: run-to-run identical results.
//   tree_sd_walk    (tree_sd_walk.h) strict SD on a token tree only: the walk over the children
//   warp_select     (warp_select.h) warped calls only: the cut of temperature / top-k / top-p
//   accept_sample   (accept_sample.h) per sequence: the accepted prefix (Sec. 4, eq. 4) or accepted
//                   tree path (Sec. 6.4) or the strict-SD acceptance (Sec. 3, eq. 1-2), then the extra
//                   token by Gumbel-max over the vocabulary of one target row, split over GS workgroups.
// and fsd_calibrate_threshold the kernels of calibrate.h.
//
// Nothing here is shared with the CPU oracle: Philox4x32-10 and the exact-operation logarithm
// are implemented a second time from their published / stated definitions.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <float.h>
#include <math.h>

#include <atomic>
#include <chrono>

#include "fsd.h"

#include "device_common.h"
#include "pair_kernel.h"
#include "accept_sample.h"
#include "tree_sd_walk.h"
#include "warp_select.h"
#include "calibrate.h"

// Workspace of fsd_verify_chain_static, the entry point for callers that cannot allocate: device
// memory that exists from the moment the library is loaded until the process ends, one copy per
// GPU.  Host code never uses this name as an address (on the host it is only a stand-in for the
// symbol): static_scratch() asks the runtime for the array's device address once per device.
static __device__ __align__(256) unsigned char scratch[FSD_STATIC_SCRATCH_BYTES];

namespace {

// ------------------------------------------------------------------------------------------
// host side: planning, workspace, launches

struct Plan {
    int VE, NV, G, spm, GS, sps;   // G = wavefronts per pair
    long nslots;
    size_t off_counters, n_counters, off_state, off_wz, off_part1, off_arrive, zero_bytes, off_div, off_pst, off_lse2, off_lr, off_spart,
        off_thr, off_tsd, off_tsdz, bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kMaxTeam = 256;     // wavefronts per pair (merged in rounds of 64)
int g_shape_nv = 0;               // 0 = chosen by make_plan (see fsd_debug_set_shape)

// wavefronts per pair when every lane holds nv slots of each row.  A team is a run of consecutive
// wavefronts of the grid, not of whole workgroups: at V = 128256 (bfloat16, 5 slots per lane) 51
// members do, 40 teams fit the device instead of the 39 of 52, and 512 pairs take 13 rounds, not 14.
long team_size(long nslots, int nv) {
    const long per_wave = 64L * nv;
    return (nslots + per_wave - 1) / per_wave;
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
    long GS = (kSampleWGs + B - 1) / B;
    const long maxgs = (p.nslots + kWG - 1) / kWG;
    if (GS > maxgs) GS = maxgs;
    if (GS > 64) GS = 64;
    if (GS < 1) GS = 1;
    p.GS = static_cast<int>(GS);
    p.sps = static_cast<int>((p.nslots + GS - 1) / GS);
    const size_t R = static_cast<size_t>(B) * rows;
    size_t o = 0;
    p.off_counters = o; p.n_counters = 64 + static_cast<size_t>(B) * kSdoneStride; o = align_up(o + p.n_counters * 4, 256);
    p.off_state = o; o = align_up(o + R * 8, 256);
    p.off_wz = o; o = align_up(o + R * kWalkShare * 8, 256);
    p.off_spart = o; o = align_up(o + static_cast<size_t>(B) * p.GS * 32, 256);
    // the two exchange arrays, sized for the mode that posts most (4 words per member in each); a call
    // lays them out densely for its own mode (see carve) and clears only that much
    p.off_part1 = o; o = align_up(o + R * p.G * 32, 256) + align_up(R * p.G * 32, 256);
    p.zero_bytes = o;
    p.off_div = o; o = align_up(o + R * 4, 256);
    p.off_pst = o; o = align_up(o + R * 4, 256);
    p.off_lse2 = o; o = align_up(o + R * 16, 256);
    p.off_lr = o; o = align_up(o + R * 8, 256);
    p.off_thr = o; o = align_up(o + static_cast<size_t>(B) * 4, 256);
    p.off_tsd = o; o = align_up(o + static_cast<size_t>(B) * (4 + rows) * 4, 256);
    p.off_tsdz = o; o = align_up(o + static_cast<size_t>(B) * rows * 4, 256);
    p.off_arrive = o; o = align_up(o + static_cast<size_t>(kMaxArrive) * 8, 256);
    p.bytes = o;
    return true;
}

// upper bound of the wavefronts a grid of this device can hold at once (32 per compute unit)
long max_resident_wavefronts() {
    static long cached[16] = {};
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 16) dev = 0;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 1024;
        cached[dev] = static_cast<long>(cus) * 32;
    }
    return cached[dev];
}

// a number for every call: never 0, never the same twice in a process, and unlikely to be what
// another process left in memory (the failure word and the arrival slots compare against it)
unsigned long long next_nonce() {
    static std::atomic<unsigned long long> counter{
        static_cast<unsigned long long>(std::chrono::steady_clock::now().time_since_epoch().count()) * 0x9E3779B97F4A7C15ull};
    unsigned long long n = 0;
    while (n == 0) n = counter.fetch_add(0x9E3779B97F4A7C15ull, std::memory_order_relaxed);
    return n;
}

// G, n1, n2: wavefronts per pair and exchange words per member of this call's reduction kernel (never
// more than the plan allowed for); zero_bytes: how much of the workspace's head the call has to clear
Ws carve(void* workspace, const Plan& p, int B, int rows, int G, int n1, int n2, size_t& zero_bytes) {
    char* base = static_cast<char*>(workspace);
    const size_t R = static_cast<size_t>(B) * rows;
    Ws w;
    w.counters = reinterpret_cast<unsigned*>(base + p.off_counters);
    w.sdone = w.counters + 64;
    w.state = reinterpret_cast<unsigned long long*>(base + p.off_state);
    w.part1 = reinterpret_cast<unsigned long long*>(base + p.off_part1);
    const size_t off_part2 = align_up(p.off_part1 + R * G * n1 * 8, 256);
    w.part2 = reinterpret_cast<double*>(base + off_part2);
    zero_bytes = align_up(off_part2 + R * G * n2 * 8, 256);
    w.div = reinterpret_cast<float*>(base + p.off_div);
    w.pst = reinterpret_cast<int*>(base + p.off_pst);
    w.lse2 = reinterpret_cast<double*>(base + p.off_lse2);
    w.lr = reinterpret_cast<double*>(base + p.off_lr);
    w.spart = reinterpret_cast<unsigned long long*>(base + p.off_spart);
    w.thr = reinterpret_cast<float*>(base + p.off_thr);
    w.tsd = reinterpret_cast<int*>(base + p.off_tsd);
    w.tsd_invz = reinterpret_cast<float*>(base + p.off_tsdz);
    w.wz = reinterpret_cast<unsigned long long*>(base + p.off_wz);
    w.arrive = reinterpret_cast<unsigned long long*>(base + p.off_arrive);
    w.nonce = next_nonce();
    return w;
}

unsigned g_spin_limit = 1u << 22;
// The entropy form of JS (bfloat16 logits) carries an absolute error of a few 1e-7 whatever the
// result: below this floor (nats) a pair is evaluated again in the pointwise form, so that what the
// caller sees is within 2e-3 relative everywhere (with a margin of five to ten).
float g_js_floor = 1e-3f;
bool g_exact_js = false;   // test hook: bfloat16 JS in the pointwise form only
bool g_self_clear = true;  // test hook: 0 = every call launches the clearing kernel
#ifdef FSD_PHASE_TIMING
unsigned long long* g_dbg = nullptr;
#endif

// ---- optional event timing of pair_kernel
constexpr int kMaxProf = 4096;
bool g_prof_on = false;
int g_prof_n = 0;
hipEvent_t g_prof_ev[2 * kMaxProf];
bool g_prof_made = false;
hipEvent_t* g_prof_pair = nullptr;   // the two events of the reduction launch being timed, if any

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

template <bool BF16, int NV, int MODE, bool ALIGNED, bool TSHARED = false>
void launch_pair_k(hipStream_t st, const PairParams& P0) {
    // persistent grid: as many whole teams as fit on the device at once (at least one, whose workgroups
    // fit by the limit on the team size), in whole workgroups; the wavefronts left over leave at once
    static Residency cache[16] = {};
    const Residency res = residency_of(pair_kernel<BF16, NV, MODE, ALIGNED, TSHARED>, kWG, cache);
    const long waves_per_wg = kWG / 64;
    long nteams = res.total * waves_per_wg / P0.G;
    if (nteams > P0.npairs) nteams = P0.npairs;
    if (nteams < 1) nteams = 1;
    const long grid = (nteams * P0.G + waves_per_wg - 1) / waves_per_wg;
    PairParams P = P0;
    P.nteams = static_cast<int>(nteams);
    g_last_grid = static_cast<int>(grid);
    if (g_prof_pair) {
        // timed launch: the events take the start and the end of this dispatch itself (what a
        // kernel trace shows), not the time between two markers around it in the stream
        hipExtLaunchKernelGGL((pair_kernel<BF16, NV, MODE, ALIGNED, TSHARED>), dim3(static_cast<unsigned>(grid)), dim3(kWG), res.pad_lds, st,
                              g_prof_pair[0], g_prof_pair[1], 0, P);
    } else {
        hipLaunchKernelGGL((pair_kernel<BF16, NV, MODE, ALIGNED, TSHARED>), dim3(static_cast<unsigned>(grid)), dim3(kWG), res.pad_lds, st, P);
    }
}
template <bool BF16, int NV, int MODE>
void launch_pair_a(bool aligned, hipStream_t st, const PairParams& P) {
    if (!aligned) {
        launch_pair_k<BF16, NV, MODE, false>(st, P);   // (rows that are not 16-byte aligned: no tree variant, a tree's target rows are then not kept cached)
    } else {
        if (P.parent != nullptr) launch_pair_k<BF16, NV, MODE, true, true>(st, P);   // a tree: shared target rows
        else launch_pair_k<BF16, NV, MODE, true>(st, P);
    }
}
template <bool BF16, int NV>
void launch_pair_m(int mode, bool aligned, hipStream_t st, const PairParams& P) {
    switch (mode) {
        case MODE_KL: launch_pair_a<BF16, NV, MODE_KL>(aligned, st, P); break;
        case MODE_JS: launch_pair_a<BF16, NV, MODE_JS>(aligned, st, P); break;
        case MODE_TV: launch_pair_a<BF16, NV, MODE_TV>(aligned, st, P); break;
        case MODE_KLP: launch_pair_a<BF16, NV, MODE_KLP>(aligned, st, P); break;
        case MODE_JSE: launch_pair_a<BF16, NV, MODE_JS>(aligned, st, P); break;   // (its own shape is launched by launch_pair)
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
        g_prof_pair = &g_prof_ev[2 * g_prof_n];
    }
    if (dtype == FSD_BF16) {
        if (NV == 2) launch_pair_m<true, 2>(mode, aligned, st, P);
        else if (NV == 6) {   // the library's own shape of the two-phase kernels
            if (mode == MODE_JSE) launch_pair_a<true, 6, MODE_JSE>(aligned, st, P);
            else if (mode == MODE_TV) launch_pair_a<true, 6, MODE_TV>(aligned, st, P);
            else launch_pair_a<true, 6, MODE_JS>(aligned, st, P);
        }
        else if (NV == 5) launch_pair_m<true, 5>(mode, aligned, st, P);
        else launch_pair_m<true, 4>(mode, aligned, st, P);
    } else {
        if (NV == 2) launch_pair_m<false, 2>(mode, aligned, st, P);
        else if (NV == 4) launch_pair_m<false, 4>(mode, aligned, st, P);
        else launch_pair_m<false, 8>(mode, aligned, st, P);
    }
    if (prof) {
        g_prof_pair = nullptr;
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

// Device address of the static scratch array on the current device (nullptr if the runtime will not
// give it).  Every GPU holds its own copy of the array at its own address, so the address is looked
// up once per device, with that device current, and kept.
void* static_scratch() {
    static std::atomic<void*> ptr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    void* p = ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[dev].store(p, std::memory_order_release);
    }
    return p;
}

// the common body of the entry points
int run(int kind, const void* target, const void* draft, const int32_t* tokens, const int32_t* parent, int B,
        int rows, int max_depth, int V, int dtype, int div, float T, int mode, uint64_t seed, uint64_t offset,
        int32_t* out_len, int32_t* path_nodes, int32_t* out_tokens, float* user_vals, float* user_ratio,
        int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream,
        float temperature = 1.0f, int top_k = 0, float top_p = 1.0f, bool static_ws = false) {
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
    if (static_ws) {
        // the library's own buffer instead of the caller's
        if (p.bytes > static_cast<size_t>(FSD_STATIC_SCRATCH_BYTES)) return FSD_ERR_TOO_LARGE;
        workspace = static_scratch();
        if (!workspace) return FSD_ERR_LAUNCH;
    } else if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || workspace_bytes < p.bytes) {
        return FSD_ERR_WORKSPACE;
    }

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool aligned = is_aligned(target, draft, V, p.VE);
    const int R = B * rows;

    // which reduction kernel, and its shape
    int k1mode = (kind == KIND_SD || kind == KIND_TREESD) ? MODE_LSE : div;
    if (k1mode == MODE_KL && dtype == FSD_F32) k1mode = MODE_KLP;
    // bfloat16 JS: the entropy form (reducible FSD, whose finisher also forms the candidates' log-ratios,
    // and the shapes of the tuning hook stay with the pointwise form)
    if (k1mode == MODE_JS && dtype == FSD_BF16 && kind != KIND_RFSD && !g_exact_js && !g_shape_nv) k1mode = MODE_JSE;
    if (dtype == FSD_BF16 && !g_shape_nv && (k1mode == MODE_JS || k1mode == MODE_TV || k1mode == MODE_JSE)) {
        // The bfloat16 two-phase kernels are bound by instruction issue, a third of it per step and not
        // per entry: they hold 6 slots of each row per lane (96 logits a step), which fits two wavefronts
        // per SIMD (256 registers) because 5 of the 12 chunks of each set of kept exponentials live in
        // LDS.  The workspace is laid out for the larger team of the 4-slot shape.
        p.NV = 6;
        p.G = static_cast<int>(team_size(p.nslots, p.NV));
        p.spm = static_cast<int>((p.nslots + p.G - 1) / p.G);
        // entropy form: whole chunks of 64 NV slots per member, so that only the last one with any
        // slots has lanes without one (those lanes cost it selections the others do not pay for)
        if (k1mode == MODE_JSE) p.spm = 64 * p.NV;
    }
    // exchange words a member posts in this mode: only those are laid out and cleared
    const bool two_phase = (k1mode == MODE_JS || k1mode == MODE_TV || k1mode == MODE_KLP || k1mode == MODE_JSE);
    const int n1 = two_phase ? 2 : 4;
    const int n2 = (k1mode == MODE_TV || k1mode == MODE_KLP) ? 2 : two_phase ? 1 : 0;
    size_t zero_bytes = 0;
    const Ws ws = carve(workspace, p, B, rows, p.G, n1, n2, zero_bytes);

    // The calls have no clearing kernel: the reduction clears what it and the kernels after it need (see
    // clear_own_words in pair_kernel.h; C2: -3 us a call, C4: -2 us), unless there are more than 4 MB to
    // clear (inside the reduction kernel that costs what the kernel of its own costs, C3: 7.5 MB) or
    // the grid is too large for the arrival slots.
    const bool warped = (temperature != 1.0f) || (top_k > 0 && top_k < V) || (top_p < 1.0f);
    const bool self_clear = g_self_clear && zero_bytes <= (4u << 20) && max_resident_wavefronts() <= kMaxArrive;
    if (!self_clear) {
        const long n16 = static_cast<long>(zero_bytes / 16);
        hipLaunchKernelGGL(zero_counters, dim3(static_cast<unsigned>((n16 + 255) / 256)), dim3(256), 0, st,
                           reinterpret_cast<uint4*>(ws.counters), n16);
    }

    PairParams pp;
    pp.self_clear = self_clear ? 1 : 0;
    // what no team owns: the sampler's counters (all but the first four words: the failure word, words 2-3,
    // is never cleared here, so that a flag raised early cannot be lost) and its shares
    pp.clear_a = reinterpret_cast<uint4*>(ws.counters + 4);
    pp.clear_a16 = static_cast<long>((p.n_counters - 4) * 4 / 16);
    // (the walk's shares lie right before the sampler's: strict SD over a tree has both cleared)
    pp.clear_b = reinterpret_cast<uint4*>(kind == KIND_TREESD ? reinterpret_cast<char*>(ws.wz) : reinterpret_cast<char*>(ws.spart));
    pp.clear_b16 = static_cast<long>((p.off_part1 - (kind == KIND_TREESD ? p.off_wz : p.off_spart)) / 16);
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
    pp.js_floor = g_js_floor;
    pp.ws = ws;
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
    sp.spin_limit = g_spin_limit;
    sp.thr = nullptr;
    sp.inv_temp = 1.0f;
    sp.clear_arrive = self_clear ? 1 : 0;
    if (warped && mode == FSD_SAMPLE) {
        // warpers: one more kernel finds, per sequence, the smallest kept scaled logit
        WarpParams wp;
        wp.target = static_cast<const char*>(target);
        wp.parent = (kind == KIND_TREE) ? parent : nullptr;
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
        case FSD_ERR_TOO_LARGE: return "sizes need more scratch memory than the static buffer holds (FSD_STATIC_SCRATCH_BYTES)";
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

int fsd_verify_tree_warped(const void* target_logits, const void* draft_logits, const int32_t* node_tokens,
                           const int32_t* parent, int B, int N, int max_depth, int V, int dtype, int div, float T,
                           int mode, uint64_t seed, uint64_t offset, float temperature, int top_k, float top_p,
                           int32_t* path_len, int32_t* path_nodes, int32_t* out_tokens, float* divergences,
                           int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(KIND_TREE, target_logits, draft_logits, node_tokens, parent, B, N, max_depth, V, dtype, div, T, mode,
               seed, offset, path_len, path_nodes, out_tokens, divergences, nullptr, row_status, workspace,
               workspace_bytes, hip_stream, temperature, top_k, top_p);
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

int fsd_verify_chain_static(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens, int B,
                            int K, int V, int dtype, int div, float T, int mode, uint64_t seed, uint64_t offset,
                            int32_t* accept_len, int32_t* out_tokens, float* divergences, int32_t* row_status,
                            void* hip_stream) {
    return run(KIND_CHAIN, target_logits, draft_logits, cand_tokens, nullptr, B, K, 0, V, dtype, div, T, mode, seed,
               offset, accept_len, nullptr, out_tokens, divergences, nullptr, row_status, nullptr, 0, hip_stream,
               1.0f, 0, 1.0f, true);
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

float fsd_debug_set_js_floor(float floor_nats) {
    const float prev = g_js_floor;
    g_js_floor = floor_nats;
    return prev;
}

int fsd_debug_set_exact_js(int on) {
    const int prev = g_exact_js ? 1 : 0;
    g_exact_js = (on != 0);
    return prev;
}

int fsd_debug_set_self_clear(int on) {
    const int prev = g_self_clear ? 1 : 0;
    g_self_clear = (on != 0);
    return prev;
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
