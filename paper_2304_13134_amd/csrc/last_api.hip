// C ABI of the lattice library (see include/last.h): argument validation,
// workspace planning and kernel launches.  No allocation, no synchronisation.
#include "../../include/last.h"

#include <hip/hip_runtime.h>

#include "common.hpp"
#include "solo_kernels.hpp"
#include "numerator_kernels.hpp"
#include "table_kernels.hpp"
#include "cluster_kernels.hpp"
#include "cluster2_kernels.hpp"
#include "cluster2v_kernels.hpp"
#include "cluster3_kernels.hpp"
#include "cluster3v_kernels.hpp"
#include "fused_kernels.hpp"
#include "fused_numerator_kernels.hpp"
#include "probe_kernels.hpp"
#include <algorithm>

#include <atomic>
#include <cstdlib>
#include <mutex>
#include <set>
#include <utility>
#include <type_traits>

using namespace last;

namespace {

// process-wide settings (last_set_option)
std::atomic<int> g_opt[LAST_OPT_COUNT_] = {{0}, {0}, {1}, {1 << 20}, {2}, {1}};
inline int opt(int o) { return g_opt[o].load(std::memory_order_relaxed); }

constexpr size_t kAlign = 256;
inline size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

// bump allocator over the caller's workspace; with base == nullptr it only measures
struct Carver {
    char* base;
    size_t used = 0;
    explicit Carver(void* p) : base((char*)p) {}
    template <typename T>
    T* take(size_t count)
    {
        T* p = base ? (T*)(base + used) : nullptr;
        used += align_up(count * sizeof(T));
        return p;
    }
};

struct Shape {
    int B, T, V, V1, C, order;
    const int* nx;       // order 0: device next-state table [C][V]
};

last_status_t check_common(const last_weights_t* wt, const last_context_t* cx, Shape* s)
{
    if (!wt || !cx) return LAST_ERR_NULL;
    if (cx->order < 0 || cx->order > 2) return LAST_ERR_CONTEXT;
    if (cx->vocab < 1) return LAST_ERR_CONTEXT;
    const long long V = cx->vocab;
    long long C = cx->order == 1 ? 1 + V : 1 + V + V * V;
    if (cx->order == 0) {
        // any deterministic automaton, as a table; the weights stay dense
        if (!cx->next_table) return LAST_ERR_NULL;
        if (cx->num_states < 1) return LAST_ERR_CONTEXT;
        if (wt && wt->kind != LAST_WEIGHTS_DENSE) return LAST_ERR_UNSUPPORTED;
        // (the fixed-point sums of the table kernels hold at most 2^24 arcs into one state)
        if ((long long)cx->num_states * V > (1ll << 24)) return LAST_ERR_UNSUPPORTED;
        C = cx->num_states;
    }
    if (C != cx->num_states || C > (1 << 24) || C * (V + 1) > (1ll << 31) - 2) return LAST_ERR_CONTEXT;
    if (wt->B < 1 || wt->T < 0) return LAST_ERR_SHAPE;
    if (wt->B > 65535 || wt->T > (1 << 24)) return LAST_ERR_SHAPE;
    if (wt->kind == LAST_WEIGHTS_DENSE) {
        if (!wt->w) return LAST_ERR_NULL;
    } else if (wt->kind == LAST_WEIGHTS_SHARED_EMB) {
        if (!wt->f || !wt->e || !wt->W) return LAST_ERR_NULL;
        if (wt->hidden < 1) return LAST_ERR_SHAPE;
    } else {
        return LAST_ERR_UNSUPPORTED;
    }
    s->B = wt->B;
    s->T = wt->T;
    s->V = cx->vocab;
    s->V1 = cx->vocab + 1;
    s->C = (int)C;
    s->order = cx->order;
    s->nx = cx->order == 0 ? cx->next_table : nullptr;
    return LAST_OK;
}

Ctx make_ctx(const Shape& s) { return Ctx{s.V, s.order, s.C, s.V1, s.nx}; }

// thread layout of the one-workgroup-per-item forward kernels
struct SoloLayout {
    int CPAD, R;
    size_t lds_forward, lds_viterbi, lds_backward;
};

SoloLayout solo_layout(const Shape& s)
{
    SoloLayout l;
    int cpad = (s.C + 63) / 64 * 64;
    if (cpad > 1024) cpad = 1024;
    l.CPAD = cpad;
    l.R = 1024 / cpad;
    l.lds_forward = (size_t)(2 * s.C + 2 * l.R * l.CPAD + 32) * sizeof(float);
    l.lds_viterbi = (size_t)(2 * s.C + 2 * l.R * l.CPAD + 64) * sizeof(float);
    l.lds_backward = (size_t)(2 * s.C + 32) * sizeof(float);
    if (s.order == 0) {   // arcs by source state (table_kernels.hpp)
        l.lds_forward = (size_t)s.C * 16 + 32 * sizeof(float);
        l.lds_viterbi = (size_t)s.C * 12 + 64 * sizeof(float);
    }
    return l;
}

constexpr size_t kMaxLds = 64 * 1024;

// In table mode the workspace starts with the flag that the table check of the call sets.
int* carve_table_flag(Carver& cv, const Shape& s) { return s.order == 0 ? cv.take<int>(64) : nullptr; }

void launch_table_check(const Shape& s, int* flag, hipStream_t st)
{
    hipLaunchKernelGGL(table_clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    hipLaunchKernelGGL(table_check_kernel, dim3(64), dim3(256), 0, st, s.nx, s.C, s.V, flag);
}

struct PosteriorWs {
    float* alpha;
    double* offs;
    double* D;
};

PosteriorWs carve_posteriors(Carver& cv, const Shape& s)
{
    PosteriorWs p;
    p.alpha = cv.take<float>((size_t)s.B * (s.T + 1) * s.C);
    p.offs = cv.take<double>((size_t)s.B * (s.T + 1));
    p.D = cv.take<double>((size_t)s.B);
    return p;
}

struct PathWs {
    int* bp;
    int* final_state;
    int* map;            // backtrace: [B][nseg][C] state at the lower end of a segment, by state at its upper end
    int* bnd;            // backtrace: [B][nseg+1] states of the path at the segment boundaries
    int S, nseg;         // frames per segment (about sqrt(T)), number of segments
    u64* xv;             // exchange buffer of the clustered tropical kernel (xwords > 0)
};

PathWs carve_path(Carver& cv, const Shape& s, size_t xwords)
{
    PathWs p;
    p.S = 8;
    while (p.S * p.S < s.T) ++p.S;
    p.nseg = s.T > 0 ? (s.T + p.S - 1) / p.S : 1;
    p.bp = cv.take<int>((size_t)s.B * (s.T > 0 ? s.T : 1) * s.C);
    p.final_state = cv.take<int>((size_t)s.B);
    p.map = cv.take<int>((size_t)s.B * p.nseg * s.C);
    p.bnd = cv.take<int>((size_t)s.B * (p.nseg + 1));
    p.xv = xwords ? cv.take<u64>(xwords) : nullptr;
    return p;
}

struct NumWs {
    float2* wi;
    double* a;
    double* bk;
    double* N;
    int* status;
    int* ctxs;
    int* link;
    double* lz;          // locally normalised only
};

NumWs carve_num(Carver& cv, const Shape& s, int Umax, bool local)
{
    NumWs p;
    const size_t U1 = (size_t)Umax + 1;
    p.ctxs = cv.take<int>((size_t)s.B * U1);
    p.link = cv.take<int>((size_t)s.B * U1 * 2);
    p.lz = local ? cv.take<double>((size_t)s.B * (s.T > 0 ? s.T : 1) * U1) : nullptr;
    p.wi = cv.take<float2>((size_t)s.B * (s.T > 0 ? s.T : 1) * U1);
    p.a = cv.take<double>((size_t)s.B * (s.T + 1) * U1);
    p.bk = cv.take<double>((size_t)s.B * (s.T + 1) * U1);
    p.N = cv.take<double>((size_t)s.B);
    p.status = cv.take<int>((size_t)s.B);
    return p;
}

// geometry of the clustered bigram path (see cluster_kernels.hpp)
struct ClusterPlan {
    bool ok;
    int gen;             // 2: one exchange per two frames (cluster2_kernels.hpp); 3: the same with the work cut
                         // down to the wave and 16-byte accesses throughout (cluster3_kernels.hpp, 256 labels
                         // only); 1: one exchange per frame
    int K, RPW, ncl, XS, XSB, grid;
};

// The cooperating-workgroup kernels spin on each other: every workgroup of a launch must be resident
// at once, one per compute unit, on a chip of eight XCDs of 32 compute units each (a cluster of an
// item sits on the XCD its workgroup ids select).  Anything else takes the one-workgroup kernels.
// (Without a device, e.g. when only sizes are asked for on a build machine, the layout is assumed.)
std::mutex g_chip_mutex;
int g_chip_state[64] = {};                 // per device: 0 unknown, 1 takes clusters, 2 does not
bool chip_takes_clusters()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return true; }
    if (dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(g_chip_mutex);
    if (!g_chip_state[dev]) {
        int cus = 0;
        const hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) (void)hipGetLastError();
        g_chip_state[dev] = (e == hipSuccess && cus >= 256) ? 1 : 2;
    }
    return g_chip_state[dev] == 1;
}

ClusterPlan cluster_plan(const Shape& s, int kind)
{
    ClusterPlan p{};
    if (opt(LAST_OPT_FORCE_SOLO) || !chip_takes_clusters()) return p;
    if (kind != LAST_WEIGHTS_DENSE || s.order != 1 || s.C > kClMaxC || s.C < 5 || s.T < 1) return p;   // (tiny label sets: one workgroup per item)
    // one item must fit a 32-bit buffer descriptor
    if ((double)s.T * s.C * s.C * sizeof(float) >= 4.0e9) return p;
    const int want_gen = opt(LAST_OPT_CLUSTER_GENERATION);      // 0: the newest that takes the shape
    if ((want_gen == 0 || want_gen == 3) && s.C == kC3C) {
        p.gen = 3;
        p.K = kC3K;
        p.RPW = 32;
        const int want3 = (s.B + 7) / 8;
        p.ncl = want3 < 2 ? want3 : 2;       // one workgroup per compute unit: 32 per XCD, 16 per item
        p.XS = kC3XS;
        p.XSB = 0;
        p.grid = 8 * p.ncl * 2 * p.K;
        p.ok = true;
        return p;
    }
    p.K = (s.C + 32) / 33;                   // at most 33 rows per workgroup
    if (p.K > kClMaxK) return p;
    p.RPW = (s.C + p.K - 1) / p.K;
    if (s.C - (p.K - 1) * p.RPW < 1) return p;   // every workgroup must own at least one row
    const int max_ncl = 32 / (2 * p.K);      // one workgroup per compute unit: 32 per XCD
    if (max_ncl < 1) return p;
    int want = (s.B + 7) / 8;
    p.ncl = want < max_ncl ? want : max_ncl;
    p.XS = s.C + 4;                          // exchange rows: C states, 1 header row, read-ahead pad
    p.XSB = kClMaxC;                         // 11 waves x 24 words
    p.grid = 8 * p.ncl * 2 * p.K;
    p.ok = true;
    // the second generation (one exchange per two frames) unless the first is asked for
    p.gen = (want_gen != 1 && s.C <= kC2Hdr && s.C >= 5) ? 2 : 1;   // (16-byte accesses: four label columns at least)
    return p;
}

struct ClusterWs {
    float* ahat;
    float* bhat;
    int* Sa;
    int* Sb;
    u64* xa;
    u64* xb;
    u64* ph;
    u64* fin;
    size_t xwords;
};

ClusterWs carve_cluster(Carver& cv, const Shape& s, const ClusterPlan& p)
{
    ClusterWs c;
    const size_t st = (size_t)s.B * (s.T + 1);
    const size_t per_state = p.gen == 3 ? 2 : 1;          // third generation: (value, exponent) pairs
    c.ahat = cv.take<float>(st * s.C * per_state);
    c.bhat = cv.take<float>(st * s.C * per_state);
    const size_t nblk = p.gen == 3 ? kC3K : kClMaxK;      // one exponent per block of states
    c.Sa = cv.take<int>(st * nblk);
    c.Sb = cv.take<int>(st * nblk);
    const size_t ncl = (size_t)8 * p.ncl;
    const size_t per_role = p.gen == 3 ? (size_t)2 * kC3K * kC3XS
                                       : std::max((size_t)2 * p.XS * kClXK, (size_t)2 * kClMaxK * kC2XS);
    const size_t nxa = ncl * per_role, nxb = std::max(ncl * 2 * p.XSB, ncl * per_role), nph = ncl * 32;
    const size_t nfin = (size_t)2 * s.B;
    // one contiguous block so that a single launch clears all tags
    c.xa = cv.take<u64>(nxa + nxb + nph + nfin);
    c.xb = c.xa ? c.xa + nxa : nullptr;
    c.ph = c.xb ? c.xb + nxb : nullptr;
    c.fin = c.ph ? c.ph + nph : nullptr;
    c.xwords = nxa + nxb + nph + nfin;
    return c;
}

// Set while last_globally_normalized_loss enqueues its denominator: the numerator's kernels run beside it
// on another stream, and only the leaner instantiation of cluster3_kernel leaves them registers to do so.
thread_local bool g_numerator_beside = false;

template <bool GAMMA>
void launch_cluster(const Shape& s, const ClusterPlan& p, const ClusterWs& c, const float* w,
                    const int* lengths, float* dist, int* item_status, float* dw, float scale,
                    int accumulate, hipStream_t st)
{
    hipLaunchKernelGGL(cluster_clear_kernel, dim3(64), dim3(256), 0, st, c.xa, c.xwords);
    ClusterArgs a;
    a.w = w; a.len = lengths; a.dw = dw; a.dist = dist; a.item_status = item_status;
    a.ahat = c.ahat; a.bhat = c.bhat; a.Sa = c.Sa; a.Sb = c.Sb;
    a.xa = c.xa; a.xb = c.xb; a.ph = c.ph; a.fin = c.fin;
    a.B = s.B; a.T = s.T; a.C = s.C;
    a.K = p.K; a.RPW = p.RPW; a.ncl = p.ncl; a.XS = p.XS; a.XSB = p.XSB;
    a.scale = scale; a.accumulate = accumulate;
    a.spin_limit = opt(LAST_OPT_SPIN_LIMIT);
    if (p.gen == 3) {
        if (GAMMA && accumulate)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster3_kernel<GAMMA, GAMMA, 2>), dim3(p.grid), dim3(kC3Threads), 0, st, a);
        else if (GAMMA && !g_numerator_beside)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster3_kernel<GAMMA, false, GAMMA ? 3 : 2>), dim3(p.grid), dim3(kC3Threads), 0, st, a);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster3_kernel<GAMMA, false, 2>), dim3(p.grid), dim3(kC3Threads), 0, st, a);
        return;
    }
    if (p.gen == 2) {
        if (GAMMA && accumulate)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2_kernel<GAMMA, GAMMA, false>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
        else if (p.K == kClMaxK)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2_kernel<GAMMA, false, true>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2_kernel<GAMMA, false, false>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
        return;
    }
    auto go = [&](auto KC) {
        constexpr int KT = decltype(KC)::value;
        if (GAMMA && accumulate)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster_fb_kernel<3, GAMMA, GAMMA, KT>), dim3(p.grid),
                               dim3(kClThreads), 0, st, a);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster_fb_kernel<3, GAMMA, false, KT>), dim3(p.grid),
                               dim3(kClThreads), 0, st, a);
    };
    switch (p.K) {
    case 1: go(std::integral_constant<int, 1>()); break;
    case 2: go(std::integral_constant<int, 2>()); break;
    case 3: go(std::integral_constant<int, 3>()); break;
    case 4: go(std::integral_constant<int, 4>()); break;
    case 5: go(std::integral_constant<int, 5>()); break;
    case 6: go(std::integral_constant<int, 6>()); break;
    case 7: go(std::integral_constant<int, 7>()); break;
    default: go(std::integral_constant<int, 8>()); break;
    }
}

hipError_t g_last_hip_error = hipSuccess;     // diagnostics only: what the last failing HIP call said

last_status_t hip_status()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) g_last_hip_error = e;
    return e == hipSuccess ? LAST_OK : LAST_ERR_HIP;
}

template <typename F>
void dispatch_group(int V1, F&& f)
{
    if (V1 <= 4) f(std::integral_constant<int, 4>());
    else if (V1 <= 8) f(std::integral_constant<int, 8>());
    else if (V1 <= 16) f(std::integral_constant<int, 16>());
    else if (V1 <= 48) f(std::integral_constant<int, 32>());
    else f(std::integral_constant<int, 64>());
}

constexpr size_t kBigLds = 160 * 1024;

// A kernel that wants more than 64 KiB of LDS has to be told so once on every device it runs on.
last_status_t allow_lds(const void* kernel, size_t bytes)
{
    static std::mutex mu;
    static std::set<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({dev, kernel})) return LAST_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    done.insert({dev, kernel});
    return LAST_OK;
}

// ---- context dependency given as a table: one workgroup per item, arcs by source state ----
last_status_t launch_table_forward(const Shape& s, const SoloLayout& l, const float* w, const int* lengths,
                                   float* alpha, double* offs, double* D, float* dist, int* item_status,
                                   const int* flag, hipStream_t st)
{
    if (l.lds_forward > kBigLds) return LAST_ERR_UNSUPPORTED;
    const Ctx c = make_ctx(s);
    last_status_t rc = LAST_OK;
    dispatch_group(s.V1, [&](auto G) {
        auto k = table_forward_log<decltype(G)::value>;
        if (l.lds_forward > kMaxLds) rc = allow_lds((const void*)k, kBigLds);
        if (rc == LAST_OK)
            hipLaunchKernelGGL(k, dim3(s.B), dim3(1024), l.lds_forward, st, w, lengths, c, s.T, alpha, offs,
                               D, dist, item_status, flag);
    });
    return rc;
}

last_status_t launch_table_viterbi(const Shape& s, const SoloLayout& l, const float* w, const int* lengths,
                                   int* bp, int* final_state, float* score, int* item_status,
                                   const int* flag, hipStream_t st)
{
    if (l.lds_viterbi > kBigLds) return LAST_ERR_UNSUPPORTED;
    const Ctx c = make_ctx(s);
    last_status_t rc = LAST_OK;
    dispatch_group(s.V1, [&](auto G) {
        auto k = table_viterbi<decltype(G)::value>;
        if (l.lds_viterbi > kMaxLds) rc = allow_lds((const void*)k, kBigLds);
        if (rc == LAST_OK)
            hipLaunchKernelGGL(k, dim3(s.B), dim3(1024), l.lds_viterbi, st, w, lengths, c, s.T, bp,
                               final_state, score, item_status, flag);
    });
    return rc;
}

// geometry of the fused trigram path (see fused_kernels.hpp)
constexpr int kFusedMaxLds = 160 * 1024 - 2048;   // dynamic LDS; the kernel also has a little static LDS
constexpr size_t kFusedKeepBytes = (size_t)8 << 30;   // most that is kept of the marginals between two kernels
struct FusedPlan {
    bool ok;
    int ncl, XW, KC, R, Mpad, MT;
    int NF;              // frames whose weights the forward kernel computes at a time
    size_t gamma_elems;  // bf16 values of the marginals the backward kernel keeps for the dW kernel; 0: none kept
    size_t lds;          // forward kernel
    size_t lds_bwd;      // backward recursion kernel
    size_t lds_dw;       // dW kernel
    int nch, TC;         // frame chunks of the dW kernel
};

template <typename F>
void fused_dispatch(int MT, F&& f)
{
    if (MT == 1) f(std::integral_constant<int, 1>());
    else if (MT == 3) f(std::integral_constant<int, 3>());
    else f(std::integral_constant<int, 5>());
}

FusedPlan fused_plan(const Shape& s, const last_weights_t* wt)
{
    FusedPlan p{};
    if (wt->kind != LAST_WEIGHTS_SHARED_EMB || s.order != 2 || !chip_takes_clusters()) return p;
    const int H = wt->hidden;
    if (s.V > 64 || H % kFuKC != 0 || H < kFuKC || H > 512) return p;
    // the kernels fetch f and e with 16-byte loads
    if (((uintptr_t)wt->f | (uintptr_t)wt->e | (uintptr_t)wt->W) % 16 != 0) return p;
    p.R = s.V + 2;
    p.Mpad = (p.R + 15) / 16 * 16;
    p.KC = H < kFuKC ? H : kFuKC;
    p.ncl = 256 / s.V;                        // one workgroup per compute unit
    if (p.ncl > s.B) p.ncl = s.B;
    p.XW = (s.V + 7) / 8 * 8;
    p.MT = p.Mpad / 16 <= 1 ? 1 : p.Mpad / 16 <= 3 ? 3 : 5;   // instantiated row-tile counts
    auto lds_forward = [&](int nf) {
        return (size_t)p.R * H * 2 + (size_t)2 * nf * 16 * p.MT * kFuHS * 2 + (size_t)(6 * kFuMaxRows + 8 + 32 + 8) * 4
               + (size_t)nf * H * 2;
    };
    p.NF = opt(LAST_OPT_FUSED_FRAMES_PER_TILE) == 2 && lds_forward(2) <= (size_t)kFusedMaxLds ? 2 : 1;
    p.lds = lds_forward(p.NF);
    const size_t tiles = (size_t)kFuMaxRows * kFuWS * 4 + (size_t)2 * kFuMaxRows * kFuGS * 2;
    p.lds_bwd = (size_t)kFuMaxRows * kFuHF * 2 + tiles + (size_t)(5 * kFuMaxRows + 8) * 4;
    p.lds_dw = (size_t)(32 * ((16 * p.MT + 31) / 32)) * kFuHF * 2 + tiles + (size_t)(4 * kFuMaxRows) * 4;
    p.nch = 256 / (s.B * s.V);                // fill the chip when the batch is small
    if (p.nch > (s.T + 15) / 16) p.nch = (s.T + 15) / 16;
    if (p.nch < 1) p.nch = 1;
    p.TC = (s.T + p.nch - 1) / p.nch;
    p.ok = p.lds <= (size_t)kFusedMaxLds && p.lds_bwd <= (size_t)kFusedMaxLds
           && p.lds_dw <= (size_t)kFusedMaxLds;
    // marginals kept between the backward and the dW kernel: two bf16 planes of [V + 2][V + 1 rounded up to 8]
    // per frame and last label, as long as they stay below kFusedKeepBytes
    const size_t ge = (size_t)s.B * s.T * s.V * 2 * p.R * (size_t)((s.V1 + 7) / 8 * 8);
    p.gamma_elems = opt(LAST_OPT_FUSED_KEEP_MARGINALS) && ge * 2 <= kFusedKeepBytes ? ge : 0;
    return p;
}

// shapes the on-the-fly numerator takes: every lane of a wavefront owns H/64 hidden units, in pairs
bool fused_numerator_ok(const last_weights_t* wt)
{
    const int H = wt->hidden;
    if (H % 128 != 0 || H < 128 || H > 128 * kFnMaxPairs) return false;
    return (((uintptr_t)wt->f | (uintptr_t)wt->e | (uintptr_t)wt->W) % 16) == 0;
}

struct FusedWs {
    float* alpha;
    float* beta;
    __bf16* gamma;
    bf16x8* Wf;
    bf16x8* Wt;
    double* offs;
    float* part;
    double* Aend;
    double* D;
    u64* xb;
    size_t xwords;
};

FusedWs carve_fused(Carver& cv, const Shape& s, const FusedPlan& p, bool keep_alpha)
{
    FusedWs f;
    f.alpha = keep_alpha ? cv.take<float>((size_t)s.B * (s.T + 1) * s.C) : nullptr;
    f.beta = keep_alpha ? cv.take<float>((size_t)s.B * (s.T + 1) * s.C) : nullptr;
    f.gamma = keep_alpha && p.gamma_elems ? cv.take<__bf16>(p.gamma_elems) : nullptr;
    f.Wf = cv.take<bf16x8>((size_t)kFuMaxNT * kFuMaxKS * 64);
    f.Wt = keep_alpha ? cv.take<bf16x8>((size_t)32 * 3 * 64) : nullptr;
    f.offs = cv.take<double>((size_t)s.B * (s.T + 1));
    f.part = cv.take<float>((size_t)s.B * s.V);
    f.Aend = cv.take<double>((size_t)s.B);
    f.D = cv.take<double>((size_t)s.B);
    f.xwords = (size_t)p.ncl * 2 * (s.V + 1) * p.XW;
    f.xb = cv.take<u64>(f.xwords);
    return f;
}

last_status_t launch_fused_forward(const Shape& s, const FusedPlan& p, const FusedWs& f,
                                   const last_weights_t* wt, const int* lengths, float* dist,
                                   int* item_status, bool keep_alpha, hipStream_t st)
{
    {
        const void* kernels[15] = {
            (const void*)fused_forward_kernel<1, 1>, (const void*)fused_forward_kernel<3, 1>, (const void*)fused_forward_kernel<5, 1>,
            (const void*)fused_forward_kernel<1, 2>, (const void*)fused_forward_kernel<3, 2>, (const void*)fused_forward_kernel<5, 2>,
            (const void*)fused_backward_kernel<1>, (const void*)fused_backward_kernel<3>, (const void*)fused_backward_kernel<5>,
            (const void*)fused_dw_kernel<1>, (const void*)fused_dw_kernel<3>, (const void*)fused_dw_kernel<5>,
            (const void*)fused_dw_kept_kernel<1>, (const void*)fused_dw_kept_kernel<3>, (const void*)fused_dw_kept_kernel<5>};
        for (const void* k : kernels) {
            const last_status_t rc = allow_lds(k, kFusedMaxLds);
            if (rc != LAST_OK) return rc;
        }
    }
    hipLaunchKernelGGL(cluster_clear_kernel, dim3(64), dim3(256), 0, st, f.xb, f.xwords);
    const int npack = std::max(kFuMaxNT * kFuMaxKS * 64, (wt->hidden / 16) * 3 * 64);
    hipLaunchKernelGGL(fused_pack_w_kernel, dim3((npack + 255) / 256), dim3(256), 0, st,
                       (const __bf16*)wt->W, wt->hidden, s.V1, f.Wf, f.Wt);
    FusedArgs a;
    a.f = (const __bf16*)wt->f; a.e = (const __bf16*)wt->e; a.Wf = f.Wf;
    a.len = lengths; a.dist = dist; a.item_status = item_status;
    a.alpha_ws = keep_alpha ? f.alpha : nullptr; a.offs = f.offs; a.part = f.part; a.Aend = f.Aend;
    a.xb = f.xb;
    a.B = s.B; a.T = s.T; a.V = s.V; a.H = wt->hidden; a.C = s.C;
    a.ncl = p.ncl; a.XW = p.XW; a.spin_limit = opt(LAST_OPT_SPIN_LIMIT);
    fused_dispatch(p.MT, [&](auto MT) {
        if (p.NF == 2)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(fused_forward_kernel<decltype(MT)::value, 2>), dim3(p.ncl * s.V),
                               dim3(kFuThreads), p.lds, st, a);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(fused_forward_kernel<decltype(MT)::value, 1>), dim3(p.ncl * s.V),
                               dim3(kFuThreads), p.lds, st, a);
    });
    hipLaunchKernelGGL(fused_finalize_kernel, dim3((s.B + 63) / 64), dim3(64), 0, st,
                       (const float*)f.part, (const double*)f.Aend, s.B, s.V, dist, f.D, item_status);
    return hip_status();
}

// beta recursion + gradients of the fused path; the forward pass (with alpha kept) has been enqueued
last_status_t launch_fused_backward(const Shape& s, const FusedPlan& p, const FusedWs& f, float* dist,
                                    const last_weights_t* wt, const int* lengths, const last_grads_t* out,
                                    int* item_status, hipStream_t st)
{
    const int H = wt->hidden;
    if (!out->accumulate) {
        hipLaunchKernelGGL(zero_fill_kernel, dim3(256), dim3(256), 0, st, out->df, (size_t)s.B * s.T * H);
        hipLaunchKernelGGL(zero_fill_kernel, dim3(256), dim3(256), 0, st, out->de, (size_t)s.C * H);
        hipLaunchKernelGGL(zero_fill_kernel, dim3(64), dim3(256), 0, st, out->dW, (size_t)H * s.V1);
    }
    if (s.T == 0) return hip_status();
    hipLaunchKernelGGL(cluster_clear_kernel, dim3(64), dim3(256), 0, st, f.xb, f.xwords);
    FusedBwdArgs a;
    a.f = (const __bf16*)wt->f; a.e = (const __bf16*)wt->e; a.Wf = f.Wf; a.Wt = f.Wt;
    a.len = lengths; a.alpha_ws = f.alpha; a.offs = f.offs; a.Dws = f.D; a.beta_ws = f.beta;
    a.gamma_ws = f.gamma;
    a.df = out->df; a.de = out->de; a.dW = out->dW; a.scale = out->scale;
    a.item_status = item_status; a.dist = dist; a.xb = f.xb;
    a.B = s.B; a.T = s.T; a.V = s.V; a.H = H; a.C = s.C;
    a.ncl = p.ncl; a.XW = p.XW; a.spin_limit = opt(LAST_OPT_SPIN_LIMIT); a.nch = p.nch; a.TC = p.TC;
    fused_dispatch(p.MT, [&](auto MT) {
        hipLaunchKernelGGL(HIP_KERNEL_NAME(fused_backward_kernel<decltype(MT)::value>), dim3(p.ncl * s.V),
                           dim3(kFuThreads), p.lds_bwd, st, a);
        if (a.gamma_ws)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(fused_dw_kept_kernel<decltype(MT)::value>), dim3(s.B * s.V * p.nch),
                               dim3(kFuThreads), p.lds_dw, st, a);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(fused_dw_kernel<decltype(MT)::value>), dim3(s.B * s.V * p.nch),
                               dim3(kFuThreads), p.lds_dw, st, a);
    });
    return hip_status();
}

// streaming tropical kernel for the full 1-gram context dependency (129 <= C <= 264); false: not applicable
bool launch_bigram_viterbi(const Shape& s, const float* w, const int* lengths, int* bp, int* final_state,
                           float* score, int* item_status, hipStream_t st)
{
    if (s.order != 1 || s.C < 129 || s.C > kClMaxC || opt(LAST_OPT_FORCE_SOLO)) return false;
    if ((size_t)s.T * s.C * s.C * 4 >= ((size_t)1 << 31)) return false;   // one buffer descriptor per item
    if (s.C <= 256) {
        const int CPAD = 256;
        const size_t lds = (size_t)(2 * CPAD + 2 * 4 * CPAD + 64) * sizeof(float);
        hipLaunchKernelGGL(HIP_KERNEL_NAME(bigram_viterbi<64, 4>), dim3(s.B), dim3(1024), lds, st, w, lengths,
                           s.C, s.T, CPAD, bp, final_state, score, item_status);
    } else {
        const int CPAD = 320;
        const size_t lds = (size_t)(2 * CPAD + 2 * 3 * CPAD + 64) * sizeof(float);
        hipLaunchKernelGGL(HIP_KERNEL_NAME(bigram_viterbi<88, 3>), dim3(s.B), dim3(1024), lds, st, w, lengths,
                           s.C, s.T, CPAD, bp, final_state, score, item_status);
    }
    return true;
}

// geometry of the clustered tropical kernel (cluster2v_kernels.hpp): K workgroups per item
struct ViterbiPlan {
    bool ok;
    int gen;             // 3: cluster3v_kernels.hpp (256 labels), 2: cluster2v_kernels.hpp
    int K, RPW, ncl, grid;
    size_t xwords;
};

ViterbiPlan viterbi_plan(const Shape& s, int kind)
{
    ViterbiPlan p{};
    if (opt(LAST_OPT_FORCE_SOLO) || !opt(LAST_OPT_CLUSTER_VITERBI) || !chip_takes_clusters()) return p;
    if (kind != LAST_WEIGHTS_DENSE || s.order != 1 || s.C > kC2Hdr || s.T < 1) return p;
    if ((double)s.T * s.C * s.C * sizeof(float) >= 4.0e9) return p;      // one 32-bit buffer descriptor per item
    if ((size_t)s.C * s.C >= (size_t)kVNone) return p;                    // 17-bit arc indices in the exchange
    p.K = (s.C + 32) / 33;
    if (p.K > kClMaxK) return p;
    p.RPW = (s.C + p.K - 1) / p.K;
    if (s.C - (p.K - 1) * p.RPW < 1) return p;
    const int max_ncl = 32 / p.K;               // one workgroup per compute unit: 32 per XCD
    if (max_ncl < 1) return p;
    const int want = (s.B + 7) / 8;
    p.ncl = want < max_ncl ? want : max_ncl;
    p.grid = 8 * p.ncl * p.K;
    p.xwords = (size_t)8 * p.ncl * 2 * kClMaxK * kC2XS + (size_t)2 * s.B;    // exchange slots + per-item end words
    p.gen = (s.C == kV3C && opt(LAST_OPT_CLUSTER_VITERBI) != 2) ? 3 : 2;
    static_assert(kV3K == kClMaxK && kV3XS == kC2XS, "both kernels use the same exchange area");
    p.ok = true;
    return p;
}

void launch_cluster_viterbi(const Shape& s, const ViterbiPlan& p, u64* xv, const float* w, const int* lengths,
                            int* bp, int* final_state, float* score, int* item_status, hipStream_t st)
{
    hipLaunchKernelGGL(cluster_clear_kernel, dim3(64), dim3(256), 0, st, xv, p.xwords);
    ClusterVArgs a;
    a.w = w; a.len = lengths; a.bp = bp; a.final_state = final_state; a.score = score;
    a.item_status = item_status; a.xa = xv; a.fin = xv + (p.xwords - (size_t)2 * s.B);
    a.B = s.B; a.T = s.T; a.C = s.C; a.K = p.K; a.RPW = p.RPW; a.ncl = p.ncl;
    a.spin_limit = opt(LAST_OPT_SPIN_LIMIT);
    if (p.gen == 3) {
        if (bp) hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster3v_kernel<true>), dim3(p.grid), dim3(kC3Threads), 0, st, a);
        else hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster3v_kernel<false>), dim3(p.grid), dim3(kC3Threads), 0, st, a);
        return;
    }
    const bool full = p.K == kClMaxK;      // (the instantiation without a test per exchanged word)
    if (bp && full) hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2v_kernel<true, true>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
    else if (bp) hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2v_kernel<true, false>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
    else if (full) hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2v_kernel<false, true>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
    else hipLaunchKernelGGL(HIP_KERNEL_NAME(cluster2v_kernel<false, false>), dim3(p.grid), dim3(kC2Threads), 0, st, a);
}

last_status_t check_ws(void* ws, size_t have, size_t need)
{
    if (need == 0) return LAST_OK;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || have < need) return LAST_ERR_WORKSPACE;
    return LAST_OK;
}


}  // namespace

extern "C" {

int32_t last_version(void) { return 4; }

last_status_t last_set_option(int32_t option, int32_t value)
{
    if (option < 0 || option >= LAST_OPT_COUNT_) return LAST_ERR_UNSUPPORTED;
    if (option == LAST_OPT_CLUSTER_GENERATION && (value < 0 || value > 3)) return LAST_ERR_UNSUPPORTED;
    if (option == LAST_OPT_SPIN_LIMIT && value < 1) return LAST_ERR_UNSUPPORTED;
    if (option == LAST_OPT_CLUSTER_VITERBI && (value < 0 || value > 2)) return LAST_ERR_UNSUPPORTED;
    if (option == LAST_OPT_FUSED_FRAMES_PER_TILE && value != 1 && value != 2) return LAST_ERR_UNSUPPORTED;
    if (option == LAST_OPT_FUSED_KEEP_MARGINALS && value != 0 && value != 1) return LAST_ERR_UNSUPPORTED;
    g_opt[option].store(value, std::memory_order_relaxed);
    return LAST_OK;
}

int32_t last_get_option(int32_t option)
{
    return option < 0 || option >= LAST_OPT_COUNT_ ? -1 : opt(option);
}

last_status_t last_verify_placement(void* workspace, size_t workspace_bytes, void* hip_stream)
{
    constexpr int kGrid = 256;
    if (!workspace) return LAST_ERR_NULL;
    if (workspace_bytes < (kGrid + 1) * sizeof(unsigned) || (uintptr_t)workspace % 4 != 0) return LAST_ERR_WORKSPACE;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    if (dev < 0 || dev >= 64) return LAST_ERR_UNSUPPORTED;
    if (!chip_takes_clusters()) return LAST_ERR_UNSUPPORTED;     // (fewer than 256 compute units: already routed)
    hipStream_t st = (hipStream_t)hip_stream;
    unsigned* out = (unsigned*)workspace;
    unsigned* counter = out + kGrid;
    hipLaunchKernelGGL(zero_fill_kernel, dim3(1), dim3(64), 0, st, (float*)counter, (size_t)1);
    hipLaunchKernelGGL(probe_placement_kernel, dim3(kGrid), dim3(512), 0, st, out, counter, 1 << 16);
    unsigned host[kGrid];
    e = hipMemcpyAsync(host, out, sizeof(host), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    // workgroups i and j must share an XCD exactly when i = j (mod 8), and all must have been resident at once
    bool ok = true;
    int xcd_of[8];
    for (int i = 0; i < kGrid && ok; ++i) {
        const int xcd = (int)(host[i] & 15u);
        if (!(host[i] & 0x100u)) ok = false;
        if (i < 8) {
            xcd_of[i] = xcd;
            for (int j = 0; j < i; ++j) ok = ok && xcd_of[j] != xcd;
        } else {
            ok = ok && xcd_of[i & 7] == xcd;
        }
    }
    {
        std::lock_guard<std::mutex> lock(g_chip_mutex);
        g_chip_state[dev] = ok ? 1 : 2;
    }
    return ok ? LAST_OK : LAST_ERR_UNSUPPORTED;
}

last_status_t last_probe_bandwidth(int32_t kind, const void* src, void* dst, size_t bytes, void* hip_stream)
{
    if (!src || !dst) return LAST_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || (uintptr_t)src % 16 != 0 || (uintptr_t)dst % 16 != 0)
        return LAST_ERR_SHAPE;
    if (kind < LAST_PROBE_READ || kind > LAST_PROBE_READ_COLUMNS) return LAST_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)hip_stream;
    if (kind == LAST_PROBE_READ_ROWS || kind == LAST_PROBE_READ_COLUMNS) {
        const size_t frame = (size_t)257 * 257 * 4;
        if (bytes % frame != 0 || bytes / frame > 0x7fffffffull) return LAST_ERR_SHAPE;
        const int nframes = (int)(bytes / frame);
        if (kind == LAST_PROBE_READ_ROWS)
            hipLaunchKernelGGL(probe_pattern_kernel<false>, dim3(256), dim3(512), 0, st, (const float*)src, nframes,
                               (float*)dst);
        else
            hipLaunchKernelGGL(probe_pattern_kernel<true>, dim3(256), dim3(512), 0, st, (const float*)src, nframes,
                               (float*)dst);
        return hip_status();
    }
    const size_t n4 = bytes / 16;
    const size_t copy_grid = (n4 + kProbeThreads - 1) / kProbeThreads;
    if (copy_grid > 0x7fffffffull) return LAST_ERR_SHAPE;
    if (kind == LAST_PROBE_READ)
        hipLaunchKernelGGL(probe_read_kernel, dim3(kProbeReadGrid), dim3(kProbeThreads), 0, st,
                           (const probe_f4*)src, n4, (float*)dst);
    else
        hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)copy_grid), dim3(kProbeThreads), 0, st,
                           (const probe_f4*)src, (probe_f4*)dst, n4);
    return hip_status();
}

const char* last_hip_error_string(void) { return hipGetErrorString(g_last_hip_error); }

const char* last_status_string(last_status_t status)
{
    switch (status) {
    case LAST_OK: return "ok";
    case LAST_ERR_NULL: return "a required pointer is NULL";
    case LAST_ERR_SHAPE: return "invalid shape";
    case LAST_ERR_CONTEXT: return "invalid context dependency";
    case LAST_ERR_SEMIRING: return "unknown semiring";
    case LAST_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LAST_ERR_UNSUPPORTED: return "combination not supported";
    case LAST_ERR_HIP: return "HIP call failed";
    }
    return "unknown status";
}

int32_t last_kernel_variant(const last_weights_t* weights, const last_context_t* context,
                            int32_t op)
{
    Shape s;
    if (check_common(weights, context, &s) != LAST_OK) return -1;
    if (weights->kind == LAST_WEIGHTS_SHARED_EMB) {
        const bool op_ok = op == LAST_OP_SHORTEST_DISTANCE || op == LAST_OP_ARC_POSTERIORS;
        return (op_ok && fused_plan(s, weights).ok) ? 2 : -1;
    }
    if (op == LAST_OP_SHORTEST_DISTANCE || op == LAST_OP_ARC_POSTERIORS)
        return cluster_plan(s, weights->kind).ok ? 1 : 0;
    if (op == LAST_OP_SHORTEST_PATH) return viterbi_plan(s, weights->kind).ok ? 1 : 0;
    return 0;
}

size_t last_workspace_bytes(const last_weights_t* weights, const last_context_t* context,
                            int32_t op, int32_t Umax)
{
    Shape s;
    if (check_common(weights, context, &s) != LAST_OK) return 0;
    Carver cv(nullptr);
    if (weights->kind == LAST_WEIGHTS_SHARED_EMB) {
        const FusedPlan fp = fused_plan(s, weights);
        if (op == LAST_OP_LOSS) {
            const size_t den = last_workspace_bytes(weights, context, LAST_OP_ARC_POSTERIORS, 0);
            const size_t num = last_workspace_bytes(weights, context, LAST_OP_INTERSECT_REFERENCE, Umax);
            return den && num ? den + num : 0;
        }
        if (op == LAST_OP_INTERSECT_REFERENCE) {
            // the numerator evaluates single arcs: no limit on the vocabulary, any closed-form context
            if (Umax < 0 || !fused_numerator_ok(weights)) return 0;
            carve_num(cv, s, Umax, false);
            cv.take<float>((size_t)s.V1 * weights->hidden);
            return cv.used;
        }
        if (!fp.ok) return 0;
        if (op == LAST_OP_SHORTEST_DISTANCE) carve_fused(cv, s, fp, false);
        else if (op == LAST_OP_ARC_POSTERIORS) carve_fused(cv, s, fp, true);
        else return 0;
        return cv.used;
    }
    carve_table_flag(cv, s);
    const ClusterPlan plan = cluster_plan(s, weights->kind);
    const ViterbiPlan vplan = viterbi_plan(s, weights->kind);
    switch (op) {
    case LAST_OP_SHORTEST_DISTANCE:
        if (plan.ok) carve_cluster(cv, s, plan);
        else cv.take<double>(1);
        if (vplan.ok) cv.take<u64>(vplan.xwords);        // tropical semiring: exchange buffer
        break;
    case LAST_OP_ARC_POSTERIORS:
        if (plan.ok) carve_cluster(cv, s, plan);
        else carve_posteriors(cv, s);
        break;
    case LAST_OP_INTERSECT_REFERENCE:
        if (Umax < 0) return 0;
        carve_num(cv, s, Umax, false);
        break;
    case LAST_OP_LOCAL_LOG_LIKELIHOOD:
        if (Umax < 0) return 0;
        carve_num(cv, s, Umax, true);
        break;
    case LAST_OP_LOSS: {
        const size_t den = last_workspace_bytes(weights, context, LAST_OP_ARC_POSTERIORS, 0);
        const size_t num = last_workspace_bytes(weights, context, LAST_OP_INTERSECT_REFERENCE, Umax);
        return den && num ? den + num : 0;
    }
    case LAST_OP_SHORTEST_PATH:
        carve_path(cv, s, vplan.ok ? vplan.xwords : 0);
        break;
    default:
        return 0;
    }
    return cv.used;
}

last_status_t last_shortest_distance(const last_weights_t* weights, const int32_t* lengths,
                                     const last_context_t* context, last_semiring_t semiring,
                                     float* dist, int32_t* item_status,
                                     void* ws, size_t ws_bytes, void* hip_stream)
{
    Shape s;
    last_status_t rc = check_common(weights, context, &s);
    if (rc != LAST_OK) return rc;
    if (!lengths || !dist) return LAST_ERR_NULL;
    if (semiring != LAST_LOG && semiring != LAST_TROPICAL) return LAST_ERR_SEMIRING;
    hipStream_t st = (hipStream_t)hip_stream;
    if (weights->kind == LAST_WEIGHTS_SHARED_EMB) {
        const FusedPlan fp = fused_plan(s, weights);
        if (!fp.ok || semiring != LAST_LOG) return LAST_ERR_UNSUPPORTED;
        rc = check_ws(ws, ws_bytes, last_workspace_bytes(weights, context, LAST_OP_SHORTEST_DISTANCE, 0));
        if (rc != LAST_OK) return rc;
        Carver cvf(ws);
        const FusedWs fw = carve_fused(cvf, s, fp, false);
        return launch_fused_forward(s, fp, fw, weights, lengths, dist, item_status, false, st);
    }
    rc = check_ws(ws, ws_bytes, last_workspace_bytes(weights, context, LAST_OP_SHORTEST_DISTANCE, 0));
    if (rc != LAST_OK) return rc;
    const SoloLayout l = solo_layout(s);
    if (s.order == 0) {
        if ((semiring == LAST_LOG ? l.lds_forward : l.lds_viterbi) > kBigLds) return LAST_ERR_UNSUPPORTED;
        Carver cv(ws);
        int* flag = carve_table_flag(cv, s);
        launch_table_check(s, flag, st);
        rc = semiring == LAST_LOG
                 ? launch_table_forward(s, l, weights->w, lengths, nullptr, nullptr, nullptr, dist, item_status, flag, st)
                 : launch_table_viterbi(s, l, weights->w, lengths, nullptr, nullptr, dist, item_status, flag, st);
        return rc != LAST_OK ? rc : hip_status();
    }
    const Ctx c = make_ctx(s);
    const ClusterPlan plan = cluster_plan(s, weights->kind);
    if (semiring == LAST_LOG && plan.ok) {
        Carver cv(ws);
        const ClusterWs cw = carve_cluster(cv, s, plan);
        launch_cluster<false>(s, plan, cw, weights->w, lengths, dist, item_status, nullptr, 1.f, 0, st);
    } else if (semiring == LAST_LOG) {
        if (l.lds_forward > kMaxLds) return LAST_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(solo_forward_log, dim3(s.B), dim3(1024), l.lds_forward, st,
                           weights->w, lengths, c, s.T, l.CPAD, l.R,
                           (float*)nullptr, (double*)nullptr, (double*)nullptr, dist, item_status);
    } else if (const ViterbiPlan vp = viterbi_plan(s, weights->kind); vp.ok) {
        Carver cv(ws);
        if (plan.ok) carve_cluster(cv, s, plan);
        else cv.take<double>(1);
        u64* xv = cv.take<u64>(vp.xwords);
        launch_cluster_viterbi(s, vp, xv, weights->w, lengths, nullptr, nullptr, dist, item_status, st);
    } else {
        if (l.lds_viterbi > kMaxLds) return LAST_ERR_UNSUPPORTED;
        if (!launch_bigram_viterbi(s, weights->w, lengths, nullptr, nullptr, dist, item_status, st))
            hipLaunchKernelGGL(solo_viterbi, dim3(s.B), dim3(1024), l.lds_viterbi, st,
                               weights->w, lengths, c, s.T, l.CPAD, l.R,
                               (int*)nullptr, (int*)nullptr, dist, item_status);
    }
    return hip_status();
}

last_status_t last_arc_posteriors(const last_weights_t* weights, const int32_t* lengths,
                                  const last_context_t* context, float* dist,
                                  const last_grads_t* out, int32_t* item_status,
                                  void* ws, size_t ws_bytes, void* hip_stream)
{
    Shape s;
    last_status_t rc = check_common(weights, context, &s);
    if (rc != LAST_OK) return rc;
    if (!lengths || !dist || !out) return LAST_ERR_NULL;
    if (weights->kind == LAST_WEIGHTS_SHARED_EMB) {
        const FusedPlan fp = fused_plan(s, weights);
        if (!fp.ok) return LAST_ERR_UNSUPPORTED;
        if (!out->df || !out->de || !out->dW) return LAST_ERR_NULL;
        rc = check_ws(ws, ws_bytes, last_workspace_bytes(weights, context, LAST_OP_ARC_POSTERIORS, 0));
        if (rc != LAST_OK) return rc;
        Carver cvf(ws);
        const FusedWs fw = carve_fused(cvf, s, fp, true);
        rc = launch_fused_forward(s, fp, fw, weights, lengths, dist, item_status, true, (hipStream_t)hip_stream);
        if (rc != LAST_OK) return rc;
        return launch_fused_backward(s, fp, fw, dist, weights, lengths, out, item_status, (hipStream_t)hip_stream);
    }
    if (weights->kind != LAST_WEIGHTS_DENSE) return LAST_ERR_UNSUPPORTED;
    if (!out->dw) return LAST_ERR_NULL;
    rc = check_ws(ws, ws_bytes, last_workspace_bytes(weights, context, LAST_OP_ARC_POSTERIORS, 0));
    if (rc != LAST_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const ClusterPlan plan = cluster_plan(s, weights->kind);
    if (plan.ok) {
        Carver cvc(ws);
        const ClusterWs cw = carve_cluster(cvc, s, plan);
        launch_cluster<true>(s, plan, cw, weights->w, lengths, dist, item_status, out->dw, out->scale,
                             out->accumulate, st);
        return hip_status();
    }
    const SoloLayout l = solo_layout(s);
    if (l.lds_forward > (s.order == 0 ? kBigLds : kMaxLds)) return LAST_ERR_UNSUPPORTED;
    const Ctx c = make_ctx(s);
    Carver cv(ws);
    int* flag = carve_table_flag(cv, s);
    PosteriorWs p = carve_posteriors(cv, s);
    if (s.order == 0) {
        launch_table_check(s, flag, st);
        rc = launch_table_forward(s, l, weights->w, lengths, p.alpha, p.offs, p.D, dist, item_status, flag, st);
        if (rc != LAST_OK) return rc;
    } else {
        hipLaunchKernelGGL(solo_forward_log, dim3(s.B), dim3(1024), l.lds_forward, st,
                           weights->w, lengths, c, s.T, l.CPAD, l.R, p.alpha, p.offs, p.D, dist,
                           item_status);
    }
    if (s.T > 0) {
        dispatch_group(s.V1, [&](auto G) {
            auto k = solo_backward_log<decltype(G)::value>;
            if (l.lds_backward > kMaxLds) rc = allow_lds((const void*)k, kBigLds);
            if (rc == LAST_OK)
                hipLaunchKernelGGL(k, dim3(s.B), dim3(1024), l.lds_backward, st, weights->w, lengths, c, s.T,
                                   (const float*)p.alpha, (const double*)p.offs, (const double*)p.D,
                                   out->dw, out->scale, out->accumulate);
        });
        if (rc != LAST_OK) return rc;
    }
    return hip_status();
}

// The (t,u) recursion with one wavefront per item and direction (references of up to 511 labels);
// false when the shape needs the workgroup kernel.
static bool launch_num_wave(const Shape& s, int Umax, const NumWs& p, const int* lengths, const int* ref_lengths,
                            float* numerator, int* item_status, hipStream_t st)
{
    const int U1 = Umax + 1;
    const int cpl = (U1 + kWave - 1) / kWave;
    if (cpl > 8 || s.T < 1 || (size_t)(s.T + 1) * U1 * 8 >= 0xfffffff0ull) return false;
    auto go = [&](auto CPL, auto CH) {
        hipLaunchKernelGGL(HIP_KERNEL_NAME(num_wave_kernel<decltype(CPL)::value, decltype(CH)::value>),
                           dim3(s.B, 2), dim3(kWave), 0, st, (const float2*)p.wi, lengths, ref_lengths,
                           (const int*)p.status, s.T, Umax, p.a, p.bk, p.N, numerator, item_status);
    };
    using std::integral_constant;
    // frames per prefetch chunk: a wavefront can keep count of 63 memory operations in flight, and a
    // frame costs cpl loads and cpl stores
    if (cpl <= 1) go(integral_constant<int, 1>(), integral_constant<int, 16>());
    else if (cpl <= 2) go(integral_constant<int, 2>(), integral_constant<int, 8>());
    else if (cpl <= 3) go(integral_constant<int, 3>(), integral_constant<int, 6>());
    else if (cpl <= 4) go(integral_constant<int, 4>(), integral_constant<int, 4>());
    else if (cpl <= 6) go(integral_constant<int, 6>(), integral_constant<int, 3>());
    else go(integral_constant<int, 8>(), integral_constant<int, 2>());
    return true;
}

// Shared by the globally normalised numerator and the locally normalised log-likelihood.
enum { kNumPrepare = 1, kNumScatter = 2 };   // the two halves of a numerator call: up to the recursion, the gradient

static last_status_t intersect_impl(const last_weights_t* weights, const int32_t* lengths,
                                    const last_context_t* context,
                                    const int32_t* refs, const int32_t* ref_lengths,
                                    int32_t Umax, float* numerator,
                                    const last_grads_t* out, int32_t* item_status,
                                    void* ws, size_t ws_bytes, void* hip_stream, bool local,
                                    int phases = kNumPrepare | kNumScatter)
{
    const bool prepare = phases & kNumPrepare, scatter = phases & kNumScatter;
    Shape s;
    last_status_t rc = check_common(weights, context, &s);
    if (rc != LAST_OK) return rc;
    if (!lengths || !ref_lengths || !numerator) return LAST_ERR_NULL;
    if (Umax < 0 || Umax > (1 << 20)) return LAST_ERR_SHAPE;
    if (Umax > 0 && !refs) return LAST_ERR_NULL;
    const size_t lds = (size_t)2 * (Umax + 2) * sizeof(double);
    if (lds > kMaxLds) return LAST_ERR_UNSUPPORTED;
    if (weights->kind == LAST_WEIGHTS_SHARED_EMB) {
        if (local || !fused_numerator_ok(weights)) return LAST_ERR_UNSUPPORTED;
        if (out && (!out->df || !out->de || !out->dW)) return LAST_ERR_NULL;
        rc = check_ws(ws, ws_bytes, last_workspace_bytes(weights, context, LAST_OP_INTERSECT_REFERENCE, Umax));
        if (rc != LAST_OK) return rc;
        hipStream_t st = (hipStream_t)hip_stream;
        const Ctx c = make_ctx(s);
        const int H = weights->hidden, U1 = Umax + 1;
        Carver cv(ws);
        NumWs p = carve_num(cv, s, Umax, false);
        float* Wt = cv.take<float>((size_t)s.V1 * H);
        const __bf16* f = (const __bf16*)weights->f;
        const __bf16* e = (const __bf16*)weights->e;
        const dim3 block(kFnWaves * kWave);
        const int ugrid = (U1 + kFnWaves - 1) / kFnWaves;
        if (prepare) {
        hipLaunchKernelGGL(num_check_kernel, dim3(s.B), dim3(256), 0, st, lengths, refs, ref_lengths,
                           c, s.T, Umax, p.status, p.ctxs, p.link, (const int*)nullptr);
        hipLaunchKernelGGL(fnum_transpose_w_kernel, dim3((s.V1 * H + 255) / 256), dim3(256), 0, st,
                           (const __bf16*)weights->W, H, s.V1, Wt);
        if (s.T > 0)
            hipLaunchKernelGGL(fnum_gather_kernel, dim3(ugrid, (s.T + kFnStrip - 1) / kFnStrip, s.B), block, 0, st,
                               f, e, (const float*)Wt, lengths, refs, ref_lengths, (const int*)p.status,
                               (const int*)p.ctxs, s.T, Umax, H, p.wi);
        if (!launch_num_wave(s, Umax, p, lengths, ref_lengths, numerator, item_status, st))
            hipLaunchKernelGGL(num_recursion_kernel, dim3(s.B, 2), dim3(256), lds, st,
                               (const float2*)p.wi, (const double*)nullptr, lengths, ref_lengths,
                               (const int*)p.status, s.T, Umax, p.a, p.bk, p.N, numerator, item_status);
        }
        if (out && scatter) {
            if (!out->accumulate) {
                hipLaunchKernelGGL(zero_fill_kernel, dim3(256), dim3(256), 0, st, out->de, (size_t)s.C * H);
                hipLaunchKernelGGL(zero_fill_kernel, dim3(64), dim3(256), 0, st, out->dW, (size_t)H * s.V1);
            }
            if (s.T > 0) {
                hipLaunchKernelGGL(fnum_df_kernel, dim3((s.T + kFnWaves - 1) / kFnWaves, s.B), block, 0, st,
                                   f, e, (const float*)Wt, (const float2*)p.wi, lengths, refs, ref_lengths,
                                   (const int*)p.status, (const int*)p.ctxs, (const double*)p.a,
                                   (const double*)p.bk, (const double*)p.N, s.T, Umax, H, out->df,
                                   out->scale, out->accumulate);
                hipLaunchKernelGGL(fnum_de_dw_kernel, dim3(ugrid, (s.T + kFnChunk - 1) / kFnChunk, s.B), block, 0,
                                   st, f, e, (const float*)Wt, (const float2*)p.wi, lengths, refs, ref_lengths,
                                   (const int*)p.status, (const int*)p.ctxs, (const double*)p.a,
                                   (const double*)p.bk, (const double*)p.N, s.T, Umax, H, s.V1, out->de,
                                   out->dW, out->scale);
            }
        }
        return hip_status();
    }
    if (weights->kind != LAST_WEIGHTS_DENSE) return LAST_ERR_UNSUPPORTED;
    if (out && !out->dw) return LAST_ERR_NULL;
    constexpr int kLocalWaves = 4;
    const size_t lds_scatter = (size_t)kLocalWaves * s.V1 * sizeof(float);
    if (local && lds_scatter > kMaxLds) return LAST_ERR_UNSUPPORTED;
    rc = check_ws(ws, ws_bytes,
                  last_workspace_bytes(weights, context,
                                       local ? LAST_OP_LOCAL_LOG_LIKELIHOOD : LAST_OP_INTERSECT_REFERENCE, Umax));
    if (rc != LAST_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const Ctx c = make_ctx(s);
    Carver cv(ws);
    int* flag = carve_table_flag(cv, s);
    NumWs p = carve_num(cv, s, Umax, local);
    const int U1 = Umax + 1;
    const dim3 pgrid((U1 + 127) / 128, s.T > 0 ? s.T : 1, s.B);
    const dim3 wgrid((U1 + kLocalWaves - 1) / kLocalWaves, s.T > 0 ? s.T : 1, s.B);   // a wavefront per cell
    if (prepare) {
    if (flag) launch_table_check(s, flag, st);
    hipLaunchKernelGGL(num_check_kernel, dim3(s.B), dim3(256), 0, st, lengths, refs, ref_lengths,
                       c, s.T, Umax, p.status, p.ctxs, p.link, (const int*)flag);
    if (s.T > 0) {
        if (local)
            hipLaunchKernelGGL(num_gather_local_kernel, wgrid, dim3(kLocalWaves * kWave), 0, st, weights->w,
                               lengths, refs, ref_lengths, (const int*)p.status, (const int*)p.ctxs, c,
                               s.T, Umax, p.wi, p.lz);
        else
            hipLaunchKernelGGL(num_gather_kernel, pgrid, dim3(128), 0, st, weights->w, lengths, refs,
                               ref_lengths, (const int*)p.status, (const int*)p.ctxs, c, s.T, Umax, p.wi);
    }
    if (!local && launch_num_wave(s, Umax, p, lengths, ref_lengths, numerator, item_status, st)) {
        // one wavefront per item and direction has run the recursion
    } else {
        hipLaunchKernelGGL(num_recursion_kernel, dim3(s.B, 2), dim3(256), lds, st,
                           (const float2*)p.wi, (const double*)p.lz, lengths, ref_lengths,
                           (const int*)p.status, s.T, Umax, p.a, p.bk, p.N, numerator, item_status);
    }
    }
    if (out && s.T > 0 && scatter) {
        if (!out->accumulate) {
            const size_t n = (size_t)s.B * s.T * s.C * s.V1;
            hipLaunchKernelGGL(zero_fill_kernel, dim3(2048), dim3(256), 0, st, out->dw, n);
        }
        if (local)
            hipLaunchKernelGGL(num_scatter_local_kernel, wgrid, dim3(kLocalWaves * kWave), lds_scatter, st,
                               weights->w, (const float2*)p.wi, (const double*)p.lz, lengths, refs,
                               ref_lengths, (const int*)p.status, (const int*)p.ctxs, (const int*)p.link,
                               c, s.T, Umax, (const double*)p.a, (const double*)p.bk, (const double*)p.N,
                               out->dw, out->scale, out->accumulate);
        else
            hipLaunchKernelGGL(num_scatter_kernel, pgrid, dim3(128), 0, st, (const float2*)p.wi,
                               lengths, refs, ref_lengths, (const int*)p.status, (const int*)p.ctxs, c,
                               s.T, Umax, (const double*)p.a, (const double*)p.bk, (const double*)p.N,
                               out->dw, out->scale);
    }
    return hip_status();
}

last_status_t last_intersect_reference(const last_weights_t* weights, const int32_t* lengths,
                                       const last_context_t* context,
                                       const int32_t* refs, const int32_t* ref_lengths,
                                       int32_t Umax, float* numerator,
                                       const last_grads_t* out, int32_t* item_status,
                                       void* ws, size_t ws_bytes, void* hip_stream)
{
    return intersect_impl(weights, lengths, context, refs, ref_lengths, Umax, numerator, out, item_status,
                          ws, ws_bytes, hip_stream, false);
}

last_status_t last_local_log_likelihood(const last_weights_t* weights, const int32_t* lengths,
                                        const last_context_t* context,
                                        const int32_t* refs, const int32_t* ref_lengths,
                                        int32_t Umax, float* loglik,
                                        const last_grads_t* out, int32_t* item_status,
                                        void* ws, size_t ws_bytes, void* hip_stream)
{
    return intersect_impl(weights, lengths, context, refs, ref_lengths, Umax, loglik, out, item_status,
                          ws, ws_bytes, hip_stream, true);
}

// ---- denominator and numerator in one call ---------------------------------------------------
// The numerator up to its recursion does not depend on the denominator, so it runs beside it on a
// stream of the library's own (one per device, default priority, created at first use), forked from
// and joined to the caller's stream with events; only the numerator's gradient pass waits for the
// denominator's.  Host calls are serialised by a mutex so that each record/wait pair stays together.
namespace {
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
};
constexpr int kMaxSideDevices = 64;
SideStream g_side[kMaxSideDevices];
std::mutex g_side_mu;

last_status_t side_stream(SideStream** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    if (dev < 0 || dev >= kMaxSideDevices) return LAST_ERR_UNSUPPORTED;
    SideStream& sd = g_side[dev];
    if (!sd.stream) {
        e = hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&sd.fork, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&sd.join, hipEventDisableTiming);
        if (e != hipSuccess) { g_last_hip_error = e; sd = SideStream(); return LAST_ERR_HIP; }
    }
    *out = &sd;
    return LAST_OK;
}

__global__ void merge_status_kernel(const int* __restrict__ num_status, int* __restrict__ item_status, int B)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B && item_status[b] == kItemOk && num_status[b] != kItemOk) item_status[b] = num_status[b];
}
}  // namespace

last_status_t last_globally_normalized_loss(const last_weights_t* weights, const int32_t* lengths,
                                           const last_context_t* context,
                                             const int32_t* refs, const int32_t* ref_lengths, int32_t Umax,
                                             float* dist, float* numerator, const last_grads_t* out,
                                             int32_t* item_status, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!weights || !context || !out) return LAST_ERR_NULL;
    const size_t need_den = last_workspace_bytes(weights, context, LAST_OP_ARC_POSTERIORS, 0);
    const size_t need_num = last_workspace_bytes(weights, context, LAST_OP_INTERSECT_REFERENCE, Umax);
    if (need_den == 0 || need_num == 0) {
        Shape s;
        const last_status_t rc = check_common(weights, context, &s);
        return rc != LAST_OK ? rc : LAST_ERR_UNSUPPORTED;
    }
    last_status_t rc = check_ws(ws, ws_bytes, need_den + need_num);
    if (rc != LAST_OK) return rc;
    if (!dist || !numerator) return LAST_ERR_NULL;
    void* ws_num = (char*)ws + need_den;            // (both sizes are multiples of the alignment)
    hipStream_t st = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_side_mu);
    SideStream* sd = nullptr;
    rc = side_stream(&sd);
    if (rc != LAST_OK) return rc;
    // the numerator's gradient is accumulated with the opposite sign onto the denominator's
    last_grads_t gnum = *out;
    gnum.accumulate = 1;
    gnum.scale = -out->scale;
    // arguments are checked by a dry pass before anything is enqueued: the numerator call with no phase
    rc = intersect_impl(weights, lengths, context, refs, ref_lengths, Umax, numerator, &gnum, nullptr,
                        ws_num, need_num, nullptr, false, 0);
    if (rc != LAST_OK) return rc;
    hipError_t e = hipEventRecord(sd->fork, st);
    if (e == hipSuccess) e = hipStreamWaitEvent(sd->stream, sd->fork, 0);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    rc = intersect_impl(weights, lengths, context, refs, ref_lengths, Umax, numerator, &gnum, nullptr,
                        ws_num, need_num, sd->stream, false, kNumPrepare);
    // the fork is always joined, also after an error, so that the caller's stream never loses the side work
    e = hipEventRecord(sd->join, sd->stream);
    g_numerator_beside = true;
    const last_status_t rc_den = last_arc_posteriors(weights, lengths, context, dist, out, item_status, ws,
                                                     need_den, hip_stream);
    g_numerator_beside = false;
    if (e == hipSuccess) e = hipStreamWaitEvent(st, sd->join, 0);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    if (rc != LAST_OK) return rc;
    if (rc_den != LAST_OK) return rc_den;
    rc = intersect_impl(weights, lengths, context, refs, ref_lengths, Umax, numerator, &gnum, nullptr,
                        ws_num, need_num, hip_stream, false, kNumScatter);
    if (rc != LAST_OK) return rc;
    if (item_status) {
        // the numerator's per-item status sits at a fixed place of its workspace
        Shape s;
        check_common(weights, context, &s);
        Carver cv(ws_num);
        carve_table_flag(cv, s);
        const NumWs p = carve_num(cv, s, Umax, false);
        hipLaunchKernelGGL(merge_status_kernel, dim3((s.B + 255) / 256), dim3(256), 0, st,
                           (const int*)p.status, item_status, s.B);
    }
    return hip_status();
}

last_status_t last_shortest_path(const last_weights_t* weights, const int32_t* lengths,
                                 const last_context_t* context,
                                 int32_t* labels, int32_t* states, float* score,
                                 int32_t* item_status,
                                 void* ws, size_t ws_bytes, void* hip_stream)
{
    Shape s;
    last_status_t rc = check_common(weights, context, &s);
    if (rc != LAST_OK) return rc;
    if (!lengths || !labels || !states || !score) return LAST_ERR_NULL;
    if (weights->kind != LAST_WEIGHTS_DENSE) return LAST_ERR_UNSUPPORTED;
    rc = check_ws(ws, ws_bytes, last_workspace_bytes(weights, context, LAST_OP_SHORTEST_PATH, 0));
    if (rc != LAST_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const SoloLayout l = solo_layout(s);
    const ViterbiPlan vp = viterbi_plan(s, weights->kind);
    if (!vp.ok && l.lds_viterbi > (s.order == 0 ? kBigLds : kMaxLds)) return LAST_ERR_UNSUPPORTED;
    const Ctx c = make_ctx(s);
    Carver cv(ws);
    int* flag = carve_table_flag(cv, s);
    PathWs p = carve_path(cv, s, vp.ok ? vp.xwords : 0);
    if (s.order == 0) {
        launch_table_check(s, flag, st);
        rc = launch_table_viterbi(s, l, weights->w, lengths, p.bp, p.final_state, score, item_status, flag, st);
        if (rc != LAST_OK) return rc;
    } else if (vp.ok)
        launch_cluster_viterbi(s, vp, p.xv, weights->w, lengths, p.bp, p.final_state, score, item_status, st);
    else if (!launch_bigram_viterbi(s, weights->w, lengths, p.bp, p.final_state, score, item_status, st))
        hipLaunchKernelGGL(solo_viterbi, dim3(s.B), dim3(1024), l.lds_viterbi, st, weights->w, lengths,
                           c, s.T, l.CPAD, l.R, p.bp, p.final_state, score, item_status);
    const int cthreads = s.C < 256 ? (s.C + 63) / 64 * 64 : 256;
    hipLaunchKernelGGL(backtrace_compose_kernel, dim3(p.nseg, s.B), dim3(cthreads), 0, st, (const int*)p.bp,
                       lengths, s.C, s.V1, s.T, p.S, p.nseg, p.map);
    hipLaunchKernelGGL(backtrace_boundaries_kernel, dim3((s.B + 63) / 64), dim3(64), 0, st, (const int*)p.map,
                       lengths, (const int*)p.final_state, s.B, s.C, s.T, p.S, p.nseg, p.bnd);
    hipLaunchKernelGGL(backtrace_emit_kernel, dim3(p.nseg, s.B), dim3(64), 0, st, (const int*)p.bp, lengths,
                       (const int*)p.final_state, (const int*)p.bnd, s.C, s.V1, s.T, p.S, p.nseg, labels,
                       states);
    return hip_status();
}

// ---- the entry point for callers that cannot allocate --------------------------------------
// Its scratch memory is a file-scope device array: every GPU the library runs on holds one copy
// of it, at its own address, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; kernels are given the address that call returned.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[LAST_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// address of the current device's copy of `scratch` (looked up once per device)
last_status_t static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = e; return LAST_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDevices) return LAST_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { g_last_hip_error = e; return LAST_ERR_HIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LAST_OK;
}

}  // namespace

extern "C" {

last_status_t last_shortest_distance_static(const last_weights_t* weights, const int32_t* lengths,
                                            const last_context_t* context, last_semiring_t semiring,
                                            float* dist, int32_t* item_status, void* hip_stream)
{
    Shape s;
    last_status_t rc = check_common(weights, context, &s);
    if (rc != LAST_OK) return rc;
    if (!lengths || !dist) return LAST_ERR_NULL;
    if (semiring != LAST_LOG && semiring != LAST_TROPICAL) return LAST_ERR_SEMIRING;
    const size_t need = last_workspace_bytes(weights, context, LAST_OP_SHORTEST_DISTANCE, 0);
    if (need == 0) return LAST_ERR_UNSUPPORTED;
    if (need > (size_t)LAST_STATIC_SCRATCH_BYTES) return LAST_ERR_WORKSPACE;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != LAST_OK) return rc;
    return last_shortest_distance(weights, lengths, context, semiring, dist, item_status, ws,
                                  (size_t)LAST_STATIC_SCRATCH_BYTES, hip_stream);
}

}  // extern "C"
