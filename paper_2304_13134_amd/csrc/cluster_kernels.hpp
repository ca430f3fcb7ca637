// Clustered forward-backward for the bigram (context size 1) complete lattice
// with dense weights: the bandwidth path.
//
// The recursion of Eq. 2 (arXiv 2304.13134) is serial in t, but a single frame
// of one item is a C x C slab (264 KB at C = 257), far more than one compute
// unit can stream.  Each item is therefore spread over a cluster of 2K
// persistent workgroups that live on one XCD (workgroup ids are dealt
// round-robin over the 8 XCDs, so a cluster takes ids with equal id % 8):
//   K "alpha" workgroups run the forward weights from frame 0 upwards,
//   K "beta"  workgroups run the backward weights from frame len-1 downwards,
// both at the same time.  They meet in the middle: once alpha has reached
// frame mid = len/2 and beta has come down to it, D is known
// (D = log sum_q alpha_mid[q] beta_mid[q]) and each side keeps going over the
// other half, now also writing the arc marginals of Eq. 1 against the state
// vectors the other side stored on its way (forward-backward with O(|Q|)
// extra space, Section 4.2.2).  Every weight is read twice and every marginal
// written once (12 bytes per arc) in len serial steps instead of 2 len.
//
// Work split inside a role: workgroup k owns the source states (rows)
// [k*RPW, (k+1)*RPW) of every frame, a contiguous chunk of memory.
//   alpha: thread <-> destination column (two half-workgroups of 5 waves share
//          the rows); partial column sums over the own rows are exchanged
//          (reduce-scatter: workgroup k only needs the sums for its own states);
//   beta : wavefront <-> row, lanes <-> columns; complete row sums are
//          exchanged (all-gather).
// Arithmetic is in the scaled linear domain: E = 2^(w*log2(e) - s) with an
// integer shift s per column (alpha) or per row (beta) chosen from the data so
// that E <= 1; state vectors carry a common integer binary exponent (Sa, Sb)
// that advances by a predicted amount P every step, P being derived from the
// magnitudes seen one or two steps earlier so that all workgroups agree on it
// without an extra round trip.  exp(w) does not depend on the recursion, so it
// is evaluated while the previous step's exchange is in flight; the serial
// chain per frame is: FMA loop, publish, poll, add.
//
// Exchange: 64-bit words [value:32 | tag:32] written with relaxed agent-scope
// atomic stores; the tag (a running step counter) makes each word
// self-validating, so no fences are needed on the per-frame path.  Two slots
// (step parity) suffice: nobody can publish step s+2 before everybody has
// consumed step s.  Words are polled through the SCALAR memory path (64-byte
// scalar loads that bypass the scalar cache): the vector memory pipeline
// returns loads in order, so a vector poll would queue behind the streaming
// loads of the same compute unit, while the scalar path is independent of
// them.  This needs the cluster on one XCD (one L2); if the placement ever
// differs the polls time out and the item reports status 5 instead of a
// wrong result.  Every poll loop is bounded.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace last {

typedef unsigned long long u64;

constexpr int kClMaxR = 40;      // LDS row slots per workgroup and parity: rows 0..16 at [0..16],
                                 // rows 17..33 at [20..36], so that both halves start 16-byte aligned
__device__ __forceinline__ int lds_row(int r) { return r < 17 ? r : r + 3; }
constexpr int kClRT = 17;        // rows per alpha thread: each workgroup splits its rows in two halves
constexpr int kClHW = 5;         // compute waves per half (alpha): 5 * 64 >= kClMaxC columns
constexpr int kClWaves = 10;     // compute waves per workgroup
constexpr int kClRW = 4;         // max rows per compute wave (beta): ceil(34 / 10)
constexpr int kClNC = 5;         // max columns per lane (beta): ceil(320 / 64)
constexpr int kClMaxC = 264;     // max number of states / labels on this path (11 waves x 24 words)
constexpr int kClThreads = (kClWaves + 1) * kWave;
constexpr int kClMaxK = 8;       // max workgroups per role
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kShiftNone = -30000;
constexpr int kClXK = 8;         // words per exchange row (alpha): one 64-byte scalar load
constexpr int kClAuxDelay = 4;   // units of 256 clocks the polling wave waits before its first look (measured best)
constexpr int kClCH = 24;        // exchange words gathered per wave: three 64-byte scalar loads
constexpr int kClLds = 2 * kClMaxR * 2 + 2 * 320 + 320 + 64 + 32 + 64;   // floats


struct ClusterArgs {
    const float* w;
    const int* len;
    float* dw;
    float* dist;
    int* item_status;
    float* ahat;   // [B][T+1][C] forward vectors (scaled), rows t <= mid
    float* bhat;   // [B][T+1][C] backward vectors (scaled), rows t >= mid
    int* Sa;       // [B][T+1] binary exponent of ahat rows
    int* Sb;       // [B][T+1]
    u64* xa;       // [ncl_total][2][XS][2K] alpha partials: row = destination (row C = headers),
                   //                        column = producer half-workgroup
    u64* xb;       // [ncl_total][2][XSB]   beta values
    u64* ph;       // [ncl_total][32]       phase flags
    u64* fin;      // [B][2]                third generation: workgroups through with an item, time-out mark
    int B, T, C;
    int K, RPW, ncl;   // workgroups per role, rows per workgroup, clusters per XCD
    int XS, XSB;
    float scale;
    int accumulate;
    int spin_limit;
};

// ---- cross-lane helpers on DPP (the critical path cannot afford LDS permutes)
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_f(float old, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL,
                                                      ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_i(int old, int v)
{
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}
// full-wave sum / max, result broadcast to every lane
__device__ __forceinline__ float wave_sum_dpp(float v)
{
    v += dpp_f<0x111>(0.f, v);
    v += dpp_f<0x112>(0.f, v);
    v += dpp_f<0x114>(0.f, v);
    v += dpp_f<0x118>(0.f, v);
    v += dpp_f<0x142, 0xa>(0.f, v);
    v += dpp_f<0x143, 0xc>(0.f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_dpp(float v)
{
    v = fmaxf(v, dpp_f<0x111>(v, v));
    v = fmaxf(v, dpp_f<0x112>(v, v));
    v = fmaxf(v, dpp_f<0x114>(v, v));
    v = fmaxf(v, dpp_f<0x118>(v, v));
    v = fmaxf(v, dpp_f<0x142, 0xa>(v, v));
    v = fmaxf(v, dpp_f<0x143, 0xc>(v, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ int wave_max_dpp(int v)
{
    v = max(v, dpp_i<0x111>(v, v));
    v = max(v, dpp_i<0x112>(v, v));
    v = max(v, dpp_i<0x114>(v, v));
    v = max(v, dpp_i<0x118>(v, v));
    v = max(v, dpp_i<0x142, 0xa>(v, v));
    v = max(v, dpp_i<0x143, 0xc>(v, v));
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ u64 xload(const u64* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void xstore(u64* p, u64 v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Per-frame publish: a plain 8-byte store that lands in the XCD's L2, where the scalar-path
// polls of the other workgroups of the cluster read it.  (An agent-scope store would be written
// through to memory, one partial line at a time.)
__device__ __forceinline__ void xpublish(u64* p, u64 v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ u64 pack_word(float v, unsigned tag)
{
    return (u64)__float_as_uint(v) | ((u64)tag << 32);
}
__device__ __forceinline__ u64 pack_int(int v, unsigned tag)
{
    return (u64)(unsigned)v | ((u64)tag << 32);
}

__device__ __forceinline__ int float_exponent(float x)   // floor(log2 x) for normal x > 0; -127 for 0
{
    return (int)((__float_as_uint(x) >> 23) & 0xFFu) - 127;
}
__device__ __forceinline__ int shift_for(float mx)        // integer s >= mx*log2(e)
{
    if (!(mx > -3.0e4f)) return kShiftNone;
    float s = ceilf(mx * kLog2e);
    return (int)fminf(s, 30000.f);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Streaming access through buffer descriptors: one descriptor per item (4 scalar registers),
// a loop-invariant 32-bit per-thread byte offset and a scalar per-frame byte offset.  This keeps
// the address arithmetic of the 17-20 loads per thread and frame out of the vector registers.
#ifndef LAST_LOAD_AUX
#define LAST_LOAD_AUX 0    // cache policy of the streaming loads (2 = non-temporal measured slower)
#endif
#ifndef LAST_STORE_AUX
#define LAST_STORE_AUX 0   // cache policy of the streaming stores
#endif
typedef __amdgpu_buffer_rsrc_t buf_t;
__device__ __forceinline__ buf_t make_buf(const void* p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load_nt(buf_t r, unsigned voff, unsigned soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, LAST_LOAD_AUX));
}
__device__ __forceinline__ void buf_store_nt(float v, buf_t r, unsigned voff, unsigned soff)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, LAST_STORE_AUX);
}
__device__ __forceinline__ float buf_load(buf_t r, unsigned voff, unsigned soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}
__device__ __forceinline__ void buf_store(float v, buf_t r, unsigned voff, unsigned soff)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, 0);
}

// ---- scalar-path gathers -------------------------------------------------------
// Three (or four) 64-byte scalar loads that bypass the scalar cache, issued and
// awaited inside one asm statement so that no compiler-generated code can touch
// the destination registers while the loads are in flight.
typedef unsigned v16u __attribute__((ext_vector_type(16)));
__device__ __forceinline__ void sgather3(const void* p, v16u& a, v16u& b, v16u& c)
{
    asm volatile("s_load_dwordx16 %0, %3, 0x0 glc\n\t"
                 "s_load_dwordx16 %1, %3, 0x40 glc\n\t"
                 "s_load_dwordx16 %2, %3, 0x80 glc\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&s"(a), "=&s"(b), "=&s"(c) : "s"(p) : "memory");
}
__device__ __forceinline__ void sgather4(const void* p, const void* q, v16u& a, v16u& b, v16u& c, v16u& d)
{
    asm volatile("s_load_dwordx16 %0, %4, 0x0 glc\n\t"
                 "s_load_dwordx16 %1, %4, 0x40 glc\n\t"
                 "s_load_dwordx16 %2, %4, 0x80 glc\n\t"
                 "s_load_dwordx16 %3, %5, 0x0 glc\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&s"(a), "=&s"(b), "=&s"(c), "=&s"(d) : "s"(p), "s"(q) : "memory");
}
// number of leading words (of 8) whose tag matches, and their sum in fixed order
__device__ __forceinline__ bool block_ready(const v16u& v, int count, unsigned tag)
{
    bool ok = true;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < count && v[2 * j + 1] != tag) ok = false;
    return ok;
}
__device__ __forceinline__ float block_sum8(const v16u& v, int count)
{
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < count) s += __uint_as_float(v[2 * j]);
    return s;
}

struct ClusterGeom {
    int role;     // 0 alpha, 1 beta
    int k;        // workgroup index inside the role
    int cg;       // global cluster index
    int r0, nr;   // owned rows
};

// poll one word (vector path; only used outside the per-frame loop)
__device__ __forceinline__ bool poll_flag(const u64* p, u64 target, int limit)
{
    for (int n = 0; n <= limit; ++n) {
        const u64 x = xload(p);
        if (x != ~0ull && x >= target) return true;
        __builtin_amdgcn_s_sleep(2);
    }
    return false;
}

// barrier among the 2K workgroups of a cluster with release/acquire semantics
// for plain global stores (used once per item, at the meeting frame)
__device__ __forceinline__ void cluster_sync(const ClusterArgs& a, const ClusterGeom& g, unsigned tag,
                                             int* dead_s)
{
    __threadfence();
    __syncthreads();
    u64* flags = a.ph + (size_t)g.cg * 32;
    const int me = g.role * a.K + g.k;
    const u64 target = (u64)tag + 1;          // flags count items; ~0 = never written
    if (threadIdx.x == 0) xstore(flags + me, target);
    if ((int)threadIdx.x < 2 * a.K && !*dead_s)
        if (!poll_flag(flags + threadIdx.x, target, a.spin_limit)) *dead_s = 1;
    __syncthreads();
    __threadfence();
}

// Called by one thread of every workgroup of an item (nwg of them) when it is through with the item.
// An item on which any workgroup gave up waiting gets dist = NaN and status 5, whoever wrote dist
// before: the last workgroup through looks at the mark.  fin: [B][2] words, cleared to ~0 before the
// launch: [0] counts the workgroups that are through, [1] is written by a workgroup that timed out.
__device__ __forceinline__ void cluster_finish_item(const ClusterArgs& a, int b, bool timed_out, bool bad, int nwg)
{
    u64* fin = a.fin + (size_t)b * 2;
    if (timed_out) __hip_atomic_store(fin + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    const u64 old = __hip_atomic_fetch_add(fin, 1ull, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (u64)(nwg - 2)) {
        __threadfence();
        if (__hip_atomic_load(fin + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != ~0ull && !bad) {
            __hip_atomic_store(a.dist + b, __builtin_nanf(""), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.item_status)
                __hip_atomic_store(a.item_status + b, (int)kItemTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// D at the meeting frame: (Sa_mid + Sb_mid) + log2 sum_q ahat_mid[q] bhat_mid[q], in units of ln 2.
// Called by every thread of the workgroup (contains workgroup barriers).
__device__ __forceinline__ double meeting_value(const float* ah, const float* bh, const int* Sa,
                                                const int* Sb, int mid, int C, float* red)
{
    float part = 0.f;
    for (int q = threadIdx.x; q < C; q += blockDim.x)
        part += ah[(size_t)mid * C + q] * bh[(size_t)mid * C + q];
    const float tot = block_sum(part, red);
    return (double)(Sa[mid] + Sb[mid]) + (double)__log2f(tot);
}

// ------------------------------------------------------------------ alpha role
// LDS protocol (par = i & 1 is the parity of the state index i):
//   ap_s[par][r]   sum of the partial column sums for the workgroup's rows (part of a_i)
//   bl_s[par][r]   empty-label contribution a_i[r] E_i[r][0], written during step i (part of a_{i+1})
//   a_i[r] = ap_s[par][r] + bl_s[par^1][r]
//   ctl: [par] P_i (exponent step applied to the results of step i), [2 + par] exponent of a_i,
//        [40] timeout flag, [44..48] half-workgroup handshake flags
template <int D, bool GAMMA, bool ACC, int KT>
__device__ __forceinline__ void alpha_role(const ClusterArgs& a, const ClusterGeom& g, float* smem,
                                           unsigned& gstep, unsigned& ptag)
{
    float* ap_s = smem;
    float* bl_s = ap_s + 2 * kClMaxR;
    float* bv_s = bl_s + 2 * kClMaxR;         // [2][320] bhat_{i+1} staging (GAMMA)
    float* pacc_s = bv_s + 2 * 320;           // [320] scaled partial sums of the second half
    int* ctl_s = (int*)(pacc_s + 320);        // [64]
    float* red = (float*)(ctl_s + 64);        // [32]
    volatile int* flag_s = ctl_s + 44;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, keep it scalar
    const bool aux = wave == kClWaves;        // the eleventh wave streams nothing
    const int half = wave >= kClHW ? 1 : 0;   // which half of the workgroup's rows
    const int c = tid - half * kClHW * kWave; // column of a compute thread
    const int C = a.C, V1 = a.C;
    const bool colok = !aux && c < C;
    const int rb = half * kClRT;              // first row (inside the workgroup) of this thread
    // rows gathered by this wave: [3 wave, 3 wave + 3) within the workgroup's rows
    const int gr0 = 3 * wave;
    const int grn = max(0, min(3, g.nr - gr0));

    for (int b = g.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : mid;                        // steps of this role
        const int nex = GAMMA ? (L > 0 ? L - 1 : 0) : mid;    // steps that exchange
        const size_t fr = (size_t)C * V1;
        const unsigned frb = (unsigned)(fr * sizeof(float));  // bytes per frame
        float* ah = a.ahat + (size_t)b * (a.T + 1) * C;
        const float* bh = a.bhat + (size_t)b * (a.T + 1) * C;
        int* Sa = a.Sa + (size_t)b * (a.T + 1);
        const int* Sb = a.Sb + (size_t)b * (a.T + 1);
        u64* xbase = a.xa + (size_t)g.cg * 2 * a.XS * kClXK;

        if (tid < kClMaxR) {
            ap_s[tid] = (g.r0 == 0 && tid == 0) ? 1.f : 0.f;
            ap_s[kClMaxR + tid] = 0.f;
            bl_s[tid] = 0.f;
            bl_s[kClMaxR + tid] = 0.f;
        }
        if (tid == 0) { ctl_s[40] = 0; ctl_s[0] = 0; ctl_s[1] = 0; ctl_s[2] = 0; ctl_s[3] = 0; }
        if (tid < 8) ctl_s[44 + tid] = 0;
        __syncthreads();

        // ---- per-wave state ----
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        const unsigned coff = (unsigned)(min(c, C - 1) * (int)sizeof(float));     // per thread
        const unsigned pitch = (unsigned)(V1 * (int)sizeof(float));
        const unsigned rbase = (unsigned)(g.r0 + rb) * pitch;                    // scalar
        const int nrt = max(0, min(kClRT, g.nr - rb));      // real rows of this thread
        float E[D][kClRT];
        int sc[D];
        float bcol[2] = {0.f, 0.f};
        int sbn[2] = {0, 0};
        double D2 = 0.0;
        int dead = 0;
        // aux wave bookkeeping (identical in every alpha workgroup of the cluster)
        int sig = 0, P_cur = 0, P_prev = 0, mu_prev = 0;

        // Rows beyond the owned range are read anyway (in bounds of the item, or answered
        // with 0 by the buffer bounds check) and then forced to -inf, i.e. E = 0.
        auto issue = [&](int slot, int f) __attribute__((always_inline)) {
            const unsigned fo = (unsigned)f * frb + rbase;
#pragma unroll
            for (int r = 0; r < kClRT; ++r) E[slot][r] = buf_load_nt(wrs, coff, fo + (unsigned)r * pitch);
        };
        auto prep = [&](int slot) __attribute__((always_inline)) {
            float mx = LAST_NEG_INF;
#pragma unroll
            for (int r = 0; r < kClRT; ++r) {
                if (r >= nrt) E[slot][r] = LAST_NEG_INF;
                mx = fmaxf(mx, E[slot][r]);
            }
            const int s = shift_for(mx);
            sc[slot] = s;
            const float fs = (float)s;
#pragma unroll
            for (int r = 0; r < kClRT; ++r) E[slot][r] = fast_exp2(fmaf(E[slot][r], kLog2e, -fs));
        };
        // Loads and the exp pass are unconditional (the frame index is clamped to the last
        // frame of this role): conditional ones would leave registers "possibly pending" at
        // control-flow joins and force full memory waits on the serial path.
        const int nlast = max(n - 1, 0);
        if (!aux) {
#pragma unroll
            for (int f = 0; f < D - 1; ++f) issue(f, min(f, nlast));
            prep(0);
        }

        int i = 0;
        auto step = [&](auto SLOT) __attribute__((always_inline)) -> bool {
            constexpr int S = decltype(SLOT)::value;
            const int par = i & 1;
            // ---- top of state i: the aux wave completes a_i, stores it, publishes its magnitude
            const unsigned tag = gstep + 1;
            u64* xs = xbase + (size_t)(gstep & 1) * a.XS * kClXK;
            if (aux) {
                float av = 0.f;
                if (lane < g.nr) av = ap_s[par * kClMaxR + lds_row(lane)] + bl_s[(par ^ 1) * kClMaxR + lds_row(lane)];
                const int mu_own = wave_max_dpp((lane < g.nr) ? float_exponent(av) : -127);
                if (i <= mid) {
                    if (lane < g.nr) ah[(size_t)i * C + g.r0 + lane] = av;
                    if (lane == 0 && g.k == 0) Sa[i] = sig;
                }
                if (i < nex && lane == 0) xpublish(xs + (size_t)C * kClXK + g.k, pack_int(mu_own, tag));
            }
            if (i == mid) {
                if (aux && __builtin_amdgcn_ballot_w64(dead != 0) != 0 && lane == 0) ctl_s[40] = 1;
                cluster_sync(a, g, ptag, &ctl_s[40]);
                ptag += 1;
                D2 = meeting_value(ah, bh, Sa, Sb, mid, C, red);
                if (g.k == 0 && tid == 0) {
                    a.dist[b] = bad ? __builtin_nanf("") : (float)(D2 * 0.6931471805599453);
                    if (a.item_status)
                        a.item_status[b] = bad ? kItemBadLength : (ctl_s[40] ? kItemTimeout : kItemOk);
                }
                if (GAMMA && colok) {
                    // first two frames of the second half: fetch the other side's vectors now
                    if (mid < n) { bcol[mid & 1] = bh[(size_t)(mid + 1) * C + c]; sbn[mid & 1] = Sb[mid + 1]; }
                    if (mid + 1 < n) { bcol[(mid + 1) & 1] = bh[(size_t)(mid + 2) * C + c]; sbn[(mid + 1) & 1] = Sb[mid + 2]; }
                    if (mid < n) bv_s[(mid & 1) * 320 + c] = bcol[mid & 1];
                }
                __syncthreads();
            }
            if (i >= n) return false;
            const bool exch = i < nex;
            if (!aux) {
                // ---- FMA loop, hand-over between the two halves, publish
                const int P = ctl_s[par];
                // a_i for the 17 rows of this half: five 16-byte LDS reads per array, issued together
                float av[20];
                {
                    const float4* pa = (const float4*)(ap_s + par * kClMaxR + half * 20);
                    const float4* pb = (const float4*)(bl_s + (par ^ 1) * kClMaxR + half * 20);
#pragma unroll
                    for (int q4 = 0; q4 < 5; ++q4) {
                        const float4 x = pa[q4], y = pb[q4];
                        av[4 * q4] = x.x + y.x; av[4 * q4 + 1] = x.y + y.y;
                        av[4 * q4 + 2] = x.z + y.z; av[4 * q4 + 3] = x.w + y.w;
                    }
                }
                auto a_of = [&](int r) __attribute__((always_inline)) { return av[r]; };
                float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
                for (int r = 0; r < kClRT; ++r) {
                    if (r & 1) acc1 = fmaf(av[r], E[S][r], acc1); else acc0 = fmaf(av[r], E[S][r], acc0);
                }
                if (c == 0) {
#pragma unroll
                    for (int r = 0; r < kClRT; ++r)
                        bl_s[par * kClMaxR + half * 20 + r] = __builtin_ldexpf(av[r] * E[S][r], sc[S] - P);
                }
                float pub = __builtin_ldexpf(acc0 + acc1, sc[S] - P);
                if (half == 1) {
                    pacc_s[c] = pub;
                    if (lane == 0) flag_s[wave - kClHW] = i + 1;
                } else {
                    int spins = 0;
                    while (flag_s[wave] != i + 1 && ++spins < (1 << 22)) { }
                    pub += ((volatile float*)pacc_s)[c];
                    if (exch && colok && c >= 1) xpublish(xs + (size_t)c * kClXK + g.k, pack_word(pub, tag));
                }
                if (GAMMA && i >= mid && colok) {
                    const float kx = (float)((double)(ctl_s[2 + par] + sbn[par]) - D2);
                    const float fac = a.scale * fast_exp2(kx + (float)sc[S]) * (c == 0 ? 1.f : bcol[par]);
                    const unsigned gso = (unsigned)i * frb + rbase;
#pragma unroll
                    for (int r = 0; r < kClRT; ++r)
                        if (r < nrt) {
                            // the empty label (column 0) returns to the row's own state
                            const float f2 = (c == 0) ? fac * bv_s[par * 320 + g.r0 + rb + r] : fac;
                            const float gv = a_of(r) * E[S][r] * f2;
                            if (ACC) buf_store(buf_load(grs, coff, gso + (unsigned)r * pitch) + gv, grs, coff, gso + (unsigned)r * pitch);
                            else buf_store_nt(gv, grs, coff, gso + (unsigned)r * pitch);
                        }
                }
                // state vectors of the other side for the marginals two frames ahead
                if (GAMMA && i >= mid && i + 2 < n && colok) {
                    bcol[par] = bh[(size_t)(i + 3) * C + c];
                    sbn[par] = Sb[i + 3];
                }
                issue((S + D - 1) % D, min(i + D - 1, nlast));
                prep((S + 1) % D);
                if (GAMMA && i + 1 < n && i + 1 >= mid && colok) bv_s[(par ^ 1) * 320 + c] = bcol[par ^ 1];
            }
            if (exch) {
                // ---- gather: every wave sums the partial columns of three of the own rows
                float s0 = 0.f, s1 = 0.f, s2 = 0.f;
                int mu = 0;
                if ((grn > 0 || aux) && !dead) {
                    v16u v0, v1, v2, vh;
                    // the aux wave has nothing else to do: do not poll before the producers can
                    // have published (a poll served too early costs a whole extra round trip)
                    if (aux)
                        for (int dly = 0; dly < kClAuxDelay; ++dly) __builtin_amdgcn_s_sleep(4);
                    // rows beyond the owned range are still loaded (inside the buffer) and ignored
                    const void* rowp = xs + (size_t)(g.r0 + min(gr0, g.nr - 1)) * kClXK;
                    // the start state (q = 0) receives no label arcs: its row is never written
                    const bool skip0 = g.r0 + gr0 == 0;
                    int np = 0;
                    for (;;) {
                        if (aux) sgather4(rowp, xs + (size_t)C * kClXK, v0, v1, v2, vh);
                        else sgather3(rowp, v0, v1, v2);
                        bool ok = (grn < 1 || skip0 || block_ready(v0, KT, tag))
                                  && (grn < 2 || block_ready(v1, KT, tag))
                                  && (grn < 3 || block_ready(v2, KT, tag));
                        if (aux) ok = ok && block_ready(vh, KT, tag);
                        if (ok) break;
                        if (++np > a.spin_limit) { dead = 1; break; }
                    }
                    s0 = skip0 ? 0.f : block_sum8(v0, KT);
                    s1 = block_sum8(v1, KT);
                    s2 = block_sum8(v2, KT);
                    if (aux) {
                        mu = -127;
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            if (j < KT) mu = max(mu, (int)vh[2 * j]);
                    }
                }
                if (lane == 0) {
                    if (grn > 0) ap_s[(par ^ 1) * kClMaxR + lds_row(gr0)] = s0;
                    if (grn > 1) ap_s[(par ^ 1) * kClMaxR + lds_row(gr0 + 1)] = s1;
                    if (grn > 2) ap_s[(par ^ 1) * kClMaxR + lds_row(gr0 + 2)] = s2;
                }
                if (aux) {
                    // exponent step for the next publish, from magnitudes every workgroup has seen
                    const int G = mu - mu_prev + P_prev;          // growth observed in step i - 1
                    const int P_next = mu + 2 * G - P_cur;
                    sig += P_cur;
                    if (lane == 0) { ctl_s[par ^ 1] = P_next; ctl_s[2 + (par ^ 1)] = sig; }
                    mu_prev = mu; P_prev = P_cur; P_cur = P_next;
                    if (dead && lane == 0) ctl_s[40] = 1;
                } else if (dead && lane == 0) {
                    ctl_s[40] = 1;
                }
                gstep += 1;
            }
            __syncthreads();
            ++i;
            return true;
        };
        for (;;) {
            if (!step(std::integral_constant<int, 0>())) break;
            if (!step(std::integral_constant<int, 1>())) break;
            if (!step(std::integral_constant<int, 2>())) break;
            if constexpr (D > 3) { if (!step(std::integral_constant<int, 3>())) break; }
        }
        __syncthreads();
        if (tid == 0) cluster_finish_item(a, b, ctl_s[40] != 0, bad, 2 * a.K);
        __syncthreads();
    }
}

// ------------------------------------------------------------------- beta role
// LDS: b_s[par][q] = b_{t+1} for all states (par = step parity); mu_s[par][wave] = largest
// binary exponent among the words gathered by each wave; every wave keeps (mu, P, exponent)
// of the current vector in registers, identically.
template <int D, bool GAMMA, bool ACC, int KT>
__device__ __forceinline__ void beta_role(const ClusterArgs& a, const ClusterGeom& g, float* smem,
                                          unsigned& gstep, unsigned& ptag)
{
    float* b_s = smem;                        // [2][320]
    int* ctl_s = (int*)(b_s + 2 * 320);       // [0..31] mu_s[2][16], [40] timeout flag
    float* red = (float*)(ctl_s + 64);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool aux = wave == kClWaves;
    const int C = a.C, V1 = a.C;
    // rows of this wave: wave, wave + 10, ... (index inside the workgroup's rows)
    int nrw = 0;
    if (!aux) nrw = (g.nr - wave + kClWaves - 1) / kClWaves;
    if (nrw < 0) nrw = 0;
    const int ncol = (C + 63) / 64;
    // exchange words gathered by this wave: [24 wave, 24 wave + 24) of the C state values
    const int gq0 = kClCH * wave;
    const int gqn = max(0, min(kClCH, C - gq0));

    for (int b = g.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : L - mid;
        // the last frame's result is not needed, except that b_mid must exist (L = 1: mid = 0)
        const int nex = GAMMA ? max(L - 1, L - mid) : L - mid;
        const int ph1 = L - mid;                     // step at which the state index reaches mid
        const size_t fr = (size_t)C * V1;
        const unsigned frb = (unsigned)(fr * sizeof(float));
        const float* ah = a.ahat + (size_t)b * (a.T + 1) * C;
        float* bh = a.bhat + (size_t)b * (a.T + 1) * C;
        const int* Sa = a.Sa + (size_t)b * (a.T + 1);
        int* Sb = a.Sb + (size_t)b * (a.T + 1);
        u64* xbase = a.xb + (size_t)g.cg * 2 * a.XSB;

        if (tid == 0) ctl_s[40] = 0;
        if (tid < 32) ctl_s[tid] = -127;                     // no words gathered yet
        // both slots: entries for columns >= C stay 0 for the whole item (clamped loads meet them)
        for (int q = tid; q < 2 * 320; q += blockDim.x) b_s[q] = q < C ? 1.f : 0.f;
        // b_L = 1 with exponent 0
        if (g.k == 0) {
            for (int q = tid; q < C; q += blockDim.x) bh[(size_t)L * C + q] = 1.f;
            if (tid == 0) Sb[L] = 0;
        }
        __syncthreads();

        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        // Byte offsets of this lane's elements inside a frame (shared by w and the marginals).
        // Rows / columns beyond the valid range are clamped: such rows are never published or
        // stored, such columns meet a zero in the b vector.
        unsigned coff[kClNC];                                                    // per lane
#pragma unroll
        for (int j = 0; j < kClNC; ++j) coff[j] = (unsigned)(min(lane + 64 * j, C - 1) * (int)sizeof(float));
        const unsigned pitch = (unsigned)(V1 * (int)sizeof(float));
        auto roff = [&](int ri) __attribute__((always_inline)) {              // scalar
            return (unsigned)(g.r0 + min(wave + ri * kClWaves, g.nr - 1)) * pitch;
        };
        float E[D][kClRW][kClNC];
        int sr[D][kClRW];
        float apre[2] = {0.f, 0.f};   // lane ri < nrw holds ahat_t[row ri] two frames ahead
        int san[2] = {0, 0};
        double D2 = 0.0;
        int dead = 0;
        int sig = 0, P_cur = 0, mu_cur = 0;     // exponent bookkeeping, identical in every wave

        auto issue = [&](int slot, int f) __attribute__((always_inline)) {       // frame t = L-1-f
            const unsigned so = (unsigned)max(L - 1 - f, 0) * frb;
#pragma unroll
            for (int ri = 0; ri < kClRW; ++ri)
#pragma unroll
                for (int j = 0; j < kClNC; ++j) E[slot][ri][j] = buf_load_nt(wrs, coff[j], so + roff(ri));
        };
        auto prep = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
            for (int ri = 0; ri < kClRW; ++ri) {
                float mx = E[slot][ri][0];
#pragma unroll
                for (int j = 1; j < kClNC; ++j) mx = fmaxf(mx, E[slot][ri][j]);
                mx = wave_max_dpp(mx);
                const int s = shift_for(mx);
                sr[slot][ri] = s;
                const float fs = (float)s;
#pragma unroll
                for (int j = 0; j < kClNC; ++j)
                    E[slot][ri][j] = fast_exp2(fmaf(E[slot][ri][j], kLog2e, -fs));
            }
        };
        const int nlast = max(n - 1, 0);     // see the alpha role: unconditional, clamped
        if (!aux) {
#pragma unroll
            for (int f = 0; f < D - 1; ++f) issue(f, min(f, nlast));
            prep(0);
        }

        int i = 0;
        auto step = [&](auto SLOT) __attribute__((always_inline)) -> bool {
            constexpr int S = decltype(SLOT)::value;
            const int par = i & 1;
            const int t = L - 1 - i;
            if (i == ph1) {
                if (dead && lane == 0) ctl_s[40] = 1;
                cluster_sync(a, g, ptag, &ctl_s[40]);
                ptag += 1;
                D2 = meeting_value(ah, bh, Sa, Sb, mid, C, red);
                if (GAMMA && !aux) {
                    // forward vectors for the first two frames of the second half
                    if (ph1 < n) {
                        const int t0 = L - 1 - ph1;
                        apre[ph1 & 1] = (lane < nrw) ? ah[(size_t)t0 * C + g.r0 + wave + lane * kClWaves] : 0.f;
                        san[ph1 & 1] = Sa[t0];
                    }
                    if (ph1 + 1 < n) {
                        const int t1 = L - 2 - ph1;
                        apre[(ph1 + 1) & 1] = (lane < nrw) ? ah[(size_t)t1 * C + g.r0 + wave + lane * kClWaves] : 0.f;
                        san[(ph1 + 1) & 1] = Sa[t1];
                    }
                }
                __syncthreads();
            }
            if (i >= n) return false;
            const bool exch = i < nex;
            const unsigned tag = gstep + 1;
            u64* xs = xbase + (size_t)(gstep & 1) * a.XSB;
            if (!aux) {
                float bv[kClNC];
#pragma unroll
                for (int j = 0; j < kClNC; ++j) bv[j] = b_s[par * 320 + lane + 64 * j];
                float brow[kClRW];
#pragma unroll
                for (int ri = 0; ri < kClRW; ++ri) {
                    const int row = g.r0 + min(wave + ri * kClWaves, g.nr - 1);
                    brow[ri] = b_s[par * 320 + row];
                    // the empty label (column 0) returns to the row's own state
                    float acc = E[S][ri][0] * (lane == 0 ? brow[ri] : bv[0]);
#pragma unroll
                    for (int j = 1; j < kClNC; ++j) acc = fmaf(E[S][ri][j], bv[j], acc);
                    const float tot = wave_sum_dpp(acc);
                    if (exch && lane == 0 && ri < nrw)
                        xpublish(xs + row, pack_word(__builtin_ldexpf(tot, sr[S][ri] - P_cur), tag));
                }
                if (GAMMA && i >= ph1) {
                    const float kx = (float)((double)(san[par] + sig) - D2);
                    const unsigned gso = (unsigned)t * frb;
#pragma unroll
                    for (int ri = 0; ri < kClRW; ++ri)
                        if (ri < nrw) {
                            const float arow = __shfl(apre[par], ri, 64);
                            const float fac = a.scale * arow * fast_exp2(kx + (float)sr[S][ri]);
#pragma unroll
                            for (int j = 0; j < kClNC; ++j)
                                if (j < ncol && lane + 64 * j < C) {
                                    const float bb = (j == 0 && lane == 0) ? brow[ri] : bv[j];
                                    const float gv = E[S][ri][j] * bb * fac;
                                    if (ACC) buf_store(buf_load(grs, coff[j], gso + roff(ri)) + gv, grs, coff[j], gso + roff(ri));
                                    else buf_store_nt(gv, grs, coff[j], gso + roff(ri));
                                }
                        }
                }
                // forward vector of the frame two steps ahead (second half only)
                if (GAMMA && i >= ph1 && i + 2 < n) {
                    const int t2 = t - 2;
                    apre[par] = (lane < nrw) ? ah[(size_t)t2 * C + g.r0 + wave + lane * kClWaves] : 0.f;
                    san[par] = Sa[t2];
                }
                issue((S + D - 1) % D, min(i + D - 1, nlast));
                prep((S + 1) % D);
            }
            if (exch) {
                // ---- gather: every wave fetches 24 of the C state values through the scalar path
                if (gqn > 0) {
                    v16u v0, v1, v2;
                    const void* rowp = xs + gq0;
                    int np = 0;
                    if (!dead)
                        for (;;) {
                            sgather3(rowp, v0, v1, v2);
                            const bool ok = block_ready(v0, gqn, tag) && block_ready(v1, gqn - 8, tag)
                                            && block_ready(v2, gqn - 16, tag);
                            if (ok) break;
                            if (++np > a.spin_limit) { dead = 1; break; }
                        }
                    else
                        sgather3(rowp, v0, v1, v2);
                    // scatter the 24 scalar values over the first 24 lanes of one register
                    float val = 0.f;
                    int mu = -127;
                    auto put = [&](unsigned bits, int l) __attribute__((always_inline)) {
                        if (l < gqn) {
                            val = (lane == l) ? __uint_as_float(bits) : val;
                            mu = max(mu, (int)((bits >> 23) & 0xFFu) - 127);
                        }
                    };
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        put(v0[2 * j], j);
                        put(v1[2 * j], 8 + j);
                        put(v2[2 * j], 16 + j);
                    }
                    if (lane < gqn) {
                        b_s[(par ^ 1) * 320 + gq0 + lane] = val;
                        if (t >= mid && g.k == 0) bh[(size_t)t * C + gq0 + lane] = val;
                    }
                    if (lane == 0) ctl_s[(par ^ 1) * 16 + wave] = mu;
                    if (dead && lane == 0) ctl_s[40] = 1;
                }
                gstep += 1;
            }
            __syncthreads();
            if (exch) {
                // exponent bookkeeping for b_t (now in b_s[par ^ 1]): every wave, identically
                int mu = -127;
#pragma unroll
                for (int j = 0; j < kClWaves + 1; ++j) mu = max(mu, ctl_s[(par ^ 1) * 16 + j]);
                const int G = mu - mu_cur + P_cur;        // growth observed in this step
                sig += P_cur;
                if (t >= mid && g.k == 0 && tid == 0) Sb[t] = sig;
                P_cur = mu + G;
                mu_cur = mu;
            }
            ++i;
            return true;
        };
        for (;;) {
            if (!step(std::integral_constant<int, 0>())) break;
            if (!step(std::integral_constant<int, 1>())) break;
            if (!step(std::integral_constant<int, 2>())) break;
            if constexpr (D > 3) { if (!step(std::integral_constant<int, 3>())) break; }
        }
        __syncthreads();
        if (tid == 0) cluster_finish_item(a, b, ctl_s[40] != 0, bad, 2 * a.K);
        __syncthreads();
    }
}

// Zero the marginals of frames t >= len (they do not exist) and of items with
// an invalid length; the 2K workgroups of a cluster share the work.
__device__ __forceinline__ void cluster_zero_padding(const ClusterArgs& a, const ClusterGeom& g)
{
    const int nwg = 2 * a.K, me = g.role * a.K + g.k;
    const size_t fr = (size_t)a.C * a.C;
    for (int b = g.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        if (L < 0 || L > a.T) L = 0;
        float* p = a.dw + ((size_t)b * a.T + L) * fr;
        const size_t cnt = (size_t)(a.T - L) * fr;
        for (size_t i = (size_t)me * blockDim.x + threadIdx.x; i < cnt; i += (size_t)nwg * blockDim.x)
            __builtin_nontemporal_store(0.f, p + i);
    }
}

template <int D, bool GAMMA, bool ACC, int KT>
__global__ __launch_bounds__(kClThreads) void cluster_fb_kernel(ClusterArgs a)
{
    __shared__ float smem[kClLds];
    ClusterGeom g;
    const int id = blockIdx.x;
    const int x = id & 7, slot = id >> 3;
    const int cl = slot / (2 * a.K), member = slot - cl * 2 * a.K;
    g.cg = x + 8 * cl;
    g.role = member / a.K;
    g.k = member - g.role * a.K;
    g.r0 = g.k * a.RPW;
    g.nr = min(a.RPW, a.C - g.r0);
    if (g.nr < 0) g.nr = 0;
    if (g.r0 > a.C) g.r0 = a.C;
    unsigned gstep = 0, ptag = 0;
    if (GAMMA && !ACC) cluster_zero_padding(a, g);
    if (g.role == 0) alpha_role<D, GAMMA, ACC, KT>(a, g, smem, gstep, ptag);
    else beta_role<D, GAMMA, ACC, KT>(a, g, smem, gstep, ptag);
}

// set every exchange word to "invalid tag"
__global__ void cluster_clear_kernel(u64* p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = ~0ull;
}

}  // namespace last
