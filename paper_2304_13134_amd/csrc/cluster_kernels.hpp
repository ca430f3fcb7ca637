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
//   alpha: thread <-> destination column; partial column sums over the own
//          rows are exchanged (reduce-scatter: workgroup k only needs the
//          sums for its own states);
//   beta : wavefront <-> row, lanes <-> columns; complete row sums are
//          exchanged (all-gather).
// Arithmetic is in the scaled linear domain: E = 2^(w*log2(e) - s) with an
// integer shift s per column (alpha) or per row (beta) chosen from the data so
// that E <= 1, state vectors carry a common integer exponent (Sa, Sb), and
// partial results travel as (float value, int16 shift).  exp(w) does not depend
// on the recursion, so it is evaluated while the previous step's exchange is in
// flight; the serial chain per frame is: FMA loop, publish, poll, rescale.
//
// Exchange: 64-bit words [value:32 | shift:16 | tag:16] written and polled with
// relaxed agent-scope atomics; the tag (a running step counter) makes each word
// self-validating, so no fences are needed on the per-frame path.  Two slots
// (step parity) suffice: nobody can publish step s+2 before everybody has
// consumed step s.  One wavefront per workgroup (the "comm" wave) does all
// polling so that the streaming loads of the compute waves never sit in front
// of a poll in the in-order load return queue.  Every poll loop is bounded.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace last {

typedef unsigned long long u64;

constexpr int kClMaxR = 34;      // max rows owned by one workgroup (two halves of kClRT rows)
constexpr int kClRT = 17;        // rows per alpha thread: each workgroup splits its rows in two halves
constexpr int kClHW = 5;         // compute waves per half (alpha): 5 * 64 >= kClMaxC columns
constexpr int kClWaves = 10;     // compute waves per workgroup
constexpr int kClRW = 4;         // max rows per compute wave (beta): ceil(34 / 10)
constexpr int kClNC = 5;         // max columns per lane (beta): ceil(320 / 64)
constexpr int kClMaxC = 320;     // max number of states / labels on this path
constexpr int kClThreads = (kClWaves + 1) * kWave;
constexpr int kClMaxK = 8;       // max workgroups per role
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kShiftNone = -30000;
constexpr unsigned kTagInvalid = 0xFFFFu;

// Optional cycle-counter marks for tuning (compiled out unless LAST_TRACE is defined):
// trace[((workgroup * 2 + is_comm) * 64 + step) * 4 + k] = clock of mark k
#ifdef LAST_TRACE
#define LAST_MARK(a, iscomm, step, k)                                                          \
    do {                                                                                       \
        if ((a).trace && (step) < 64 && (threadIdx.x & 63) == 0 &&                             \
            ((iscomm) || threadIdx.x == 0))                                                    \
            (a).trace[(((size_t)blockIdx.x * 2 + (iscomm)) * 64 + (step)) * 4 + (k)] = clock64(); \
    } while (0)
#else
#define LAST_MARK(a, iscomm, step, k) do { } while (0)
#endif

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
    int B, T, C;
    int K, RPW, ncl;   // workgroups per role, rows per workgroup, clusters per XCD
    int XS, XSB;
    float scale;
    int accumulate;
    int spin_limit;
#ifdef LAST_TRACE
    unsigned long long* trace;
#endif
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
__device__ __forceinline__ u64 pack_word(float v, int shift, unsigned tag)
{
    return (u64)__float_as_uint(v) | ((u64)(unsigned)(shift & 0xFFFF) << 32) | ((u64)(tag & 0xFFFFu) << 48);
}
__device__ __forceinline__ float word_value(u64 x) { return __uint_as_float((unsigned)x); }
__device__ __forceinline__ int word_shift(u64 x) { return (int)(short)(unsigned short)(x >> 32); }
__device__ __forceinline__ unsigned word_tag(u64 x) { return (unsigned)(x >> 48); }
__device__ __forceinline__ u64 pack_header(int h, int m, unsigned tag)
{
    return (u64)(unsigned)(h & 0xFFFF) | ((u64)(unsigned)(m & 0xFFFF) << 16) | ((u64)(tag & 0xFFFFu) << 48);
}
__device__ __forceinline__ int header_h(u64 x) { return (int)(short)(unsigned short)x; }
__device__ __forceinline__ int header_m(u64 x) { return (int)(short)(unsigned short)(x >> 16); }

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
typedef __amdgpu_buffer_rsrc_t buf_t;
__device__ __forceinline__ buf_t make_buf(const void* p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load_nt(buf_t r, unsigned voff, unsigned soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 2));
}
__device__ __forceinline__ void buf_store_nt(float v, buf_t r, unsigned voff, unsigned soff)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, 2);
}
__device__ __forceinline__ float buf_load(buf_t r, unsigned voff, unsigned soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}
__device__ __forceinline__ void buf_store(float v, buf_t r, unsigned voff, unsigned soff)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, 0);
}

// poll one word until its tag matches; gives up after `limit` polls (dead = 1)
__device__ __forceinline__ u64 poll_word(const u64* p, unsigned tag, int limit, int& dead)
{
    u64 x = xload(p);
    if (dead) return x;
    int n = 0;
    while (word_tag(x) != tag) {
        if (++n > limit) { dead = 1; break; }
        __builtin_amdgcn_s_sleep(1);
        x = xload(p);
    }
    return x;
}

// Poll N words (those with want[j] set) until every tag matches.  All outstanding words are
// re-read together in each round, so the wait costs one round trip after the last word lands
// rather than one round trip per word.
template <int N>
__device__ __forceinline__ void poll_words(const u64* base, size_t stride, int count, u64 (&x)[N],
                                           unsigned tag, int limit, int& dead)
{
#pragma unroll
    for (int j = 0; j < N; ++j)
        if (j < count) x[j] = xload(base + j * stride);
    if (dead) return;
    int n = 0;
    for (;;) {
        bool ok = true;
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < count && word_tag(x[j]) != tag) ok = false;
        if (ok) break;
        if (++n > limit) { dead = 1; break; }
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < count && word_tag(x[j]) != tag) x[j] = xload(base + j * stride);
    }
}

// Poll one row of 2*K consecutive words (16-byte aligned) with 16-byte loads: a destination's
// partial sums from all producers sit in one cache line.  Volatile vector loads bypass the
// vector L1; every 8-byte word was written by a single store, so it is read whole.
typedef unsigned v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bool pair_ready(v4u v, unsigned tag)
{
    return (v.y >> 16) == tag && (v.w >> 16) == tag;
}
// sum of the 2*K partial values of a row, each scaled by 2^(shift - dl)
template <int K>
__device__ __forceinline__ float poll_row_sum(const u64* row, unsigned tag, int dl, int limit, int& dead)
{
    const volatile v4u* p = (const volatile v4u*)row;
    v4u v[K];
#pragma unroll
    for (int j = 0; j < K; ++j)
        v[j] = p[j];
    if (!dead) {
        int n = 0;
        for (;;) {
            bool ok = true;
#pragma unroll
            for (int j = 0; j < K; ++j)
                if (!pair_ready(v[j], tag)) ok = false;
            if (ok) break;
            if (++n > limit) { dead = 1; break; }
#pragma unroll
            for (int j = 0; j < K; ++j)
                if (!pair_ready(v[j], tag)) v[j] = p[j];
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < K; ++j)
        {
            s += __builtin_ldexpf(__uint_as_float(v[j].x), (int)(short)(v[j].y & 0xFFFFu) - dl);
            s += __builtin_ldexpf(__uint_as_float(v[j].z), (int)(short)(v[j].w & 0xFFFFu) - dl);
        }
    return s;
}

struct ClusterGeom {
    int role;     // 0 alpha, 1 beta
    int k;        // workgroup index inside the role
    int cg;       // global cluster index
    int r0, nr;   // owned rows
};

// barrier among the 2K workgroups of a cluster with release/acquire semantics
// for plain global stores (used once per item, at the meeting frame)
__device__ __forceinline__ void cluster_sync(const ClusterArgs& a, const ClusterGeom& g, unsigned tag,
                                             int& dead, int* dead_s)
{
    __threadfence();
    __syncthreads();
    u64* flags = a.ph + (size_t)g.cg * 32;
    const int me = g.role * a.K + g.k;
    const u64 target = (u64)tag + 1;          // flags count items; ~0 = never written
    if (threadIdx.x == 0) xstore(flags + me, target);
    if (threadIdx.x < 2 * a.K && !dead) {
        int n = 0;
        for (;;) {
            const u64 x = xload(flags + threadIdx.x);
            if (x != ~0ull && x >= target) break;
            if (++n > a.spin_limit) { *dead_s = 1; break; }
            __builtin_amdgcn_s_sleep(2);
        }
    }
    __syncthreads();
    dead = *dead_s;
    __threadfence();
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
//   ap_s[par][r]   partial-sum part of a_i for the workgroup's rows, already scaled by 2^-dl
//   bl_s[par][r]   empty-label products a_i[r] * E_i[r][0] written during step i (for a_{i+1})
//   ctl: [par] dl_{i-1}, [2 + 2 par + half] column-0 shift of step i, [6 + par] exponent of a_i,
//        [8 + 16 par + wave] per-wave max column shift of frame i, [40] timeout flag
//   a_i[r] = ap_s[par][r] + ldexp(bl_s[par^1][r], s0_{i-1} - dl_{i-1})
template <int D, bool GAMMA, bool ACC, int KT>
__device__ __forceinline__ void alpha_role(const ClusterArgs& a, const ClusterGeom& g, float* smem,
                                           unsigned& gstep, unsigned& ptag)
{
    float* ap_s = smem;
    float* bl_s = ap_s + 2 * kClMaxR;
    float* bv_s = bl_s + 2 * kClMaxR;         // [2][kClMaxC] bhat_{i+1} staging (GAMMA)
    int* ctl_s = (int*)(bv_s + 2 * kClMaxC);
    float* red = (float*)(ctl_s + 48);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, keep it scalar
    const bool comm = wave == kClWaves;
    const int half = wave >= kClHW ? 1 : 0;   // which half of the workgroup's rows
    const int c = tid - half * kClHW * kWave; // column of a compute thread
    const int C = a.C, V1 = a.C;
    const bool colok = !comm && c < C;
    const int rb = half * kClRT;              // first row (inside the workgroup) of this thread

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
        constexpr int XK = 2 * KT;                                // words per row
        u64* xbase = a.xa + (size_t)g.cg * 2 * a.XS * XK;

        if (tid < kClMaxR) {
            ap_s[tid] = (g.r0 + tid == 0 && tid < g.nr) ? 1.f : 0.f;
            ap_s[kClMaxR + tid] = 0.f;
            bl_s[tid] = 0.f;
            bl_s[kClMaxR + tid] = 0.f;
        }
        if (tid == 0) {
            ctl_s[40] = 0; ctl_s[0] = 0; ctl_s[4] = kShiftNone; ctl_s[5] = kShiftNone; ctl_s[6] = 0;
        }
        __syncthreads();

        if (comm) {
            // ================= comm wave: exchange only =================
            int dead = 0, sig = 0;
            int m_own = (g.r0 == 0) ? 0 : -127;
            __syncthreads();       // the compute waves have published the column shifts of frame 0
            for (int i = 0;; ++i) {
                const int par = i & 1;
                // complete a_i, store it for the other side, take its magnitude
                if (i == 0) {
                    if (lane < g.nr) ah[g.r0 + lane] = (g.r0 + lane == 0) ? 1.f : 0.f;
                    if (lane == 0 && g.k == 0) Sa[0] = 0;
                } else if (i <= nex) {
                    float av = 0.f;
                    if (lane < g.nr)
                        av = ap_s[par * kClMaxR + lane]
                             + __builtin_ldexpf(bl_s[(par ^ 1) * kClMaxR + lane],
                                                ctl_s[2 + (par ^ 1) * 2 + (lane >= kClRT ? 1 : 0)] - ctl_s[par]);
                    m_own = wave_max_dpp((lane < g.nr) ? float_exponent(av) : -127);
                    if (i <= mid) {
                        if (lane < g.nr) ah[(size_t)i * C + g.r0 + lane] = av;
                        if (lane == 0 && g.k == 0) Sa[i] = sig;
                    }
                }
                if (i == mid) {
                    if (__builtin_amdgcn_ballot_w64(dead != 0) != 0 && lane == 0) ctl_s[40] = 1;
                    cluster_sync(a, g, ptag, dead, &ctl_s[40]);
                    ptag += 1;
                    const double D2 = meeting_value(ah, bh, Sa, Sb, mid, C, red);
                    if (g.k == 0 && lane == 0) {
                        a.dist[b] = bad ? __builtin_nanf("") : (float)(D2 * 0.6931471805599453);
                        if (a.item_status)
                            a.item_status[b] = bad ? kItemBadLength : (dead ? kItemTimeout : kItemOk);
                    }
                    __syncthreads();
                }
                if (i >= n) break;
                if (i < nex) {
                    const unsigned tag = gstep % 65535u;
                    u64* xs = xbase + (size_t)(gstep & 1) * a.XS * XK;
                    LAST_MARK(a, 1, i, 0);
                    int h = kShiftNone;
                    if (lane < kClWaves) h = ctl_s[8 + par * 16 + lane];
                    h = wave_max_dpp(h);
                    if (lane == 0) xstore(xs + (size_t)C * XK + 2 * g.k, pack_header(h, m_own, tag));
                    // one batch: this lane's row of partial sums (16-byte loads) and, on the first
                    // KT lanes, one header word each; poll until every tag matches
                    const bool wantrow = lane < g.nr && g.r0 + lane != 0;   // q = 0 has no partials
                    const volatile v4u* rowp = (const volatile v4u*)(xs + (size_t)(g.r0 + (wantrow ? lane : 0)) * XK);
                    const u64* hp = xs + (size_t)C * XK + 2 * (lane < KT ? lane : 0);
                    v4u v[KT];
                    u64 hx = 0;
#pragma unroll
                    for (int j = 0; j < KT; ++j) v[j] = rowp[j];
                    hx = xload(hp);
                    if (!dead) {
                        int np = 0;
                        for (;;) {
                            bool ok = !(lane < KT) || word_tag(hx) == tag;
                            if (wantrow) {
#pragma unroll
                                for (int j = 0; j < KT; ++j)
                                    if (!pair_ready(v[j], tag)) ok = false;
                            }
                            if (ok) break;
                            if (++np > a.spin_limit) { dead = 1; break; }
                            if (lane < KT && word_tag(hx) != tag) hx = xload(hp);
                            if (wantrow) {
#pragma unroll
                                for (int j = 0; j < KT; ++j)
                                    if (!pair_ready(v[j], tag)) v[j] = rowp[j];
                            }
                        }
                    }
                    // every lane must know all headers: wait for the slowest lane of the wave
                    const int hh = lane < KT ? header_h(hx) : kShiftNone;
                    const int mm = lane < KT ? header_m(hx) : -127;
                    const int dl = wave_max_dpp(hh) + wave_max_dpp(mm);
                    LAST_MARK(a, 1, i, 1);
                    float v_sum = 0.f;
                    if (wantrow) {
#pragma unroll
                        for (int j = 0; j < KT; ++j) {
                            v_sum += __builtin_ldexpf(__uint_as_float(v[j].x), (int)(short)(v[j].y & 0xFFFFu) - dl);
                            v_sum += __builtin_ldexpf(__uint_as_float(v[j].z), (int)(short)(v[j].w & 0xFFFFu) - dl);
                        }
                    }
                    LAST_MARK(a, 1, i, 2);
                    if (lane < kClMaxR) ap_s[(par ^ 1) * kClMaxR + lane] = v_sum;
                    sig += dl;
                    if (lane == 0) { ctl_s[par ^ 1] = dl; ctl_s[6 + (par ^ 1)] = sig; }
                    gstep += 1;
                }
                __syncthreads();
            }
            if (__builtin_amdgcn_ballot_w64(dead != 0) != 0 && lane == 0 && g.k == 0 && a.item_status && !bad)
                a.item_status[b] = kItemTimeout;
        } else {
            // ================= compute waves =================
            const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
            const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
            // Byte offsets of this thread's elements inside a frame (the same for every frame and
            // for the marginals, which share the layout of w).  Rows beyond the owned range are
            // clamped to the last owned row: their a-values are 0.
            const unsigned coff = (unsigned)(min(c, C - 1) * (int)sizeof(float));     // per thread
            const unsigned pitch = (unsigned)(V1 * (int)sizeof(float));
            const unsigned rbase = (unsigned)(g.r0 + rb) * pitch;                    // scalar
            const int nrt = max(0, min(kClRT, g.nr - rb));      // real rows of this thread
            float E[D][kClRT];
            int sc[D];
            float bcol[2] = {0.f, 0.f};
            int sbn[2] = {0, 0};
            double D2 = 0.0;
            int hcur = kShiftNone;

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
                return s;
            };
            // Loads and the exp pass are unconditional (the frame index is clamped to the last
            // frame of this role): conditional ones would leave registers "possibly pending" at
            // control-flow joins and force full memory waits on the serial path.
            const int nlast = max(n - 1, 0);
#pragma unroll
            for (int f = 0; f < D - 1; ++f) issue(f, min(f, nlast));
            hcur = prep(0);
            {
                const int hw = wave_max_dpp(colok ? hcur : kShiftNone);
                if (lane == 0) ctl_s[8 + wave] = hw;
            }
            __syncthreads();       // frame 0 is prepared: its column shifts are visible to the comm wave

            int i = 0;
            auto step = [&](auto SLOT) __attribute__((always_inline)) -> bool {
                constexpr int S = decltype(SLOT)::value;
                const int par = i & 1;
                if (i == mid) {
                    int dead = 0;
                    cluster_sync(a, g, ptag, dead, &ctl_s[40]);
                    ptag += 1;
                    D2 = meeting_value(ah, bh, Sa, Sb, mid, C, red);
                    if (GAMMA && colok) {
                        // first two frames of the second half: fetch the other side's vectors now
                        if (mid < n) { bcol[mid & 1] = bh[(size_t)(mid + 1) * C + c]; sbn[mid & 1] = Sb[mid + 1]; }
                        if (mid + 1 < n) { bcol[(mid + 1) & 1] = bh[(size_t)(mid + 2) * C + c]; sbn[(mid + 1) & 1] = Sb[mid + 2]; }
                        if (mid < n) bv_s[(mid & 1) * kClMaxC + c] = bcol[mid & 1];
                    }
                    __syncthreads();
                }
                if (i >= n) return false;
                const bool exch = i < nex;
                const unsigned tag = gstep % 65535u;
                u64* xs = xbase + (size_t)(gstep & 1) * a.XS * XK;
                LAST_MARK(a, 0, i, 0);
                // Stream first: the vector memory pipeline returns in order, so loads issued later
                // in the step would sit in front of the comm wave's next polls for longer.
                issue((S + D - 1) % D, min(i + D - 1, nlast));
                const int dl = ctl_s[par];
                const int blsh = ctl_s[2 + (par ^ 1) * 2 + half] - dl;
                float acc0 = 0.f, acc1 = 0.f;
                auto a_of = [&](int r) __attribute__((always_inline)) {        // a_i[rb + r]
                    return ap_s[par * kClMaxR + rb + r]
                           + __builtin_ldexpf(bl_s[(par ^ 1) * kClMaxR + rb + r], blsh);
                };
#pragma unroll
                for (int r = 0; r < kClRT; ++r) {
                    const float pr = a_of(r) * E[S][r];
                    if (r & 1) acc1 += pr; else acc0 += pr;
                    if (c == 0) bl_s[par * kClMaxR + rb + r] = pr;
                }
                const float acc = acc0 + acc1;
                if (exch && colok && c >= 1)
                    xstore(xs + (size_t)c * XK + 2 * g.k + half, pack_word(acc, sc[S], tag));
                if (c == 0) ctl_s[2 + par * 2 + half] = sc[S];
                LAST_MARK(a, 0, i, 1);
                if (GAMMA && i >= mid && colok) {
                    const float kx = (float)((double)(ctl_s[6 + par] + sbn[par]) - D2);
                    const float fac = a.scale * fast_exp2(kx + (float)sc[S]) * (c == 0 ? 1.f : bcol[par]);
                    const unsigned gso = (unsigned)i * frb + rbase;
#pragma unroll
                    for (int r = 0; r < kClRT; ++r)
                        if (r < nrt) {
                            // the empty label (column 0) returns to the row's own state
                            const float f2 = (c == 0) ? fac * bv_s[par * kClMaxC + g.r0 + rb + r] : fac;
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
                LAST_MARK(a, 0, i, 2);
                {
                    hcur = prep((S + 1) % D);
                    const int hw = wave_max_dpp(colok ? hcur : kShiftNone);
                    if (lane == 0) ctl_s[8 + (par ^ 1) * 16 + wave] = hw;
                }
                if (GAMMA && i + 1 < n && i + 1 >= mid && colok) bv_s[(par ^ 1) * kClMaxC + c] = bcol[par ^ 1];
                if (exch) gstep += 1;
                LAST_MARK(a, 0, i, 3);
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
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------- beta role
// LDS: b_s[par][q] = b_{t+1} for all states (par = step parity), ctl[par] = its exponent.
template <int D, bool GAMMA, bool ACC, int KT>
__device__ __forceinline__ void beta_role(const ClusterArgs& a, const ClusterGeom& g, float* smem,
                                          unsigned& gstep, unsigned& ptag)
{
    float* b_s = smem;                        // [2][kClMaxC]
    int* ctl_s = (int*)(b_s + 2 * kClMaxC);   // [0..1] exponent, [24] timeout flag
    float* red = (float*)(ctl_s + 32);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool comm = wave == kClWaves;
    const int C = a.C, V1 = a.C;
    // rows of this wave: wave, wave + 10, ... (index inside the workgroup's rows)
    int nrw = 0;
    if (!comm) nrw = (g.nr - wave + kClWaves - 1) / kClWaves;
    if (nrw < 0) nrw = 0;
    const int ncol = (C + 63) / 64;

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

        if (tid == 0) { ctl_s[24] = 0; ctl_s[0] = 0; }
        // both slots: entries for columns >= C stay 0 for the whole item (clamped loads meet them)
        for (int q = tid; q < 2 * kClMaxC; q += blockDim.x) b_s[q] = q < C ? 1.f : 0.f;
        __syncthreads();

        if (comm) {
            // ================= comm wave =================
            int dead = 0, sig = 0;
            for (int i = 0;; ++i) {
                const int par = i & 1;
                const int t = L - 1 - i;
                if (i == 0) {
#pragma unroll
                    for (int j = 0; j < kClNC; ++j) {
                        const int q = lane + 64 * j;
                        if (q < C && q >= g.r0 && q < g.r0 + g.nr) bh[(size_t)L * C + q] = 1.f;
                    }
                    if (lane == 0 && g.k == 0) Sb[L] = 0;
                }
                if (i == ph1) {
                    if (__builtin_amdgcn_ballot_w64(dead != 0) != 0 && lane == 0) ctl_s[24] = 1;
                    cluster_sync(a, g, ptag, dead, &ctl_s[24]);
                    ptag += 1;
                    (void)meeting_value(ah, bh, Sa, Sb, mid, C, red);
                    __syncthreads();
                }
                if (i >= n) break;
                if (i < nex) {
                    const unsigned tag = gstep % 65535u;
                    u64* xs = xbase + (size_t)(gstep & 1) * a.XSB;
                    LAST_MARK(a, 1, i, 0);
                    u64 x[kClNC];
                    int e = -40000;
                    // lane l takes the words l, l + 64, ...: count of valid ones for this lane
                    const int cnt = lane < C ? (C - 1 - lane) / 64 + 1 : 0;
                    poll_words(xs + lane, (size_t)64, cnt, x, tag, a.spin_limit, dead);
#pragma unroll
                    for (int j = 0; j < kClNC; ++j)
                        if (j < cnt) {
                            const float v = word_value(x[j]);
                            if (v > 0.f) e = max(e, word_shift(x[j]) + float_exponent(v) + 1);
                        }
                    LAST_MARK(a, 1, i, 1);
                    int dl = wave_max_dpp(e);
                    if (dl < -30000) dl = 0;
                    sig += dl;
#pragma unroll
                    for (int j = 0; j < kClNC; ++j)
                        if (j < ncol && lane + 64 * j < C) {
                            const int q = lane + 64 * j;
                            const float v = __builtin_ldexpf(word_value(x[j]), word_shift(x[j]) - dl);
                            b_s[(par ^ 1) * kClMaxC + q] = v;
                            if (t >= mid && q >= g.r0 && q < g.r0 + g.nr) bh[(size_t)t * C + q] = v;
                        }
                    if (lane == 0) {
                        ctl_s[par ^ 1] = sig;
                        if (t >= mid && g.k == 0) Sb[t] = sig;
                    }
                    LAST_MARK(a, 1, i, 2);
                    gstep += 1;
                }
                __syncthreads();
            }
        } else {
            // ================= compute waves =================
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
#pragma unroll
            for (int f = 0; f < D - 1; ++f) issue(f, min(f, nlast));
            prep(0);

            int i = 0;
            auto step = [&](auto SLOT) __attribute__((always_inline)) -> bool {
                constexpr int S = decltype(SLOT)::value;
                const int par = i & 1;
                const int t = L - 1 - i;
                if (i == ph1) {
                    int dead = 0;
                    cluster_sync(a, g, ptag, dead, &ctl_s[24]);
                    ptag += 1;
                    D2 = meeting_value(ah, bh, Sa, Sb, mid, C, red);
                    if (GAMMA) {
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
                const unsigned tag = gstep % 65535u;
                u64* xs = xbase + (size_t)(gstep & 1) * a.XSB;
                LAST_MARK(a, 0, i, 0);
                issue((S + D - 1) % D, min(i + D - 1, nlast));      // stream first (see the alpha role)
                float bv[kClNC];
#pragma unroll
                for (int j = 0; j < kClNC; ++j) bv[j] = b_s[par * kClMaxC + lane + 64 * j];
                float brow[kClRW];
#pragma unroll
                for (int ri = 0; ri < kClRW; ++ri) {
                    const int row = g.r0 + min(wave + ri * kClWaves, g.nr - 1);
                    brow[ri] = b_s[par * kClMaxC + row];
                    // the empty label (column 0) returns to the row's own state
                    float acc = E[S][ri][0] * (lane == 0 ? brow[ri] : bv[0]);
#pragma unroll
                    for (int j = 1; j < kClNC; ++j) acc = fmaf(E[S][ri][j], bv[j], acc);
                    const float tot = wave_sum_dpp(acc);
                    if (exch && lane == 0 && ri < nrw) xstore(xs + row, pack_word(tot, sr[S][ri], tag));
                }
                LAST_MARK(a, 0, i, 1);
                if (GAMMA && i >= ph1) {
                    const float kx = (float)((double)(san[par] + ctl_s[par]) - D2);
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
                LAST_MARK(a, 0, i, 2);
                prep((S + 1) % D);
                if (exch) gstep += 1;
                LAST_MARK(a, 0, i, 3);
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
        }
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
    __shared__ float smem[2 * kClMaxR * 2 + 2 * kClMaxC + 48 + 32 + 64];
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
