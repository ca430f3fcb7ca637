// Third generation of the clustered forward-backward for the full 1-gram context dependency with
// exactly 256 labels (C = 257 states; arXiv 2304.13134, Eq. 2 / Eq. 1, Sections 4.1, 4.2.2):
// sixteen workgroups of four waves per role and item, TWO workgroups per compute unit.
//
// The recursion is the one of cluster2_kernels.hpp: an item is walked from both ends at once (K "alpha"
// workgroups upwards, K "beta" workgroups downwards, meeting in the middle, marginals in the second half),
// frames are taken in pairs with ONE exchange per pair (F-step: whole vector -> own states, no
// communication; P-step: own states -> partial sums for all states, published and gathered), arithmetic
// is in the scaled linear domain E = 2^(w log2 e - s).  What changes is the shape of the work:
//   * K = 16 workgroups of 256 threads per role, 256 registers per lane: two workgroups share a compute
//     unit.  They belong to different recursions (or different slices of one), so while one of them sits
//     in a barrier, waits for its exchange or for memory, the other one computes: the overlap that one
//     workgroup in lock-step cannot have comes from the hardware's wave scheduler.
//   * Ownership: workgroup k owns the 16 label states [1 + 16 k, 17 + 16 k); the start state 0, which
//     receives no label arcs, rides along as a 17th state of workgroup 0.  With 256 label states every
//     access is regular: a row of a frame is its empty-label weight followed by 256 label weights, which
//     one wave reads with one 16-byte load per lane ("own rows x all columns": alpha P-step, beta F-step);
//     "all rows x own columns" is read 16 rows per instruction, four lanes x 16 bytes per row (alpha
//     F-step, beta P-step).  The start state's row (or, in the other pattern, workgroup 0's 17th row) is a
//     fifth, mostly masked, instruction per frame.
//   * One shift s per WAVE and frame (largest weight of the wave's share), applied when the waves'
//     partial sums meet: no maxima through LDS, no barrier in the exp pass.  The empty-label weights of
//     the own states have a shift of their own, the same in every wave.
//   * Exchange words as before, [value:32 | tag:16 | exponent:16], but gathered two words per 16-byte load:
//     a lane pair shares two neighbouring states and splits the sixteen producers; the halves meet through
//     one DPP swap.  The start state's sixteen words sit on sixteen lanes and are added up by a DPP scan.
//     The order of every addition is fixed, so the gathered vector is bit-identical in all workgroups.
//
// Per pair and workgroup (alpha; beta mirrors it): F-step sums -> barrier -> own states (every wave by
// itself) -> P-step sums -> barrier -> publish -> marginals of the pair (second half of the item) -> exp
// pass of the NEXT pair, with the first look at the exchange and the requests for the pair after the next
// in its middle -> gather (two barriers).  Requests run one pair ahead of the exp pass that consumes them;
// the look is issued before them, because a wave's loads return in order.
#pragma once
#include "cluster2_kernels.hpp"

namespace last {

constexpr int kC3Threads = 256;
constexpr int kC3Waves = 4;
constexpr int kC3K = 16;        // workgroups per role and item
constexpr int kC3C = 257;       // states: the start state and 256 label states
constexpr int kC3XS = 272;      // exchange words per producer and slot (257 used; even: word pairs are 16-byte aligned)
constexpr int kC3RS = 20;       // LDS pitch of a column's sixteen partial sums (conflict-free 16-byte reads)
constexpr unsigned kC3Sc1 = 16; // cache policy of the exchange loads: agent scope, served by the XCD's L2

// LDS map (floats / ints)
constexpr int kC3Full = 0;                      // [272] whole state vector: label state y at y - 1, the start state at 256
constexpr int kC3Red = kC3Full + 272;           // [16][20] alpha F-step: partial sums per own column; [272] beta P-step: row sums
constexpr int kC3Pacc = kC3Red + 16 * kC3RS;    // [4][256] alpha P-step: partial sums per wave and column
constexpr int kC3Bl = kC3Pacc + 4 * 256;        // [32] empty-label terms of the own states
constexpr int kC3OwnS = kC3Bl + 32;             // [32] own states (beta)
constexpr int kC3Row = kC3OwnS + 32;            // [32] beta F-step: row sums, [32] their shifts
constexpr int kC3Ctl = kC3Row + 64;             // [32] ints: [0] exponent of full_s, [4..7] F shifts, [8] timeout,
                                                //            [11] range, [12..15] P shifts, [24..27] gather maxima
constexpr int kC3RedB = kC3Ctl + 32;            // [32] block reductions
constexpr int kC3Lds = kC3RedB + 32;
static_assert(kC3Red % 4 == 0 && kC3Pacc % 4 == 0 && kC3OwnS % 4 == 0 && kC3Ctl % 4 == 0, "16-byte LDS accesses");

#ifdef LAST_TRACE
#define C3_MARK(a, p, k)                                                                     \
    do {                                                                                     \
        if ((a).trace && (p) < 64 && threadIdx.x == 0)                                       \
            (a).trace[((size_t)blockIdx.x * 64 + (p)) * 16 + (k)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#define C3_NOTE(a, p, k, v)                                                                  \
    do {                                                                                     \
        if ((a).trace && (p) < 64 && threadIdx.x == 0)                                       \
            (a).trace[((size_t)blockIdx.x * 64 + (p)) * 16 + (k)] = (unsigned long long)(v); \
    } while (0)
#elif defined(C3_ASM_MARKS)
#define C3_MARK(a, p, k) asm volatile("; C3SEC " #k)
#define C3_NOTE(a, p, k, v) do { } while (0)
#else
#define C3_MARK(a, p, k) do { } while (0)
#define C3_NOTE(a, p, k, v) do { } while (0)
#endif

__device__ __forceinline__ uint4 c3_xload4(buf_t r, unsigned voff, unsigned soff)
{
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, (int)kC3Sc1);
    return __builtin_bit_cast(uint4, v);
}
__device__ __forceinline__ uint2 c3_xload2(buf_t r, unsigned voff, unsigned soff)
{
    const auto v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, (int)kC3Sc1);
    return __builtin_bit_cast(uint2, v);
}

// 2^(e - D) for a marginal, capped so that it stays finite; the largest exponent seen is kept for the
// range flag (see c2_marginal_scale)
__device__ __forceinline__ float c3_mscale(int e, double D2, float& xmax)
{
    const float x = (float)((double)e - D2);
    xmax = fmaxf(xmax, x);
    return fast_exp2(fminf(x, 126.f));
}

__device__ __forceinline__ float c3_max4(const float (&x)[4])
{
    return fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
}

// One exchange slot as a thread sees it: two neighbouring label states from eight producers (the lane
// pair's other lane has the other eight) and one of the sixteen words of the start state.
struct C3Look {
    uint4 q[8];
    uint2 z;
};

__device__ __forceinline__ void c3_look(buf_t xrs, unsigned slot_off, unsigned voffq, unsigned voffz, C3Look& lk)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) lk.q[j] = c3_xload4(xrs, voffq, slot_off + (unsigned)(j * kC3XS * 8));
    lk.z = c3_xload2(xrs, voffz, slot_off);
}

// Gathering one exchange slot: the sixteen partial values of every state, added up in a fixed order
// relative to the largest producer exponent; the vector ends in full_s, renormalised by the largest
// magnitude present, its exponent in ctl_s[0].  Every thread calls; ends with a workgroup barrier.
// `after_poll` runs once all words are there, before they are added up.
template <typename AfterPoll>
__device__ __forceinline__ void c3_gather(buf_t xrs, unsigned slot_off, unsigned voffq, unsigned voffz, unsigned tag,
                                          float* full_s, int* ctl_s, int limit, int& dead, C3Look& lk,
                                          AfterPoll&& after_poll, int* relooks = nullptr)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S0 = ctl_s[0];
    const unsigned tagw = (tag & 0xFFFFu) << 16;
    int n = 0;
    for (;;) {
        unsigned diff = lk.z.y ^ tagw;
#pragma unroll
        for (int j = 0; j < 8; ++j) diff |= (lk.q[j].y ^ tagw) | (lk.q[j].w ^ tagw);
        if ((diff >> 16) == 0 || dead) break;
        if (++n > limit) { dead = 1; break; }
        __builtin_amdgcn_s_sleep(1);
        c3_look(xrs, slot_off, voffq, voffz, lk);
    }
    if (relooks) *relooks = n;
    after_poll();
    int e[8];
    int hm = -(1 << 30);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        e[j] = (int)(short)(unsigned short)lk.q[j].y;
        hm = max(hm, e[j]);
    }
    float vlo = 0.f, vhi = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        vlo += __builtin_ldexpf(__uint_as_float(lk.q[j].x), e[j] - hm);      // (16-bit exponents: differences in [-65535, 0])
        vhi += __builtin_ldexpf(__uint_as_float(lk.q[j].z), e[j] - hm);
    }
    // the other eight producers of the same two states: the neighbouring lane (float addition commutes,
    // so both lanes of a pair end up with the same bits)
    const int ho = dpp_i<0xB1>(hm, hm);
    const float olo = dpp_f<0xB1>(vlo, vlo), ohi = dpp_f<0xB1>(vhi, vhi);
    const int href = max(hm, ho);
    vlo = __builtin_ldexpf(vlo, hm - href) + __builtin_ldexpf(olo, ho - href);
    vhi = __builtin_ldexpf(vhi, hm - href) + __builtin_ldexpf(ohi, ho - href);
    // the start state: lane l of every row of sixteen holds producer l's word; a scan leaves the sum in lane 15
    float vz = __builtin_ldexpf(__uint_as_float(lk.z.x), (int)(short)(unsigned short)lk.z.y - href);
    vz += dpp_f<0x111>(0.f, vz);
    vz += dpp_f<0x112>(0.f, vz);
    vz += dpp_f<0x114>(0.f, vz);
    vz += dpp_f<0x118>(0.f, vz);
    const float v0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(vz), 15));
    // renormalise by the largest magnitude actually present (non-negative floats order like integers)
    int mub = wave_max_dpp(max(__float_as_int(vlo), __float_as_int(vhi)));
    mub = max(mub, __float_as_int(v0));
    if (lane == 0) ctl_s[24 + wave] = mub;
    if (dead) ctl_s[8] = 1;
    c2_barrier();
    const int4 m0 = *(const int4*)&ctl_s[24];
    const int mxb = max(max(m0.x, m0.y), max(m0.z, m0.w));
    const int mx = mxb > 0 ? float_exponent(__int_as_float(mxb)) : 0;
    full_s[tid] = c2_scale((tid & 1) ? vhi : vlo, -mx);
    if (tid == 0) {
        full_s[256] = c2_scale(v0, -mx);
        ctl_s[0] = S0 + href + mx;
    }
    c2_barrier();
}

// D = log2 sum_q a_mid[q] b_mid[q] with one exponent per block of states on either side
// (block of the start state: 0; of label state q: (q - 1) / 16)
__device__ __forceinline__ double c3_meeting(const float* ah, const float* bh, const int* Sa, const int* Sb, float* red)
{
    int xmax = -(1 << 30);
    for (int k = 0; k < kC3K; ++k) xmax = max(xmax, Sa[k] + Sb[k]);
    float part = 0.f;
    for (int q = threadIdx.x; q < kC3C; q += blockDim.x) {
        const int k = q == 0 ? 0 : (q - 1) >> 4;
        part += c2_scale(ah[q] * bh[q], Sa[k] + Sb[k] - xmax);
    }
    const float tot = block_sum(part, red);
    return (double)xmax + (double)__log2f(tot);
}

// When the last workgroup of an item is through: an item on which any workgroup gave up waiting gets
// dist = NaN and status 5, whoever wrote dist before.  fin: [B][2] words, cleared to ~0 before the launch:
// [0] counts the workgroups that are through, [1] is written by a workgroup that timed out.
__device__ __forceinline__ void c3_finish_item(const ClusterArgs& a, int b, bool timed_out, bool bad)
{
    u64* fin = a.fin + (size_t)b * 2;
    if (timed_out) __hip_atomic_store(fin + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    const u64 old = __hip_atomic_fetch_add(fin, 1ull, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (u64)(2 * kC3K - 2)) {
        __threadfence();
        if (__hip_atomic_load(fin + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != ~0ull && !bad) {
            __hip_atomic_store(a.dist + b, __builtin_nanf(""), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.item_status)
                __hip_atomic_store(a.item_status + b, (int)kItemTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Geometry shared by both roles.  "Row pattern": a wave takes four rows of the workgroup's sixteen (and
// wave 0 of workgroup 0 the start state's row), a lane four neighbouring label columns of each.  "Column
// pattern": a wave takes 64 of the 256 label states' rows (and wave 0 the start state's), sixteen per
// instruction, a lane four of the workgroup's sixteen columns.
struct C3Geom {
    int lane, wave, k;
    int rg, ci;            // column pattern: row inside the instruction, quad of own columns
    bool xC, xR;           // the lane (column pattern) / the wave (row pattern) has the extra row
    bool olane;            // lane <-> own state: 0..15 the label states, 16 the start state (workgroup 0)
    int ostate, oidx;      // that state and its place in full_s
    unsigned voffC, voffCx, voffR, voffRx, voffB;
    unsigned rowC0, rowR0; // scalar: first row of the wave in either pattern
};
__device__ __forceinline__ C3Geom c3_geom(int k)
{
    constexpr unsigned pitch = kC3C * 4u;
    C3Geom g;
    g.lane = threadIdx.x & 63;
    g.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    g.k = k;
    g.rg = g.lane >> 2;
    g.ci = g.lane & 3;
    g.xC = g.wave == 0 && g.rg == 0;
    g.xR = k == 0 && g.wave == 0;
    g.olane = g.lane < 16 || (g.lane == 16 && k == 0);
    g.ostate = g.lane < 16 ? 1 + 16 * k + g.lane : 0;
    g.oidx = g.lane < 16 ? 16 * k + g.lane : 256;
    g.voffC = (unsigned)(1 + g.rg) * pitch + (unsigned)(1 + 16 * k + 4 * g.ci) * 4u;
    g.voffCx = g.xC ? (unsigned)(1 + 16 * k + 4 * g.ci) * 4u : kC2Off;
    g.voffR = (unsigned)(1 + 4 * g.lane) * 4u;
    g.voffRx = g.xR ? g.voffR : kC2Off;
    g.voffB = g.olane ? (unsigned)g.ostate * pitch : kC2Off;
    g.rowC0 = (unsigned)(64 * g.wave) * pitch;
    g.rowR0 = (unsigned)(1 + 16 * k + 4 * g.wave) * pitch;
    return g;
}

// A frame's share of one lane: five slots of four neighbouring weights, and an empty-label weight.
struct C3Frame {
    float e[5][4];
    float b;
};
__device__ __forceinline__ void c3_load_cols(C3Frame& f, buf_t wrs, const C3Geom& g, unsigned fo)
{
    constexpr unsigned pitch = kC3C * 4u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float4 x = buf_load4(wrs, g.voffC, fo + g.rowC0 + (unsigned)(16 * j) * pitch);
        f.e[j][0] = x.x; f.e[j][1] = x.y; f.e[j][2] = x.z; f.e[j][3] = x.w;
    }
    const float4 x = buf_load4(wrs, g.voffCx, fo);
    f.e[4][0] = x.x; f.e[4][1] = x.y; f.e[4][2] = x.z; f.e[4][3] = x.w;
    f.b = buf_load(wrs, g.voffB, fo);
}
__device__ __forceinline__ void c3_load_rows(C3Frame& f, buf_t wrs, const C3Geom& g, unsigned fo)
{
    constexpr unsigned pitch = kC3C * 4u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float4 x = buf_load4(wrs, g.voffR, fo + g.rowR0 + (unsigned)j * pitch);
        f.e[j][0] = x.x; f.e[j][1] = x.y; f.e[j][2] = x.z; f.e[j][3] = x.w;
    }
    const float4 x = buf_load4(wrs, g.voffRx, fo);
    f.e[4][0] = x.x; f.e[4][1] = x.y; f.e[4][2] = x.z; f.e[4][3] = x.w;
    f.b = buf_load(wrs, g.voffB, fo);
}
// exp pass of one frame: E = 2^(w log2 e - s), s the wave's shift (sw), and sb the shift of the own states'
// empty-label weights (the same in every wave).  `extra`: the lane holds the fifth slot.
__device__ __forceinline__ void c3_exp_frame(C3Frame& f, bool extra, bool olane, int& sw, int& sb)
{
    float m = fmaxf(fmaxf(c3_max4(f.e[0]), c3_max4(f.e[1])), fmaxf(c3_max4(f.e[2]), c3_max4(f.e[3])));
    m = extra ? fmaxf(m, c3_max4(f.e[4])) : m;
    const int s = shift_for(wave_max_dpp(m));
    const float fs = (float)s;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f.e[j][c] = fast_exp2(fmaf(f.e[j][c], kLog2e, -fs));
            c2_pin(f.e[j][c]);
        }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        f.e[4][c] = extra ? fast_exp2(fmaf(f.e[4][c], kLog2e, -fs)) : 0.f;
        c2_pin(f.e[4][c]);
    }
    const int s2 = shift_for(wave_max_dpp(olane ? f.b : LAST_NEG_INF));
    f.b = olane ? fast_exp2(fmaf(f.b, kLog2e, -(float)s2)) : 0.f;
    c2_pin(f.b);
    sw = s;
    sb = s2;
}

// four marginals of one row slot: two 8-byte stores
template <bool ACC>
__device__ __forceinline__ void c3_put4(const float (&x)[4], buf_t grs, unsigned voff, unsigned soff)
{
    c2_put2<ACC>(x[0], x[1], grs, voff, soff, true, true);
    c2_put2<ACC>(x[2], x[3], grs, voff + 8u, soff, true, true);
}

// ------------------------------------------------------------------ alpha role
template <bool GAMMA, bool ACC>
__device__ __forceinline__ void alpha3_role(const ClusterArgs& a, const ClusterGeom& cg, float* smem,
                                            unsigned& gstep, unsigned& ptag)
{
    constexpr int C = kC3C;
    constexpr unsigned pitch = C * 4u, frb = (unsigned)C * C * 4u;
    float* full_s = smem + kC3Full;
    float* red_s = smem + kC3Red;
    float* pacc_s = smem + kC3Pacc;
    float* bl_s = smem + kC3Bl;
    int* ctl_s = (int*)(smem + kC3Ctl);
    float* redb = smem + kC3RedB;
    const int tid = threadIdx.x;
    const C3Geom g = c3_geom(cg.k);
    const int lane = g.lane, wave = g.wave, k = g.k;
    const unsigned voffq = (unsigned)((8 * (tid & 1)) * kC3XS + 2 * (tid >> 1)) * 8u;
    const unsigned voffz = (unsigned)((lane & 15) * kC3XS + 256) * 8u;

    for (int b = cg.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : mid;
        const int nlast = max(n - 1, 0);
        const size_t fr = (size_t)C * C;
        float* ah = a.ahat + (size_t)b * (a.T + 1) * C;
        const float* bh = a.bhat + (size_t)b * (a.T + 1) * C;
        int* Sa = a.Sa + (size_t)b * (a.T + 1) * kC3K;
        const int* Sb = a.Sb + (size_t)b * (a.T + 1) * kC3K;
        u64* xbase = a.xa + (size_t)cg.cg * 2 * kC3K * kC3XS;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        const buf_t brs = make_buf(bh, (unsigned)(a.T + 1) * pitch);
        const buf_t sbrs = make_buf(Sb, (unsigned)(a.T + 1) * (unsigned)(kC3K * sizeof(int)));
        const buf_t xrs = make_buf(xbase, (unsigned)(2 * kC3K * kC3XS * sizeof(u64)));

        // a_0 = unit vector at the start state, exponent 0
        for (int q = tid; q < 272; q += kC3Threads) full_s[q] = q == 256 ? 1.f : 0.f;
        if (tid < 32) { ctl_s[tid] = 0; bl_s[tid] = 0.f; }
        if (wave == 0 && g.olane) ah[g.ostate] = g.ostate == 0 ? 1.f : 0.f;
        if (tid == 0) Sa[k] = 0;
        __syncthreads();

        C3Frame EF[2], EP[2];
        int sF[2] = {0, 0}, sP[2] = {0, 0}, sFb[2] = {0, 0}, sPb[2] = {0, 0};
        // the other side's vectors for the marginals
        float bF4[2][4], bP4[2][4], bFo[2] = {0.f, 0.f}, bPo[2] = {0.f, 0.f};
        int sbF[2] = {0, 0}, sbP[2] = {0, 0}, sbPl[2] = {0, 0};
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int c = 0; c < 4; ++c) { bF4[x][c] = 0.f; bP4[x][c] = 0.f; }
        double D2 = 0.0;
        float xwide = -3.0e38f;
        int dead = 0;
        bool met = false;

        // state vectors of the other side for the marginals of pair p (rows t + 1 of its two frames);
        // fetched with the pair's frames, and again right after the meeting for the pairs in flight
        auto other = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned tF1 = (unsigned)(min(2 * p, nlast) + 1), tP1 = (unsigned)(min(2 * p + 1, nlast) + 1);
            const float4 x = buf_load4(brs, (unsigned)(1 + 16 * k + 4 * g.ci) * 4u, tF1 * pitch);
            bF4[B_][0] = x.x; bF4[B_][1] = x.y; bF4[B_][2] = x.z; bF4[B_][3] = x.w;
            bFo[B_] = buf_load(brs, (unsigned)g.ostate * 4u, tF1 * pitch);
            // block exponents: one per lane, picked where they are used (a wave-uniform address would make
            // these scalar loads, and every workgroup barrier waits for those)
            sbF[B_] = __builtin_bit_cast(int, buf_load(sbrs, (unsigned)(lane & 15) * 4u, tF1 * (unsigned)(kC3K * sizeof(int))));
            const float4 y = buf_load4(brs, g.voffR, tP1 * pitch);
            bP4[B_][0] = y.x; bP4[B_][1] = y.y; bP4[B_][2] = y.z; bP4[B_][3] = y.w;
            bPo[B_] = buf_load(brs, (unsigned)g.ostate * 4u, tP1 * pitch);
            sbP[B_] = __builtin_bit_cast(int, buf_load(sbrs, (unsigned)(lane & 15) * 4u, tP1 * (unsigned)(kC3K * sizeof(int))));
            sbPl[B_] = __builtin_bit_cast(int, buf_load(sbrs, (unsigned)(lane >> 2) * 4u, tP1 * (unsigned)(kC3K * sizeof(int))));
        };
        auto settle = [&]() __attribute__((always_inline)) {
            int t = 0;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
#pragma unroll
                for (int c = 0; c < 4; ++c) t |= c2_touch(bF4[x][c]) | c2_touch(bP4[x][c]);
                t |= c2_touch(bFo[x]) | c2_touch(bPo[x]) | (sbF[x] == 0x7fffffff) | (sbP[x] == 0x7fffffff) | (sbPl[x] == 0x7fffffff);
            }
            if (t) ctl_s[9] = 1;          // (never; nobody reads it)
        };
        auto issue = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_load_cols(EF[B_], wrs, g, (unsigned)min(2 * p, nlast) * frb);
            c3_load_rows(EP[B_], wrs, g, (unsigned)min(2 * p + 1, nlast) * frb);
            if (GAMMA) other(BUF, p);
        };
        auto prep = [&](auto BUF, auto&& halfway) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_exp_frame(EF[B_], g.xC, g.olane, sF[B_], sFb[B_]);
            halfway();
            c3_exp_frame(EP[B_], g.xR, g.olane, sP[B_], sPb[B_]);
            if (GAMMA) {
#pragma unroll
                for (int c = 0; c < 4; ++c) { c2_pin(bF4[B_][c]); c2_pin(bP4[B_][c]); }
                c2_pin(bFo[B_]); c2_pin(bPo[B_]); c2_pin(sbF[B_]); c2_pin(sbP[B_]); c2_pin(sbPl[B_]);
            }
        };
        auto meet = [&]() __attribute__((always_inline)) {
            if (dead) ctl_s[8] = 1;
            cluster_sync(a, cg, ptag, &ctl_s[8]);
            ptag += 1;
            D2 = c3_meeting(ah + (size_t)mid * C, bh + (size_t)mid * C, Sa + (size_t)mid * kC3K,
                            Sb + (size_t)mid * kC3K, redb);
            if (k == 0 && tid == 0) {
                a.dist[b] = bad ? __builtin_nanf("") : (float)(D2 * 0.6931471805599453);
                if (a.item_status) a.item_status[b] = bad ? kItemBadLength : kItemOk;
            }
            met = true;
            __syncthreads();
        };

        issue(std::integral_constant<int, 0>(), 0);
        issue(std::integral_constant<int, 1>(), 1);
        prep(std::integral_constant<int, 0>(), [] {});

        int p = 0;
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value;
            const int tF = 2 * p, tP = 2 * p + 1;
            if (tF >= n) return false;
            auto after_meeting = [&]() __attribute__((always_inline)) {
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B_ ^ 1>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            };
            // ---------------- F-step: frame tF, all rows x own columns, from the whole vector
            if (tF == mid && !met) { meet(); after_meeting(); }
            C3_MARK(a, p, 0);
            const int S = ctl_s[0];
            float own;
            int ek;
            {
                float aq[5];
#pragma unroll
                for (int j = 0; j < 4; ++j) aq[j] = full_s[64 * wave + 16 * j + g.rg];
                aq[4] = g.xC ? full_s[256] : 0.f;
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 5; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = fmaf(aq[j], EF[B_].e[j][c], acc[c]);
                // the four rows of a group of sixteen lanes
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    acc[c] += dpp_f<0x114>(0.f, acc[c]);
                    acc[c] += dpp_f<0x118>(0.f, acc[c]);
                }
                if ((lane & 15) >= 12) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) red_s[(4 * g.ci + c) * kC3RS + 4 * wave + (lane >> 4)] = acc[c];
                }
                if (lane == 0) ctl_s[4 + wave] = sF[B_];
                if (GAMMA && tF >= mid) {
                    const int sbk = __builtin_amdgcn_readlane(sbF[B_], k);
                    const float fcs = a.scale * c3_mscale(S + sF[B_] + sbk, D2, xwide);
                    const unsigned gso = (unsigned)tF * frb;
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = aq[j] * EF[B_].e[j][c] * (bF4[B_][c] * fcs);
                        c3_put4<ACC>(x, grs, j < 4 ? g.voffC : g.voffCx, j < 4 ? gso + g.rowC0 + (unsigned)(16 * j) * pitch : gso);
                    }
                    if (wave == 0) {
                        const float fb = a.scale * bFo[B_] * c3_mscale(S + sFb[B_] + sbk, D2, xwide);
                        c2_put<ACC>(full_s[g.oidx] * EF[B_].b * fb, grs, g.voffB, gso);
                    }
                }
                C3_MARK(a, p, 1);
                c2_barrier();
                C3_MARK(a, p, 2);
                // own states: every wave by itself (the same values from the same inputs)
                const int4 sh = *(const int4*)&ctl_s[4];
                const int smax = max(max(max(sh.x, sh.y), max(sh.z, sh.w)), sFb[B_]);
                const float4* rp = (const float4*)&red_s[(lane & 15) * kC3RS];
                const float4 p0 = rp[0], p1 = rp[1], p2 = rp[2], p3 = rp[3];
                float v = c2_scale((p0.x + p0.y) + (p0.z + p0.w), sh.x - smax) + c2_scale((p1.x + p1.y) + (p1.z + p1.w), sh.y - smax)
                          + c2_scale((p2.x + p2.y) + (p2.z + p2.w), sh.z - smax) + c2_scale((p3.x + p3.y) + (p3.z + p3.w), sh.w - smax);
                v = lane < 16 ? v : 0.f;
                v = fmaf(full_s[g.oidx], c2_scale(EF[B_].b, sFb[B_] - smax), v);
                const int te = v > 0.f ? float_exponent(v) : kShiftNone;
                const int ms = wave_max_dpp(te);
                own = v > 0.f ? c2_scale(v, -ms) : 0.f;
                ek = ms == kShiftNone ? S : S + smax + ms;
                if (tF + 1 <= mid && wave == 0) {
                    if (g.olane) ah[(size_t)(tF + 1) * C + g.ostate] = own;
                    if (lane == 0) Sa[(size_t)(tF + 1) * kC3K + k] = ek;
                }
            }
            if (tP >= n) return false;
            C3_MARK(a, p, 3);
            // ---------------- P-step: frame tP, own rows x all columns, partial sums for every state
            if (tP == mid && !met) { meet(); after_meeting(); }
            {
                const unsigned tag = gstep + 1;
                const unsigned slot_off = (gstep & 1) * (unsigned)(kC3K * kC3XS * sizeof(u64));
                u64* xs = xbase + (size_t)(gstep & 1) * kC3K * kC3XS;
                float o[5];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(own), 4 * wave + j));
                o[4] = g.xR ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(own), 16)) : 0.f;
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 5; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = fmaf(o[j], EP[B_].e[j][c], acc[c]);
                float4 av;
                av.x = acc[0]; av.y = acc[1]; av.z = acc[2]; av.w = acc[3];
                *(float4*)&pacc_s[wave * 256 + 4 * lane] = av;
                if (lane == 0) ctl_s[12 + wave] = sP[B_];
                if (wave == 0 && lane < 32) bl_s[lane] = own * EP[B_].b;
                C3_MARK(a, p, 4);
                c2_barrier();
                C3_MARK(a, p, 5);
                const int4 sp = *(const int4*)&ctl_s[12];
                const int spmax = max(max(max(sp.x, sp.y), max(sp.z, sp.w)), sPb[B_]);
                float val = c2_scale(pacc_s[tid], sp.x - spmax) + c2_scale(pacc_s[256 + tid], sp.y - spmax)
                            + c2_scale(pacc_s[512 + tid], sp.z - spmax) + c2_scale(pacc_s[768 + tid], sp.w - spmax);
                if ((tid >> 4) == k) val += c2_scale(bl_s[tid & 15], sPb[B_] - spmax);
                const int rel = (spmax == kShiftNone ? ek : ek + spmax) - S;
                const bool exch = !(GAMMA && tP == L - 1);
                if (exch) {
                    xpublish(xs + (size_t)k * kC3XS + tid, c2_pack(val, tag, rel));
                    // the start state moves on by its empty-label arc only: workgroup 0 has it, the others add zero
                    if (tid == 0)
                        xpublish(xs + (size_t)k * kC3XS + 256, c2_pack(k == 0 ? c2_scale(bl_s[16], sPb[B_] - spmax) : 0.f, tag, rel));
                }
                if (GAMMA && tP >= mid) {
                    const int sbk = __builtin_amdgcn_readlane(sbP[B_], k);
                    const float fys = a.scale * c3_mscale(ek + sP[B_] + sbPl[B_], D2, xwide);
                    const unsigned gso = (unsigned)tP * frb;
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = o[j] * EP[B_].e[j][c] * (bP4[B_][c] * fys);
                        c3_put4<ACC>(x, grs, j < 4 ? g.voffR : g.voffRx, j < 4 ? gso + g.rowR0 + (unsigned)j * pitch : gso);
                    }
                    if (wave == 0) {
                        const float fb = a.scale * bPo[B_] * c3_mscale(ek + sPb[B_] + sbk, D2, xwide);
                        c2_put<ACC>(own * EP[B_].b * fb, grs, g.voffB, gso);
                    }
                }
                // exp pass of the next pair; in its middle the first look at the exchange and, behind it (a
                // wave's loads return in order), the requests for the pair after the next, into the registers
                // this pair has finished with
                C3_MARK(a, p, 6);
                C3Look lk;
                prep(std::integral_constant<int, B_ ^ 1>(), [&]() __attribute__((always_inline)) {
                    if (exch) c3_look(xrs, slot_off, voffq, voffz, lk);
                    issue(std::integral_constant<int, B_>(), p + 2);
                });
                C3_MARK(a, p, 7);
                if (exch) {
                    int relooks = 0;
                    c3_gather(xrs, slot_off, voffq, voffz, tag, full_s, ctl_s, a.spin_limit, dead, lk,
                              [&]() __attribute__((always_inline)) { C3_MARK(a, p, 8); }, &relooks);
                    C3_MARK(a, p, 9);
                    C3_NOTE(a, p, 10, relooks);
                    gstep += 1;
                    if (tP + 1 <= mid && wave == 1) {
                        if (g.olane) ah[(size_t)(tP + 1) * C + g.ostate] = full_s[g.oidx];
                        if (lane == 0) Sa[(size_t)(tP + 1) * kC3K + k] = ctl_s[0];
                    }
                }
            }
            ++p;
            return true;
        };
        for (;;) {
            if (!pair(std::integral_constant<int, 0>())) break;
            if (!pair(std::integral_constant<int, 1>())) break;
        }
        __syncthreads();
        if (!met) meet();
        if (xwide > kC2RangeBits) ctl_s[11] = 1;
        if (dead) ctl_s[8] = 1;
        __syncthreads();
        if (tid == 0) {
            if (ctl_s[11] && a.item_status && !bad) atomicMax(&a.item_status[b], (int)kItemRange);
            c3_finish_item(a, b, ctl_s[8] != 0, bad);
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------- beta role
template <bool GAMMA, bool ACC>
__device__ __forceinline__ void beta3_role(const ClusterArgs& a, const ClusterGeom& cg, float* smem,
                                           unsigned& gstep, unsigned& ptag)
{
    constexpr int C = kC3C;
    constexpr unsigned pitch = C * 4u, frb = (unsigned)C * C * 4u;
    float* full_s = smem + kC3Full;
    float* rowp_s = smem + kC3Red;            // [272] P-step: row sums (label state y at y - 1, the start state at 256)
    float* bl_s = smem + kC3Bl;
    float* own_s = smem + kC3OwnS;
    float* row_s = smem + kC3Row;             // [32] F-step: row sums
    int* rsh_s = (int*)(smem + kC3Row + 32);  // [32] their shifts
    int* ctl_s = (int*)(smem + kC3Ctl);
    float* redb = smem + kC3RedB;
    const int tid = threadIdx.x;
    const C3Geom g = c3_geom(cg.k);
    const int lane = g.lane, wave = g.wave, k = g.k;
    const unsigned voffq = (unsigned)((8 * (tid & 1)) * kC3XS + 2 * (tid >> 1)) * 8u;
    const unsigned voffz = (unsigned)((lane & 15) * kC3XS + 256) * 8u;

    for (int b = cg.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : L - mid;
        const int ph1 = L - mid;                      // step at which the state index reaches mid
        const int nlast = max(n - 1, 0);
        const size_t fr = (size_t)C * C;
        const float* ah = a.ahat + (size_t)b * (a.T + 1) * C;
        float* bh = a.bhat + (size_t)b * (a.T + 1) * C;
        const int* Sa = a.Sa + (size_t)b * (a.T + 1) * kC3K;
        int* Sb = a.Sb + (size_t)b * (a.T + 1) * kC3K;
        u64* xbase = a.xb + (size_t)cg.cg * 2 * kC3K * kC3XS;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        const buf_t ars = make_buf(ah, (unsigned)(a.T + 1) * pitch);
        const buf_t sars = make_buf(Sa, (unsigned)(a.T + 1) * (unsigned)(kC3K * sizeof(int)));
        const buf_t xrs = make_buf(xbase, (unsigned)(2 * kC3K * kC3XS * sizeof(u64)));

        // b_L = 1 for every state, exponent 0
        for (int q = tid; q < 272; q += kC3Threads) full_s[q] = q < C ? 1.f : 0.f;
        if (tid < 32) { ctl_s[tid] = 0; bl_s[tid] = 0.f; own_s[tid] = 0.f; row_s[tid] = 0.f; rsh_s[tid] = kShiftNone; }
        if (wave == 0 && g.olane) bh[(size_t)L * C + g.ostate] = 1.f;
        if (tid == 0) Sb[(size_t)L * kC3K + k] = 0;
        __syncthreads();

        C3Frame EF[2], EP[2];
        int sF[2] = {0, 0}, sP[2] = {0, 0}, sFb[2] = {0, 0}, sPb[2] = {0, 0};
        // the other side's vectors for the marginals
        float aFo[2] = {0.f, 0.f}, aPo[2] = {0.f, 0.f}, aP[2][5];
        int saF[2] = {0, 0}, saP[2] = {0, 0};
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int j = 0; j < 5; ++j) aP[x][j] = 0.f;
        double D2 = 0.0;
        float xwide = -3.0e38f;
        int dead = 0;
        bool met = false;

        // step index i -> frame L - 1 - i; pair p = steps 2p (F) and 2p + 1 (P)
        auto frameF = [&](int p) { return max(L - 1 - min(2 * p, nlast), 0); };
        auto frameP = [&](int p) { return max(L - 1 - min(2 * p + 1, nlast), 0); };
        auto other = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned tF = (unsigned)frameF(p), tP = (unsigned)frameP(p);
            aFo[B_] = buf_load(ars, (unsigned)g.ostate * 4u, tF * pitch);
            saF[B_] = __builtin_bit_cast(int, buf_load(sars, (unsigned)(lane & 15) * 4u, tF * (unsigned)(kC3K * sizeof(int))));
#pragma unroll
            for (int j = 0; j < 4; ++j)
                aP[B_][j] = buf_load(ars, (unsigned)(1 + 64 * wave + 16 * j + g.rg) * 4u, tP * pitch);
            aP[B_][4] = buf_load(ars, g.xC ? 0u : kC2Off, tP * pitch);
            aPo[B_] = buf_load(ars, (unsigned)g.ostate * 4u, tP * pitch);
            saP[B_] = __builtin_bit_cast(int, buf_load(sars, (unsigned)(lane & 15) * 4u, tP * (unsigned)(kC3K * sizeof(int))));
        };
        auto settle = [&]() __attribute__((always_inline)) {
            int t = 0;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
#pragma unroll
                for (int j = 0; j < 5; ++j) t |= c2_touch(aP[x][j]);
                t |= c2_touch(aFo[x]) | c2_touch(aPo[x]) | (saF[x] == 0x7fffffff) | (saP[x] == 0x7fffffff);
            }
            if (t) ctl_s[9] = 1;          // (never; nobody reads it)
        };
        auto issue = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_load_rows(EF[B_], wrs, g, (unsigned)frameF(p) * frb);
            c3_load_cols(EP[B_], wrs, g, (unsigned)frameP(p) * frb);
            if (GAMMA) other(BUF, p);
        };
        auto prep = [&](auto BUF, auto&& halfway) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_exp_frame(EF[B_], g.xR, g.olane, sF[B_], sFb[B_]);
            halfway();
            c3_exp_frame(EP[B_], g.xC, g.olane, sP[B_], sPb[B_]);
            if (GAMMA) {
#pragma unroll
                for (int j = 0; j < 5; ++j) c2_pin(aP[B_][j]);
                c2_pin(aFo[B_]); c2_pin(aPo[B_]); c2_pin(saF[B_]); c2_pin(saP[B_]);
            }
        };
        auto meet = [&]() __attribute__((always_inline)) {
            if (dead) ctl_s[8] = 1;
            cluster_sync(a, cg, ptag, &ctl_s[8]);
            ptag += 1;
            D2 = c3_meeting(ah + (size_t)mid * C, bh + (size_t)mid * C, Sa + (size_t)mid * kC3K,
                            Sb + (size_t)mid * kC3K, redb);
            met = true;
            __syncthreads();
        };

        issue(std::integral_constant<int, 0>(), 0);
        issue(std::integral_constant<int, 1>(), 1);
        prep(std::integral_constant<int, 0>(), [] {});

        int p = 0;
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value;
            const int iF = 2 * p, iP = 2 * p + 1;
            if (iF >= n) return false;
            auto after_meeting = [&]() __attribute__((always_inline)) {
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B_ ^ 1>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            };
            // ---------------- F-step: frame tF, own rows x all columns, from the whole vector
            if (iF == ph1 && !met) { meet(); after_meeting(); }
            C3_MARK(a, p, 0);
            const int S = ctl_s[0];
            float own;
            int ek;
            {
                const int tF = L - 1 - iF;
                const float4 bq4 = *(const float4*)&full_s[4 * lane];
                const float bq[4] = {bq4.x, bq4.y, bq4.z, bq4.w};
                float rs[5];
#pragma unroll
                for (int j = 0; j < 5; ++j) {
                    float t = EF[B_].e[j][0] * bq[0];
#pragma unroll
                    for (int c = 1; c < 4; ++c) t = fmaf(EF[B_].e[j][c], bq[c], t);
                    rs[j] = t;
                }
                // (five independent chains: their cross-lane steps overlap)
#pragma unroll
                for (int j = 0; j < 5; ++j) rs[j] = wave_sum_dpp(rs[j]);
                if (lane == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) { row_s[4 * wave + j] = rs[j]; rsh_s[4 * wave + j] = sF[B_]; }
                    if (g.xR) { row_s[16] = rs[4]; rsh_s[16] = sF[B_]; }
                }
                if (GAMMA && iF >= ph1) {
                    const int sak = __builtin_amdgcn_readlane(saF[B_], k);
                    const float frs = a.scale * c3_mscale(sak + S + sF[B_], D2, xwide);
                    const unsigned gso = (unsigned)tF * frb;
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        const float fr_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(aFo[B_]), j < 4 ? 4 * wave + j : 16)) * frs;
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = EF[B_].e[j][c] * bq[c] * fr_;
                        c3_put4<ACC>(x, grs, j < 4 ? g.voffR : g.voffRx, j < 4 ? gso + g.rowR0 + (unsigned)j * pitch : gso);
                    }
                    if (wave == 0) {
                        const float fb = a.scale * aFo[B_] * c3_mscale(sak + S + sFb[B_], D2, xwide);
                        c2_put<ACC>(full_s[g.oidx] * EF[B_].b * fb, grs, g.voffB, gso);
                    }
                }
                C3_MARK(a, p, 1);
                c2_barrier();
                C3_MARK(a, p, 2);
                // own states: every wave by itself (the same values from the same inputs, written to the same cells)
                const bool ok = g.olane;
                const float rv = ok ? row_s[min(lane, 31)] : 0.f;
                const int rsh = ok ? rsh_s[min(lane, 31)] : kShiftNone;
                const int m = max(rsh, sFb[B_]);
                const float v = fmaf(full_s[g.oidx], c2_scale(EF[B_].b, sFb[B_] - m), c2_scale(rv, rsh - m));
                const int te = v > 0.f ? m + float_exponent(v) : kShiftNone;
                const int ms = wave_max_dpp(te);
                own = v > 0.f ? c2_scale(v, m - ms) : 0.f;
                ek = ms == kShiftNone ? S : S + ms;
                if (lane < 32) own_s[lane] = own;
                if (wave == 0 && tF >= mid) {
                    if (g.olane) bh[(size_t)tF * C + g.ostate] = own;
                    if (lane == 0) Sb[(size_t)tF * kC3K + k] = ek;
                }
            }
            if (iP >= n) return false;
            C3_MARK(a, p, 3);
            // ---------------- P-step: frame tP, all rows x own columns, partial sums for every state
            if (iP == ph1 && !met) { meet(); after_meeting(); }
            {
                const int tP = L - 1 - iP;
                const unsigned tag = gstep + 1;
                const unsigned slot_off = (gstep & 1) * (unsigned)(kC3K * kC3XS * sizeof(u64));
                u64* xs = xbase + (size_t)(gstep & 1) * kC3K * kC3XS;
                const float4 ov4 = *(const float4*)&own_s[4 * g.ci];
                const float ov[4] = {ov4.x, ov4.y, ov4.z, ov4.w};
                float t[5];
#pragma unroll
                for (int j = 0; j < 5; ++j) {
                    float s = EP[B_].e[j][0] * ov[0];
#pragma unroll
                    for (int c = 1; c < 4; ++c) s = fmaf(EP[B_].e[j][c], ov[c], s);
                    t[j] = s;
                }
                // the four lanes of a row
#pragma unroll
                for (int j = 0; j < 5; ++j) {
                    t[j] += dpp_f<0xB1>(0.f, t[j]);
                    t[j] += dpp_f<0x4E>(0.f, t[j]);
                }
                if (g.ci == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) rowp_s[64 * wave + 16 * j + g.rg] = t[j];
                    if (g.xC) rowp_s[256] = t[4];
                }
                if (lane == 0) ctl_s[12 + wave] = sP[B_];
                if (wave == 0 && lane < 32) bl_s[lane] = own * EP[B_].b;
                C3_MARK(a, p, 4);
                c2_barrier();
                C3_MARK(a, p, 5);
                const int4 sp = *(const int4*)&ctl_s[12];
                const int spmax = max(max(max(sp.x, sp.y), max(sp.z, sp.w)), sPb[B_]);
                // thread <-> label state tid + 1, whose row this thread's own wave has summed
                float val = c2_scale(rowp_s[tid], sP[B_] - spmax);
                if ((tid >> 4) == k) val += c2_scale(bl_s[tid & 15], sPb[B_] - spmax);
                const int rel = (spmax == kShiftNone ? ek : ek + spmax) - S;
                const bool exch = !(GAMMA && iP == L - 1);
                if (exch) {
                    xpublish(xs + (size_t)k * kC3XS + tid, c2_pack(val, tag, rel));
                    if (tid == 0) {
                        float v0 = c2_scale(rowp_s[256], sp.x - spmax);
                        if (k == 0) v0 += c2_scale(bl_s[16], sPb[B_] - spmax);
                        xpublish(xs + (size_t)k * kC3XS + 256, c2_pack(v0, tag, rel));
                    }
                }
                if (GAMMA && iP >= ph1) {
                    // marginals: gamma[q][y] = a_t[q] M[q][y] b_{t+1}[y] / Z, b_{t+1} = the own states of the F-step
                    const unsigned gso = (unsigned)tP * frb;
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        const int saj = __builtin_amdgcn_readlane(saP[B_], j < 4 ? 4 * wave + j : 0);
                        const float fq = a.scale * aP[B_][j] * c3_mscale(saj + ek + sP[B_], D2, xwide);
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = fq * EP[B_].e[j][c] * ov[c];
                        c3_put4<ACC>(x, grs, j < 4 ? g.voffC : g.voffCx, j < 4 ? gso + g.rowC0 + (unsigned)(16 * j) * pitch : gso);
                    }
                    if (wave == 0) {
                        const float fb = a.scale * aPo[B_] * c3_mscale(__builtin_amdgcn_readlane(saP[B_], k) + ek + sPb[B_], D2, xwide);
                        c2_put<ACC>(own * EP[B_].b * fb, grs, g.voffB, gso);
                    }
                }
                C3_MARK(a, p, 6);
                C3Look lk;
                prep(std::integral_constant<int, B_ ^ 1>(), [&]() __attribute__((always_inline)) {
                    if (exch) c3_look(xrs, slot_off, voffq, voffz, lk);
                    issue(std::integral_constant<int, B_>(), p + 2);
                });
                C3_MARK(a, p, 7);
                if (exch) {
                    int relooks = 0;
                    c3_gather(xrs, slot_off, voffq, voffz, tag, full_s, ctl_s, a.spin_limit, dead, lk,
                              [&]() __attribute__((always_inline)) { C3_MARK(a, p, 8); }, &relooks);
                    C3_MARK(a, p, 9);
                    C3_NOTE(a, p, 10, relooks);
                    gstep += 1;
                    if (tP >= mid && wave == 1) {
                        if (g.olane) bh[(size_t)tP * C + g.ostate] = full_s[g.oidx];
                        if (lane == 0) Sb[(size_t)tP * kC3K + k] = ctl_s[0];
                    }
                }
            }
            ++p;
            return true;
        };
        for (;;) {
            if (!pair(std::integral_constant<int, 0>())) break;
            if (!pair(std::integral_constant<int, 1>())) break;
        }
        __syncthreads();
        if (!met) meet();
        if (xwide > kC2RangeBits) ctl_s[11] = 1;
        if (dead) ctl_s[8] = 1;
        __syncthreads();
        if (tid == 0) {
            if (ctl_s[11] && a.item_status && !bad) atomicMax(&a.item_status[b], (int)kItemRange);
            c3_finish_item(a, b, ctl_s[8] != 0, bad);
        }
        __syncthreads();
    }
}

// Two workgroups per compute unit: at most 256 registers per lane.
template <bool GAMMA, bool ACC = false>
__global__ __launch_bounds__(kC3Threads, 2) void cluster3_kernel(ClusterArgs a)
{
    __shared__ __align__(16) float smem[kC3Lds];
    ClusterGeom g;
    const int id = blockIdx.x;
    const int x = id & 7, slot = id >> 3;
    const int cl = slot / (2 * kC3K), member = slot - cl * 2 * kC3K;
    g.cg = x + 8 * cl;
    g.role = member / kC3K;
    g.k = member - g.role * kC3K;
    g.r0 = 0;
    g.nr = 0;
    unsigned gstep = 0, ptag = 0;
    if (GAMMA && !ACC) cluster_zero_padding(a, g);      // (adding leaves frames beyond the length alone)
    if (g.role == 0) alpha3_role<GAMMA, ACC>(a, g, smem, gstep, ptag);
    else beta3_role<GAMMA, ACC>(a, g, smem, gstep, ptag);
}

}  // namespace last
