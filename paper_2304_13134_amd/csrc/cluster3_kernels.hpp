// Third generation of the clustered forward-backward for the full 1-gram context dependency with
// exactly 256 labels (C = 257 states; arXiv 2304.13134, Eq. 2 / Eq. 1, Sections 4.1, 4.2.2).
//
// The recursion is the one of cluster2_kernels.hpp: an item is walked from both ends at once (K = 8 "alpha"
// workgroups upwards, K "beta" workgroups downwards, eight waves each, one workgroup per compute unit,
// meeting in the middle, marginals in the second half), frames are taken in pairs with ONE exchange per
// pair (F-step: whole vector -> own states, no communication; P-step: own states -> partial sums for all
// states, published and gathered), arithmetic is in the scaled linear domain E = 2^(w log2 e - s).  What
// changes is how the work is cut, with two things measured on this chip in mind: the address path of a
// compute unit takes a vector memory instruction lane by lane (about 0.4 clocks per lane plus 8 per
// instruction, whatever the width), so every access is 16 bytes per lane and no lane loads what another one
// has; and with two waves per SIMD the vector ALUs are the other bound, so nothing is computed twice.
//   * Ownership goes down to the wave: wave w of workgroup k ("sub-owner" u = 8 k + w) owns the four label
//     states 1 + 4 u .. 4 + 4 u; the start state 0, which receives no label arcs, is a fifth state of
//     sub-owner 0.  A wave needs the other waves of its workgroup only where sums over rows or columns
//     cross waves.  With 256 label states every access is regular: a row of a frame is its empty-label
//     weight followed by 256 label weights.
//       "row pattern" (alpha P-step, beta F-step): the wave's own four rows, one 16-byte load per lane and
//           row; sub-owner 0 reads the start state's row as a fifth one;
//       "column pattern" (alpha F-step, beta P-step): all 256 label rows x the workgroup's 32 columns,
//           eight rows per instruction (eight lanes x 16 bytes per row), 32 rows per wave;
//       "odd elements": one 4-byte load per wave and frame fetches the empty-label weights of the own
//           states (lanes 0..3, and lane 4 the start state's) and, in the column pattern, the start state's
//           label weights into the wave's own columns (lanes 8..11).
//     17 weights per lane and frame.
//   * One shift s per wave and frame (largest weight of the wave's share), carried along with the wave's
//     partial sums and applied where they meet: no maxima through LDS, no barrier in the exp pass.
//   * Stored state vectors are (value, exponent) pairs, [B][T+1][C][2]: whoever reads a state of the other
//     side gets its exponent with the same load (own states have one exponent per sub-owner).
//   * Exchange words as before, [value:32 | tag:16 | exponent:16], gathered two words per 16-byte load: the
//     four lanes of a quad share two neighbouring states and split the eight producers; their parts meet
//     through two DPP swaps.  The start state's eight words sit on eight lanes and are added up by a DPP
//     scan.  The order of every addition is fixed, so the gathered vector is bit-identical in all workgroups.
//   * Memory requests are spread over the pair instead of being issued in one burst (a wave whose request
//     finds the address path busy stands still): the F frame of the pair after the next is requested inside
//     the gather, the P frame of a later pair (the next with two register sets, the one after it with three)
//     at the top of the F-step, the other side's state vectors between the pieces of the exp pass; a wave's
//     loads return in order, so nothing slow may be in flight in front of a look at the exchange.  Marginals
//     leave as 16-byte stores, those of both frames of a pair right behind its publish.
//
// Per pair and workgroup (alpha; beta mirrors it): F-step sums -> barrier -> own states -> P-step sums ->
// barrier -> publish -> marginals of the pair (second half of the item) -> exp pass of the NEXT pair ->
// gather (two barriers).
#pragma once
#include "cluster2_kernels.hpp"

namespace last {

constexpr int kC3Waves = 8;
constexpr int kC3Threads = 64 * kC3Waves;
constexpr int kC3K = 8;         // workgroups per role and item
constexpr int kC3C = 257;       // states: the start state and 256 label states
constexpr int kC3XS = 272;      // exchange words per producer and slot (257 used; even: word pairs are 16-byte aligned)
constexpr int kC3RS = 12;       // LDS pitch of a column's eight partial sums (16-byte reads)
constexpr unsigned kC3Sc1 = 16; // cache policy of the exchange loads: agent scope, served by the XCD's L2
constexpr unsigned kC3SP = kC3C * 8u;   // bytes of a stored state vector: (value, exponent) pairs

// LDS map (floats / ints)
constexpr int kC3Full = 0;                      // [272] whole state vector: label state y at y - 1, the start state at 256
constexpr int kC3Red = kC3Full + 272;           // [32][12] alpha F-step: the waves' sums per own column; [272] beta P-step: row sums
constexpr int kC3Pacc = kC3Red + 32 * kC3RS;    // [8][256] alpha P-step: partial sums per wave and column
constexpr int kC3Bl = kC3Pacc + 8 * 256;        // [8][8] terms of the own states' empty-label arcs (per wave: 4 states, the start state)
constexpr int kC3OwnS = kC3Bl + 64;             // [36] beta: own states, [4 w + j], the start state at 32
constexpr int kC3Ctl = kC3OwnS + 40;            // [64] ints: [0] exponent of full_s, [1] timeout, [2] range, per wave: [8..15] F shift
                                                //            (alpha) / exponent of the own states (beta), [16..23] exponent of the
                                                //            P-step sums, [24..31] of the odd P-step terms (beta), [32..39] beta: the
                                                //            waves' parts of the start state's sum, [40..47] gather maxima
constexpr int kC3RedB = kC3Ctl + 64;            // [32] block reductions
constexpr int kC3Lds = kC3RedB + 32;
static_assert(kC3Red % 4 == 0 && kC3Pacc % 4 == 0 && kC3OwnS % 4 == 0 && kC3Ctl % 4 == 0, "16-byte LDS accesses");


// Weight loads use the default cache policy although every weight is read once per pass: with the
// non-temporal hint on all of them the kernel was measured 2.5 % slower (neighbouring workgroups share
// the cache lines at the ends of their row pieces), with the hint on the row-contiguous frames only it
// ran at the same speed; a plain read sweep is what gains from the hint.
constexpr int kC3WeightPolicy = 0;
__device__ __forceinline__ float4 c3_wload4(buf_t r, unsigned voff, unsigned soff)
{
    return __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, kC3WeightPolicy));
}
__device__ __forceinline__ float c3_wload(buf_t r, unsigned voff, unsigned soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, kC3WeightPolicy));
}
__device__ __forceinline__ uint4 c3_ld4(buf_t r, unsigned voff, unsigned soff)
{
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
    return __builtin_bit_cast(uint4, v);
}
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
__device__ __forceinline__ void c3_xstore(u64 w, buf_t r, unsigned voff, unsigned soff)
{
    typedef decltype(__builtin_amdgcn_raw_buffer_load_b64(r, 0, 0, 0)) b64_t;
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(b64_t, w), r, (int)voff, (int)soff, 0);
}
// (value, exponent) pair of a stored state vector
__device__ __forceinline__ void c3_load_pair(buf_t r, unsigned voff, unsigned soff, float& v, int& e)
{
    const uint2 x = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0));
    v = __uint_as_float(x.x);
    e = (int)x.y;
}
__device__ __forceinline__ void c3_store_pair(float v, int e, buf_t r, unsigned voff, unsigned soff)
{
    uint2 x;
    x.x = __float_as_uint(v);
    x.y = (unsigned)e;
    typedef decltype(__builtin_amdgcn_raw_buffer_load_b64(r, 0, 0, 0)) b64_t;
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(b64_t, x), r, (int)voff, (int)soff, 0);
}

// largest of three floats in one instruction (fmaxf alone costs a second instruction per operand that
// comes from memory: the compiler quiets signalling NaNs first)
__device__ __forceinline__ float c3_max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// largest int of a wave, wave-uniform
__device__ __forceinline__ int c3_wave_max(int v)
{
    return c2_wave_max_key(v);
}

// D split into an integer and a fraction, so that the scale of a marginal needs no double arithmetic
struct C3D {
    int i;
    float f;
};
__device__ __forceinline__ C3D c3_split(double D2)
{
    C3D d;
    if (D2 > -1.0e9 && D2 < 1.0e9) {
        const double fl = __builtin_floor(D2);
        d.i = (int)fl;
        d.f = (float)(D2 - fl);
    } else {               // (no path through the item: every marginal is a product with a zero)
        d.i = 0;
        d.f = 0.f;
    }
    return d;
}
// 2^(e - D) for a marginal, capped so that it stays finite; the largest exponent seen is kept for the
// range flag (see c2_marginal_scale)
__device__ __forceinline__ float c3_mscale(int e, const C3D& D, float& xmax)
{
    const float x = (float)(e - D.i) - D.f;
    xmax = fmaxf(xmax, x);
    return fast_exp2(fminf(x, 126.f));
}

// One exchange slot as a thread sees it: two neighbouring label states from two of the eight producers
// (the other lanes of its quad have the other six) and one of the eight words of the start state.
struct C3Look {
    uint4 q[2];
    uint2 z;
};

__device__ __forceinline__ void c3_look(buf_t xrs, unsigned slot_off, unsigned voffq, unsigned voffz, C3Look& lk)
{
    lk.q[0] = c3_xload4(xrs, voffq, slot_off);
    lk.q[1] = c3_xload4(xrs, voffq, slot_off + (unsigned)(kC3XS * 8));
    lk.z = c3_xload2(xrs, voffz, slot_off);           // (lanes 0..7 of wave 0; out of range elsewhere)
}

// sum over the wave's four rows of sixteen lanes, lane by lane (every lane gets the total of the four lanes
// that sit at its place in their rows)
__device__ __forceinline__ float c3_rows_sum(float x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// Gathering one exchange slot: the eight partial values of every state, added up in a fixed order
// relative to the largest producer exponent; the vector ends in full_s, renormalised by the largest
// magnitude present, its exponent in ctl_s[0].  Every thread calls; ends with a workgroup barrier.
// `after_poll` runs once all words are there, before they are added up.
template <typename AfterPoll>
__device__ __forceinline__ void c3_gather(buf_t xrs, unsigned slot_off, unsigned voffq, unsigned voffz, unsigned tag,
                                          float* full_s, int* ctl_s, int limit, int& dead, C3Look& lk,
                                          AfterPoll&& after_poll)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S0 = ctl_s[0];
    const unsigned tagw = (tag & 0xFFFFu) << 16;
    int n = 0;
    for (;;) {
        const unsigned zdiff = tid < 8 ? lk.z.y ^ tagw : 0u;
        const unsigned diff = zdiff | (lk.q[0].y ^ tagw) | (lk.q[0].w ^ tagw) | (lk.q[1].y ^ tagw) | (lk.q[1].w ^ tagw);
        if ((diff >> 16) == 0 || dead) break;
        if (++n > limit) { dead = 1; break; }
        __builtin_amdgcn_s_sleep(1);
        c3_look(xrs, slot_off, voffq, voffz, lk);
    }
    after_poll();
    const int e0 = (int)(short)(unsigned short)lk.q[0].y, e1 = (int)(short)(unsigned short)lk.q[1].y;
    int hm = max(e0, e1);
    // (16-bit exponents: differences in [-65535, 0])
    float vlo = __builtin_ldexpf(__uint_as_float(lk.q[0].x), e0 - hm) + __builtin_ldexpf(__uint_as_float(lk.q[1].x), e1 - hm);
    float vhi = __builtin_ldexpf(__uint_as_float(lk.q[0].z), e0 - hm) + __builtin_ldexpf(__uint_as_float(lk.q[1].z), e1 - hm);
    // the other six producers of the same two states: the other lanes of the quad, in two steps (float
    // addition commutes, so all four lanes end up with the same bits)
    {
        const int ho = dpp_i<0xB1>(hm, hm);
        const float olo = dpp_f<0xB1>(vlo, vlo), ohi = dpp_f<0xB1>(vhi, vhi);
        const int hr = max(hm, ho);
        vlo = __builtin_ldexpf(vlo, hm - hr) + __builtin_ldexpf(olo, ho - hr);
        vhi = __builtin_ldexpf(vhi, hm - hr) + __builtin_ldexpf(ohi, ho - hr);
        hm = hr;
    }
    {
        const int ho = dpp_i<0x4E>(hm, hm);
        const float olo = dpp_f<0x4E>(vlo, vlo), ohi = dpp_f<0x4E>(vhi, vhi);
        const int hr = max(hm, ho);
        vlo = __builtin_ldexpf(vlo, hm - hr) + __builtin_ldexpf(olo, ho - hr);
        vhi = __builtin_ldexpf(vhi, hm - hr) + __builtin_ldexpf(ohi, ho - hr);
        hm = hr;
    }
    const int href = hm;          // largest of the eight producers' exponents: the same in every lane
    // the start state (wave 0): lane l < 8 holds producer l's word; a scan leaves the sum in lane 7
    float vz = tid < 8 ? __builtin_ldexpf(__uint_as_float(lk.z.x), (int)(short)(unsigned short)lk.z.y - href) : 0.f;
    vz += dpp_f<0x111>(0.f, vz);
    vz += dpp_f<0x112>(0.f, vz);
    vz += dpp_f<0x114>(0.f, vz);
    const float v0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(vz), 7));
    // renormalise by the largest magnitude actually present (non-negative floats order like integers)
    int mub = c3_wave_max(max(__float_as_int(vlo), __float_as_int(vhi)));
    mub = max(mub, __float_as_int(v0));
    if (lane == 0) ctl_s[40 + wave] = mub;
    if (dead) ctl_s[1] = 1;
    c2_barrier();
    const int4 m0 = *(const int4*)&ctl_s[40], m1 = *(const int4*)&ctl_s[44];
    const int mxb = max(max(max(m0.x, m0.y), max(m0.z, m0.w)), max(max(m1.x, m1.y), max(m1.z, m1.w)));
    const int mx = mxb > 0 ? float_exponent(__int_as_float(mxb)) : 0;
    // lanes 0 and 1 of a quad write its two states
    if ((tid & 2) == 0) full_s[2 * (tid >> 2) + (tid & 1)] = __builtin_ldexpf((tid & 1) ? vhi : vlo, -mx);
    if (tid == 0) {
        full_s[256] = __builtin_ldexpf(v0, -mx);
        ctl_s[0] = S0 + href + mx;
    }
    c2_barrier();
}

// D = log2 sum_q a_mid[q] b_mid[q]; both vectors are stored as (value, exponent) pairs
__device__ __forceinline__ double c3_meeting(const uint2* ah, const uint2* bh, float* red)
{
    const int q = threadIdx.x;
    float pv = 0.f;
    int pe = 0;
    if (q < kC3C) {
        const uint2 x = ah[q], y = bh[q];
        pv = __uint_as_float(x.x) * __uint_as_float(y.x);
        pe = (int)x.y + (int)y.y;
    }
    const float xm = block_max(pv > 0.f ? (float)pe : -3.0e38f, red);
    if (!(xm > -1.0e38f)) return -(double)__builtin_huge_valf();
    const int xmax = (int)xm;
    const float tot = block_sum(pv > 0.f ? __builtin_ldexpf(pv, pe - xmax) : 0.f, red);
    return (double)xmax + (double)__log2f(tot);
}

// Geometry shared by both roles (see the patterns at the top of the file).
struct C3Geom {
    int lane, wave, k, u;
    int rg, ci;            // column pattern: row inside the instruction (0..7), quad of own columns (0..7)
    bool xR;               // sub-owner 0: the wave also owns the start state
    bool mvR, mvC;         // the lane has an odd element (row / column pattern)
    int midx;              // place in full_s of the state the lane's odd element starts from
    unsigned voffC, voffR; // lane offsets of the 16-byte accesses
    unsigned voffMr, voffMc;         // ... of the odd elements
    unsigned voffS;                  // ... of the own states in a stored state vector (lanes 0..3, 4)
    unsigned voffOc;                 // ... of the states the odd elements of the column pattern lead to
    unsigned rowC0, rowR0;           // scalar: first row of the wave in either pattern
};
__device__ __forceinline__ C3Geom c3_geom(int k)
{
    constexpr unsigned pitch = kC3C * 4u;
    C3Geom g;
    g.lane = threadIdx.x & 63;
    g.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    g.k = k;
    g.u = kC3Waves * k + g.wave;
    g.rg = g.lane >> 3;
    g.ci = g.lane & 7;
    g.xR = g.u == 0;
    const bool l4 = g.lane == 4 && g.xR, lo = g.lane < 4, l8 = g.lane >= 8 && g.lane < 12;
    g.mvR = lo || l4;
    g.mvC = lo || l4 || l8;
    g.midx = lo ? 4 * g.u + g.lane : 256;
    g.voffC = (unsigned)(1 + g.rg) * pitch + (unsigned)(1 + 32 * k + 4 * g.ci) * 4u;
    g.voffR = (unsigned)(1 + 4 * g.lane) * 4u;
    g.voffMr = lo ? (unsigned)(1 + 4 * g.u + g.lane) * pitch : (l4 ? 0u : kC2Off);
    g.voffMc = l8 ? (unsigned)(1 + 4 * g.u + g.lane - 8) * 4u : g.voffMr;
    g.voffS = lo ? (unsigned)(1 + 4 * g.u + g.lane) * 8u : (l4 ? 0u : kC2Off);
    g.voffOc = l8 ? (unsigned)(1 + 4 * g.u + g.lane - 8) * 8u : g.voffS;
    g.rowC0 = (unsigned)(32 * g.wave) * pitch;
    g.rowR0 = (unsigned)(1 + 4 * g.u) * pitch;
    return g;
}

// A frame's share of one lane: four slots of four neighbouring weights, the odd element, and (sub-owner 0,
// row pattern) the start state's row.
struct C3Frame {
    float e[4][4];
    float x[4];
    float m;
};
__device__ __forceinline__ void c3_set4(float (&d)[4], const float4& v)
{
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
}
// loads of one frame, slot by slot (so that the requests can be spread over other work); slot 4 = the odd element
// (and, row pattern, the start state's row: sub-owner 0 only)
__device__ __forceinline__ void c3_load_cols_slot(C3Frame& f, int j, buf_t wrs, const C3Geom& g, unsigned fo)
{
    constexpr unsigned pitch = kC3C * 4u;
    if (j < 4) c3_set4(f.e[j], c3_wload4(wrs, g.voffC, fo + g.rowC0 + (unsigned)(8 * j) * pitch));
    else f.m = c3_wload(wrs, g.voffMc, fo);
}
__device__ __forceinline__ void c3_load_rows_slot(C3Frame& f, int j, buf_t wrs, const C3Geom& g, unsigned fo)
{
    constexpr unsigned pitch = kC3C * 4u;
    if (j < 4) {
        c3_set4(f.e[j], c3_wload4(wrs, g.voffR, fo + g.rowR0 + (unsigned)j * pitch));
    } else {
        f.m = c3_wload(wrs, g.voffMr, fo);
        if (g.xR) c3_set4(f.x, c3_wload4(wrs, g.voffR, fo));
    }
}
__device__ __forceinline__ void c3_load_cols(C3Frame& f, buf_t wrs, const C3Geom& g, unsigned fo)
{
#pragma unroll
    for (int j = 0; j < 5; ++j) c3_load_cols_slot(f, j, wrs, g, fo);
#pragma unroll
    for (int c = 0; c < 4; ++c) f.x[c] = 0.f;         // (unused in this pattern)
}
__device__ __forceinline__ void c3_load_rows(C3Frame& f, buf_t wrs, const C3Geom& g, unsigned fo)
{
#pragma unroll
    for (int c = 0; c < 4; ++c) f.x[c] = 0.f;
#pragma unroll
    for (int j = 0; j < 5; ++j) c3_load_rows_slot(f, j, wrs, g, fo);
}
// exp pass of one frame: E = 2^(w log2 e - s), s = the wave's shift.  mvalid: the lane has an odd element;
// extra: the wave has the start state's row.
template <typename Between>
__device__ __forceinline__ int c3_exp_frame(C3Frame& f, bool mvalid, bool extra, Between&& between)
{
    float m = c3_max3(f.e[0][0], f.e[0][1], f.e[0][2]);
    m = c3_max3(m, f.e[0][3], f.e[1][0]);
    m = c3_max3(m, f.e[1][1], f.e[1][2]);
    m = c3_max3(m, f.e[1][3], f.e[2][0]);
    m = c3_max3(m, f.e[2][1], f.e[2][2]);
    m = c3_max3(m, f.e[2][3], f.e[3][0]);
    m = c3_max3(m, f.e[3][1], f.e[3][2]);
    m = c3_max3(m, f.e[3][3], mvalid ? f.m : LAST_NEG_INF);
    if (extra) {
        m = c3_max3(m, f.x[0], f.x[1]);
        m = c3_max3(m, f.x[2], f.x[3]);
    }
    // integer s >= m log2 e, within [kShiftNone, 30000]; -inf (no arc at all) gives kShiftNone
    const int sl = (int)__builtin_amdgcn_fmed3f(__builtin_ceilf(m * kLog2e), (float)kShiftNone, 30000.f);
    const int s = c3_wave_max(sl);
    const float nfs = -(float)s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f.e[j][c] = fast_exp2(fmaf(f.e[j][c], kLog2e, nfs));
            c2_pin(f.e[j][c]);
        }
        between(j);
    }
    if (extra) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f.x[c] = fast_exp2(fmaf(f.x[c], kLog2e, nfs));
            c2_pin(f.x[c]);
        }
    }
    f.m = mvalid ? fast_exp2(fmaf(f.m, kLog2e, nfs)) : 0.f;
    c2_pin(f.m);
    return s;
}

// Four marginals of one row slot: one 16-byte store (the address path takes a vector memory instruction
// lane by lane, whatever its width).  The store sits in an asm statement together with the wait states
// that must pass before its data registers are written again: with a scalar offset the compiler leaves
// none, and on this chip lanes of such a store were seen to pick up the new contents.  (Adding to the
// gradient tensor: load - add - store, eight bytes at a time.)
typedef float c3_v4f __attribute__((ext_vector_type(4)));
template <bool ACC>
__device__ __forceinline__ void c3_put4(const float (&x)[4], buf_t grs, unsigned voff, unsigned soff)
{
    if constexpr (ACC) {
        c2_put2<true>(x[0], x[1], grs, voff, soff, true, true);
        c2_put2<true>(x[2], x[3], grs, voff + 8u, soff, true, true);
    } else {
        c3_v4f d;
        d.x = x[0]; d.y = x[1]; d.z = x[2]; d.w = x[3];
        asm volatile("buffer_store_dwordx4 %0, %1, %2, %3 offen\n\ts_nop 2" :: "v"(d), "v"(voff), "s"(grs), "s"(soff));
    }
}

// ------------------------------------------------------------------ alpha role
template <bool GAMMA, bool ACC, int NS>
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
    // gather: quad <-> two neighbouring states, its lanes <-> two producers each
    const unsigned voffq = (unsigned)((2 * (tid & 3)) * kC3XS + 2 * (tid >> 2)) * 8u;
    const unsigned voffz = tid < 8 ? (unsigned)(tid * kC3XS + 256) * 8u : kC2Off;
    // publish: threads 0..255 <-> label states; the thread of an own state adds the state's empty-label term
    const unsigned voffpub = tid < 256 ? (unsigned)(k * kC3XS + tid) * 8u : kC2Off;
    const int pcol = tid & 255;
    const bool pubown = (pcol >> 5) == k;
    const int pubw = (pcol & 31) >> 2;               // the wave that owns the state
    const int pubbl = 8 * pubw + (pcol & 3);

    for (int b = cg.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : mid;
        const int nlast = max(n - 1, 0);
        const size_t fr = (size_t)C * C;
        float* ah = a.ahat + (size_t)b * (a.T + 1) * C * 2;
        const float* bh = a.bhat + (size_t)b * (a.T + 1) * C * 2;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        const buf_t srs = make_buf(ah, (unsigned)(a.T + 1) * kC3SP);        // own side's stored vectors
        const buf_t ors = make_buf(bh, (unsigned)(a.T + 1) * kC3SP);        // other side's
        const buf_t xrs = make_buf(a.xa + (size_t)cg.cg * 2 * kC3K * kC3XS, (unsigned)(2 * kC3K * kC3XS * sizeof(u64)));

        // a_0 = unit vector at the start state, exponent 0
        if (tid < 272) full_s[tid] = tid == 256 ? 1.f : 0.f;
        if (tid < 64) { ctl_s[tid] = 0; bl_s[tid] = 0.f; }
        c3_store_pair(lane == 4 ? 1.f : 0.f, 0, srs, g.voffS, 0u);
        __syncthreads();

        C3Frame EF[3], EP[3];
        int sF[3] = {0, 0, 0}, sP[3] = {0, 0, 0};
        // the other side's vectors for the marginals: values and exponents
        float bF4[3][4], bP4[3][4], bFm[3] = {0.f, 0.f, 0.f}, bPm[3] = {0.f, 0.f, 0.f};
        int eF4[3] = {0, 0, 0}, eP4[3] = {0, 0, 0}, eFm[3] = {0, 0, 0}, ePm[3] = {0, 0, 0};
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int c = 0; c < 4; ++c) { bF4[x][c] = 0.f; bP4[x][c] = 0.f; }
        C3D D{0, 0.f};
        float xwide = -3.0e38f;
        int dead = 0;
        bool met = false;

        // state vectors of the other side for the marginals of pair p (rows t + 1 of its two frames), in four
        // pieces; fetched once the two sides have met, and right after the meeting for the pairs in flight
        auto other_piece = [&](auto BUF, int p, int piece) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned tF1 = (unsigned)(min(2 * p, nlast) + 1) * kC3SP, tP1 = (unsigned)(min(2 * p + 1, nlast) + 1) * kC3SP;
            const unsigned vF = (unsigned)(1 + 32 * k + 4 * g.ci) * 8u, vP = (unsigned)(1 + 4 * lane) * 8u;
            if (piece == 0) {
                const uint4 x0 = c3_ld4(ors, vF, tF1), x1 = c3_ld4(ors, vF + 16u, tF1);
                bF4[B_][0] = __uint_as_float(x0.x); bF4[B_][1] = __uint_as_float(x0.z);
                bF4[B_][2] = __uint_as_float(x1.x); bF4[B_][3] = __uint_as_float(x1.z);
                eF4[B_] = (int)x0.y;                 // (the four states have one sub-owner: one exponent)
            } else if (piece == 1) {
                c3_load_pair(ors, g.voffOc, tF1, bFm[B_], eFm[B_]);
            } else if (piece == 2) {
                const uint4 y0 = c3_ld4(ors, vP, tP1), y1 = c3_ld4(ors, vP + 16u, tP1);
                bP4[B_][0] = __uint_as_float(y0.x); bP4[B_][1] = __uint_as_float(y0.z);
                bP4[B_][2] = __uint_as_float(y1.x); bP4[B_][3] = __uint_as_float(y1.z);
                eP4[B_] = (int)y0.y;
            } else {
                c3_load_pair(ors, g.voffS, tP1, bPm[B_], ePm[B_]);
            }
        };
        auto other = [&](auto BUF, int p) __attribute__((always_inline)) {
#pragma unroll
            for (int piece = 0; piece < 4; ++piece) other_piece(BUF, p, piece);
        };
        auto settle = [&]() __attribute__((always_inline)) {
            int t = 0;
#pragma unroll
            for (int x = 0; x < 3; ++x) {
#pragma unroll
                for (int c = 0; c < 4; ++c) t |= c2_touch(bF4[x][c]) | c2_touch(bP4[x][c]);
                t |= c2_touch(bFm[x]) | c2_touch(bPm[x]) | (eF4[x] == 0x7fffffff) | (eP4[x] == 0x7fffffff)
                     | (eFm[x] == 0x7fffffff) | (ePm[x] == 0x7fffffff);
            }
            if (t) ctl_s[3] = 1;          // (never; nobody reads it)
        };
        auto issue = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_load_cols(EF[B_], wrs, g, (unsigned)min(2 * p, nlast) * frb);
            c3_load_rows(EP[B_], wrs, g, (unsigned)min(2 * p + 1, nlast) * frb);
        };
        // exp pass of a pair's two frames; the callbacks place memory requests between its pieces
        auto prep = [&](auto BUF, auto&& duringF, auto&& middle, auto&& duringP) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            sF[B_] = c3_exp_frame(EF[B_], g.mvC, false, duringF);
            middle();
            sP[B_] = c3_exp_frame(EP[B_], g.mvR, g.xR, duringP);
            if (GAMMA) {
#pragma unroll
                for (int c = 0; c < 4; ++c) { c2_pin(bF4[B_][c]); c2_pin(bP4[B_][c]); }
                c2_pin(bFm[B_]); c2_pin(bPm[B_]); c2_pin(eF4[B_]); c2_pin(eP4[B_]); c2_pin(eFm[B_]); c2_pin(ePm[B_]);
            }
        };
        auto meet = [&]() __attribute__((always_inline)) {
            if (dead) ctl_s[1] = 1;
            cluster_sync(a, cg, ptag, &ctl_s[1]);
            ptag += 1;
            const double D2 = c3_meeting((const uint2*)ah + (size_t)mid * C, (const uint2*)bh + (size_t)mid * C, redb);
            D = c3_split(D2);
            if (k == 0 && tid == 0) {
                a.dist[b] = bad ? __builtin_nanf("") : (float)(D2 * 0.6931471805599453);
                if (a.item_status) a.item_status[b] = bad ? kItemBadLength : kItemOk;
            }
            met = true;
            __syncthreads();
        };

        issue(std::integral_constant<int, 0>(), 0);
        if (NS == 3) issue(std::integral_constant<int, 1>(), 1);
        else c3_load_cols(EF[1], wrs, g, (unsigned)min(2, nlast) * frb);  // (its P frame: requested in pair 0)
        prep(std::integral_constant<int, 0>(), [](int) {}, [] {}, [](int) {});

        int p = 0;
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value, B1_ = (B_ + 1) % NS, B2_ = (B_ + 2) % NS;   // this pair, the next, the one after
            constexpr int BQ_ = NS == 3 ? B2_ : B1_, dq = NS == 3 ? 2 : 1;                       // the pair whose P frame is requested
            const int tF = 2 * p, tP = 2 * p + 1;
            if (tF >= n) return false;
            auto after_meeting = [&]() __attribute__((always_inline)) {
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B1_>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            };
            // ---------------- F-step: frame tF, all rows x own columns, from the whole vector
            if (tF == mid && !met) { meet(); after_meeting(); }
            const int S = ctl_s[0];
            float own;        // lanes 0..3: the wave's own states, lane 4: the start state (sub-owner 0); zero elsewhere
            int ek;           // their exponent
            // the P frame of a later pair is requested first of all (into registers no pair in flight uses): a
            // wave's loads return in order, and what is still in flight when the look at the exchange is issued
            // holds up its answer
            {
                const unsigned foP2 = (unsigned)min(2 * (p + dq) + 1, nlast) * frb;
#pragma unroll
                for (int j = 0; j < 5; ++j) c3_load_rows_slot(EP[BQ_], j, wrs, g, foP2);
            }
            float aq[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) aq[j] = full_s[32 * wave + 8 * j + g.rg];
            const float am = full_s[g.midx];
            // marginals of the F frame (second half of the item); they leave after the publish of the pair, or
            // at its end if the P frame is beyond the item
            auto marginalsF = [&]() __attribute__((always_inline)) {
                if (GAMMA && tF >= mid) {
                    const unsigned gso = (unsigned)tF * frb;
                    const float fcs = a.scale * c3_mscale(S + sF[B_] + eF4[B_], D, xwide);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = aq[j] * EF[B_].e[j][c] * (bF4[B_][c] * fcs);
                        c3_put4<ACC>(x, grs, g.voffC, gso + g.rowC0 + (unsigned)(8 * j) * pitch);
                    }
                    const float fm = a.scale * bFm[B_] * c3_mscale(S + sF[B_] + eFm[B_], D, xwide);
                    c2_put<ACC>(am * EF[B_].m * fm, grs, g.voffMc, gso);
                }
            };
            {
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = fmaf(aq[j], EF[B_].e[j][c], acc[c]);
                // the eight rows of an instruction: the two of a group of sixteen lanes, then the wave's four groups
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    acc[c] += dpp_f<0x118>(0.f, acc[c]);
                    acc[c] = c3_rows_sum(acc[c]);
                }
                if (lane >= 8 && lane < 16) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) red_s[(4 * g.ci + c) * kC3RS + wave] = acc[c];
                }
                if (lane == 0) ctl_s[8 + wave] = sF[B_];
                // odd elements: the empty-label arc of an own state (lanes 0..4) and the start state's label arc
                // into it (lanes 8..11, moved to lanes 0..3)
                float mt = am * EF[B_].m;
                mt += dpp_f<0x108>(0.f, mt);
                c2_barrier();
                // own states: lane j < 4 adds up the eight waves' sums of column 4 wave + j
                const int4 sh0 = *(const int4*)&ctl_s[8], sh1 = *(const int4*)&ctl_s[12];
                const int smax = max(max(max(sh0.x, sh0.y), max(sh0.z, sh0.w)), max(max(sh1.x, sh1.y), max(sh1.z, sh1.w)));
                const float4* rp = (const float4*)&red_s[(4 * wave + (lane & 3)) * kC3RS];
                const float4 p0 = rp[0], p1 = rp[1];
                float v = ((__builtin_ldexpf(p0.x, sh0.x - smax) + __builtin_ldexpf(p0.y, sh0.y - smax))
                           + (__builtin_ldexpf(p0.z, sh0.z - smax) + __builtin_ldexpf(p0.w, sh0.w - smax)))
                          + ((__builtin_ldexpf(p1.x, sh1.x - smax) + __builtin_ldexpf(p1.y, sh1.y - smax))
                             + (__builtin_ldexpf(p1.z, sh1.z - smax) + __builtin_ldexpf(p1.w, sh1.w - smax)));
                v = lane < 4 ? v : 0.f;
                v += __builtin_ldexpf(mt, sF[B_] - smax);
                v = g.mvR ? v : 0.f;
                const int ms = c3_wave_max(v > 0.f ? float_exponent(v) : kShiftNone);
                own = __builtin_ldexpf(v, -ms);
                ek = ms == kShiftNone ? S : S + smax + ms;
                if (tF + 1 <= mid) c3_store_pair(own, ek, srs, g.voffS, (unsigned)(tF + 1) * kC3SP);
            }
            if (tP >= n) { marginalsF(); return false; }
            // ---------------- P-step: frame tP, own rows x all columns, partial sums for every state
            if (tP == mid && !met) { meet(); after_meeting(); }
            {
                const unsigned tag = gstep + 1;
                const unsigned slot_off = (gstep & 1) * (unsigned)(kC3K * kC3XS * sizeof(u64));
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(own), j));
                const float o0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(own), 4));
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = fmaf(o[j], EP[B_].e[j][c], acc[c]);
                if (g.xR) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = fmaf(o0, EP[B_].x[c], acc[c]);
                }
                float4 av;
                av.x = acc[0]; av.y = acc[1]; av.z = acc[2]; av.w = acc[3];
                *(float4*)&pacc_s[wave * 256 + 4 * lane] = av;
                const int tw = ek + sP[B_];                 // exponent of this wave's sums
                if (lane == 0) ctl_s[16 + wave] = tw;
                if (lane < 8) bl_s[8 * wave + lane] = own * EP[B_].m;      // empty-label arcs of the own states
                c2_barrier();
                const bool exch = !(GAMMA && tP == L - 1);
                if (exch && tid < 256) {
                    const int4 tw0 = *(const int4*)&ctl_s[16], tw1 = *(const int4*)&ctl_s[20];
                    const int tmax = max(max(max(tw0.x, tw0.y), max(tw0.z, tw0.w)), max(max(tw1.x, tw1.y), max(tw1.z, tw1.w)));
                    float val = ((__builtin_ldexpf(pacc_s[tid], tw0.x - tmax) + __builtin_ldexpf(pacc_s[256 + tid], tw0.y - tmax))
                                 + (__builtin_ldexpf(pacc_s[512 + tid], tw0.z - tmax) + __builtin_ldexpf(pacc_s[768 + tid], tw0.w - tmax)))
                                + ((__builtin_ldexpf(pacc_s[1024 + tid], tw1.x - tmax) + __builtin_ldexpf(pacc_s[1280 + tid], tw1.y - tmax))
                                   + (__builtin_ldexpf(pacc_s[1536 + tid], tw1.z - tmax) + __builtin_ldexpf(pacc_s[1792 + tid], tw1.w - tmax)));
                    if (pubown) val += __builtin_ldexpf(bl_s[pubbl], ctl_s[16 + pubw] - tmax);
                    const int rel = tmax - S;
                    c3_xstore(c2_pack(val, tag, rel), xrs, voffpub, slot_off);
                    // the start state moves on by its empty-label arc only: workgroup 0 has it, the others add zero
                    if (tid == 0)
                        c3_xstore(c2_pack(k == 0 ? __builtin_ldexpf(bl_s[4], tw0.x - tmax) : 0.f, tag, rel), xrs,
                                  (unsigned)(k * kC3XS + 256) * 8u, slot_off);
                }
                C3Look lk;
                auto marginalsP = [&]() __attribute__((always_inline)) {
                  if (GAMMA && tP >= mid) {
                    const unsigned gso = (unsigned)tP * frb;
                    const float fys = a.scale * c3_mscale(tw + eP4[B_], D, xwide);
                    float fy[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) fy[c] = bP4[B_][c] * fys;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = o[j] * EP[B_].e[j][c] * fy[c];
                        c3_put4<ACC>(x, grs, g.voffR, gso + g.rowR0 + (unsigned)j * pitch);
                    }
                    if (g.xR) {
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = o0 * EP[B_].x[c] * fy[c];
                        c3_put4<ACC>(x, grs, g.voffR, gso);
                    }
                    const float fm = a.scale * bPm[B_] * c3_mscale(tw + ePm[B_], D, xwide);
                    c2_put<ACC>(own * EP[B_].m * fm, grs, g.voffMr, gso);
                  }
                };
                // (the stores of both frames right behind the publish: the stretch from the gather to the publish,
                // on which every other workgroup of the group waits, then has no store of this one in its way)
                marginalsF();
                marginalsP();
                // exp pass of the next pair, with the requests for the pair after the next (into the registers
                // this pair has finished with) between its pieces; the look at the exchange comes before the
                // frames' requests, because a wave's loads return in order
                const unsigned foF2 = (unsigned)min(2 * p + 4, nlast) * frb;
                prep(std::integral_constant<int, B1_>(),
                     [&](int j) __attribute__((always_inline)) {
                         if (GAMMA && met) other_piece(std::integral_constant<int, B2_>(), p + 2, j);
                     },
                     [&]() __attribute__((always_inline)) {
                         if (exch) c3_look(xrs, slot_off, voffq, voffz, lk);
                     },
                     [](int) {});
                if (!exch) {
#pragma unroll
                    for (int j = 0; j < 5; ++j) c3_load_cols_slot(EF[B2_], j, wrs, g, foF2);
                }
                if (exch) {
                    c3_gather(xrs, slot_off, voffq, voffz, tag, full_s, ctl_s, a.spin_limit, dead, lk,
                              [&]() __attribute__((always_inline)) {
#pragma unroll
                                  for (int j = 0; j < 5; ++j) c3_load_cols_slot(EF[B2_], j, wrs, g, foF2);
                              });
                    gstep += 1;
                    if (tP + 1 <= mid) c3_store_pair(full_s[g.midx], ctl_s[0], srs, g.voffS, (unsigned)(tP + 1) * kC3SP);
                }
            }
            ++p;
            return true;
        };
        for (;;) {
            if (!pair(std::integral_constant<int, 0>())) break;
            if (!pair(std::integral_constant<int, 1>())) break;
            if constexpr (NS == 3) {
                if (!pair(std::integral_constant<int, 2>())) break;
            }
        }
        __syncthreads();
        if (!met) meet();
        if (xwide > kC2RangeBits) ctl_s[2] = 1;
        if (dead) ctl_s[1] = 1;
        __syncthreads();
        if (tid == 0) {
            if (ctl_s[2] && a.item_status && !bad) atomicMax(&a.item_status[b], (int)kItemRange);
            cluster_finish_item(a, b, ctl_s[1] != 0, bad, 2 * kC3K);
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------- beta role
template <bool GAMMA, bool ACC, int NS>
__device__ __forceinline__ void beta3_role(const ClusterArgs& a, const ClusterGeom& cg, float* smem,
                                           unsigned& gstep, unsigned& ptag)
{
    constexpr int C = kC3C;
    constexpr unsigned pitch = C * 4u, frb = (unsigned)C * C * 4u;
    float* full_s = smem + kC3Full;
    float* rowp_s = smem + kC3Red;            // [272] P-step: row sums (label state y at y - 1)
    float* bl_s = smem + kC3Bl;
    float* own_s = smem + kC3OwnS;
    int* ctl_s = (int*)(smem + kC3Ctl);
    float* z_s = smem + kC3Ctl + 32;          // [8] the waves' parts of the start state's sum
    float* redb = smem + kC3RedB;
    const int tid = threadIdx.x;
    const C3Geom g = c3_geom(cg.k);
    const int lane = g.lane, wave = g.wave, k = g.k;
    const unsigned voffq = (unsigned)((2 * (tid & 3)) * kC3XS + 2 * (tid >> 2)) * 8u;
    const unsigned voffz = tid < 8 ? (unsigned)(tid * kC3XS + 256) * 8u : kC2Off;
    const unsigned voffpub = tid < 256 ? (unsigned)(k * kC3XS + tid) * 8u : kC2Off;
    const int pcol = tid & 255;
    const bool pubown = (pcol >> 5) == k;
    const int pubw = (pcol & 31) >> 2;
    const int pubbl = 8 * pubw + (pcol & 3);
    const int prow = pcol >> 5;               // the wave that has summed the row of label state pcol + 1
    // odd elements of the column pattern lead to the own states (lanes 0..3, 8..11) or the start state (lane 4)
    const int oidx = (lane & 7) < 4 ? 4 * wave + (lane & 3) : 32;

    for (int b = cg.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : L - mid;
        const int ph1 = L - mid;                      // step at which the state index reaches mid
        const int nlast = max(n - 1, 0);
        const size_t fr = (size_t)C * C;
        const float* ah = a.ahat + (size_t)b * (a.T + 1) * C * 2;
        float* bh = a.bhat + (size_t)b * (a.T + 1) * C * 2;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        const buf_t srs = make_buf(bh, (unsigned)(a.T + 1) * kC3SP);
        const buf_t ors = make_buf(ah, (unsigned)(a.T + 1) * kC3SP);
        const buf_t xrs = make_buf(a.xb + (size_t)cg.cg * 2 * kC3K * kC3XS, (unsigned)(2 * kC3K * kC3XS * sizeof(u64)));

        // b_L = 1 for every state, exponent 0
        if (tid < 272) full_s[tid] = tid < C ? 1.f : 0.f;
        if (tid < 64) { ctl_s[tid] = 0; bl_s[tid] = 0.f; }
        if (tid < 40) own_s[tid] = 0.f;
        c3_store_pair(1.f, 0, srs, g.voffS, (unsigned)L * kC3SP);
        __syncthreads();

        C3Frame EF[3], EP[3];
        int sF[3] = {0, 0, 0}, sP[3] = {0, 0, 0};
        // the other side's vectors for the marginals: values and exponents
        float aFm[3] = {0.f, 0.f, 0.f}, aPm[3] = {0.f, 0.f, 0.f}, aP[3][4];
        int eFm[3] = {0, 0, 0}, ePm[3] = {0, 0, 0}, eP[3][4];
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int j = 0; j < 4; ++j) { aP[x][j] = 0.f; eP[x][j] = 0; }
        C3D D{0, 0.f};
        float xwide = -3.0e38f;
        int dead = 0;
        bool met = false;

        // step index i -> frame L - 1 - i; pair p = steps 2p (F) and 2p + 1 (P)
        auto frameF = [&](int p) { return max(L - 1 - min(2 * p, nlast), 0); };
        auto frameP = [&](int p) { return max(L - 1 - min(2 * p + 1, nlast), 0); };
        auto other_piece = [&](auto BUF, int p, int piece) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned tF = (unsigned)frameF(p) * kC3SP, tP = (unsigned)frameP(p) * kC3SP;
            const unsigned vr = (unsigned)(1 + g.rg) * 8u, r0 = tP + (unsigned)(32 * wave) * 8u;
            if (piece == 0) {
                c3_load_pair(ors, g.voffS, tF, aFm[B_], eFm[B_]);
                // odd elements of the P frame: the own states' empty-label arcs (lanes 0..3, the start state's on
                // lane 4) and the start state's label arcs (lanes 8..11) leave from these states
                c3_load_pair(ors, lane >= 8 && lane < 12 ? 0u : g.voffS, tP, aPm[B_], ePm[B_]);
            } else if (piece == 1) {
                c3_load_pair(ors, vr, r0, aP[B_][0], eP[B_][0]);
                c3_load_pair(ors, vr, r0 + 64u, aP[B_][1], eP[B_][1]);
            } else if (piece == 2) {
                c3_load_pair(ors, vr, r0 + 128u, aP[B_][2], eP[B_][2]);
                c3_load_pair(ors, vr, r0 + 192u, aP[B_][3], eP[B_][3]);
            }
        };
        auto other = [&](auto BUF, int p) __attribute__((always_inline)) {
#pragma unroll
            for (int piece = 0; piece < 3; ++piece) other_piece(BUF, p, piece);
        };
        auto settle = [&]() __attribute__((always_inline)) {
            int t = 0;
#pragma unroll
            for (int x = 0; x < 3; ++x) {
#pragma unroll
                for (int j = 0; j < 4; ++j) t |= c2_touch(aP[x][j]) | (eP[x][j] == 0x7fffffff);
                t |= c2_touch(aFm[x]) | c2_touch(aPm[x]) | (eFm[x] == 0x7fffffff) | (ePm[x] == 0x7fffffff);
            }
            if (t) ctl_s[3] = 1;          // (never; nobody reads it)
        };
        auto issue = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_load_rows(EF[B_], wrs, g, (unsigned)frameF(p) * frb);
            c3_load_cols(EP[B_], wrs, g, (unsigned)frameP(p) * frb);
        };
        auto prep = [&](auto BUF, auto&& duringF, auto&& middle, auto&& duringP) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            sF[B_] = c3_exp_frame(EF[B_], g.mvR, g.xR, duringF);
            middle();
            sP[B_] = c3_exp_frame(EP[B_], g.mvC, false, duringP);
            if (GAMMA) {
#pragma unroll
                for (int j = 0; j < 4; ++j) { c2_pin(aP[B_][j]); c2_pin(eP[B_][j]); }
                c2_pin(aFm[B_]); c2_pin(aPm[B_]); c2_pin(eFm[B_]); c2_pin(ePm[B_]);
            }
        };
        auto meet = [&]() __attribute__((always_inline)) {
            if (dead) ctl_s[1] = 1;
            cluster_sync(a, cg, ptag, &ctl_s[1]);
            ptag += 1;
            D = c3_split(c3_meeting((const uint2*)ah + (size_t)mid * C, (const uint2*)bh + (size_t)mid * C, redb));
            met = true;
            __syncthreads();
        };

        issue(std::integral_constant<int, 0>(), 0);
        if (NS == 3) issue(std::integral_constant<int, 1>(), 1);
        else c3_load_rows(EF[1], wrs, g, (unsigned)frameF(1) * frb);      // (its P frame: requested in pair 0)
        prep(std::integral_constant<int, 0>(), [](int) {}, [] {}, [](int) {});

        int p = 0;
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value, B1_ = (B_ + 1) % NS, B2_ = (B_ + 2) % NS;   // this pair, the next, the one after
            constexpr int BQ_ = NS == 3 ? B2_ : B1_, dq = NS == 3 ? 2 : 1;                       // the pair whose P frame is requested
            const int iF = 2 * p, iP = 2 * p + 1;
            if (iF >= n) return false;
            auto after_meeting = [&]() __attribute__((always_inline)) {
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B1_>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            };
            // ---------------- F-step: frame tF, own rows x all columns, from the whole vector
            if (iF == ph1 && !met) { meet(); after_meeting(); }
            const int S = ctl_s[0];
            float own;        // lanes 0..3: the wave's own states, lane 4: the start state (sub-owner 0); zero elsewhere
            int ek;           // their exponent
            const int tF = L - 1 - iF;
            {                 // (the P frame of a later pair: see the alpha role)
                const unsigned foP2 = (unsigned)frameP(p + dq) * frb;
#pragma unroll
                for (int j = 0; j < 5; ++j) c3_load_cols_slot(EP[BQ_], j, wrs, g, foP2);
            }
            const float4 bq4 = *(const float4*)&full_s[4 * lane];
            const float bq[4] = {bq4.x, bq4.y, bq4.z, bq4.w};
            const float bm = full_s[g.midx];
            // marginals of the F frame (second half of the item); they leave after the publish of the pair, or
            // at its end if the P frame is beyond the item
            auto marginalsF = [&]() __attribute__((always_inline)) {
                if (GAMMA && iF >= ph1) {
                    const unsigned gso = (unsigned)tF * frb;
                    const float frs = a.scale * c3_mscale(__builtin_amdgcn_readlane(eFm[B_], 0) + S + sF[B_], D, xwide);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float fr_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(aFm[B_]), j)) * frs;
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = EF[B_].e[j][c] * bq[c] * fr_;
                        c3_put4<ACC>(x, grs, g.voffR, gso + g.rowR0 + (unsigned)j * pitch);
                    }
                    if (g.xR) {
                        const float fr_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(aFm[B_]), 4)) * frs;
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = EF[B_].x[c] * bq[c] * fr_;
                        c3_put4<ACC>(x, grs, g.voffR, gso);
                    }
                    const float fm = a.scale * aFm[B_] * c3_mscale(eFm[B_] + S + sF[B_], D, xwide);
                    c2_put<ACC>(bm * EF[B_].m * fm, grs, g.voffMr, gso);
                }
            };
            {
                float rs[5];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float t = EF[B_].e[j][0] * bq[0];
#pragma unroll
                    for (int c = 1; c < 4; ++c) t = fmaf(EF[B_].e[j][c], bq[c], t);
                    rs[j] = t;
                }
                rs[4] = 0.f;
                if (g.xR) {
                    float t = EF[B_].x[0] * bq[0];
#pragma unroll
                    for (int c = 1; c < 4; ++c) t = fmaf(EF[B_].x[c], bq[c], t);
                    rs[4] = t;
                }
                // (independent chains: their cross-lane steps overlap)
#pragma unroll
                for (int j = 0; j < 4; ++j) rs[j] = wave_sum_dpp(rs[j]);
                if (g.xR) rs[4] = wave_sum_dpp(rs[4]);
                // own states: row sum plus the empty-label arc, lane j <-> own state j (lane 4: the start state)
                float v = lane == 0 ? rs[0] : lane == 1 ? rs[1] : lane == 2 ? rs[2] : lane == 3 ? rs[3] : rs[4];
                v = fmaf(bm, EF[B_].m, v);
                v = g.mvR ? v : 0.f;
                const int ms = c3_wave_max(v > 0.f ? float_exponent(v) : kShiftNone);
                own = __builtin_ldexpf(v, -ms);
                ek = ms == kShiftNone ? S : S + sF[B_] + ms;
                if (lane < 4) own_s[4 * wave + lane] = own;
                if (lane == 4 && g.xR) own_s[32] = own;
                if (lane == 0) ctl_s[8 + wave] = ek;
                if (tF >= mid) c3_store_pair(own, ek, srs, g.voffS, (unsigned)tF * kC3SP);
                c2_barrier();
            }
            if (iP >= n) { marginalsF(); return false; }
            // ---------------- P-step: frame tP, all rows x own columns, partial sums for every state
            if (iP == ph1 && !met) { meet(); after_meeting(); }
            {
                const int tP = L - 1 - iP;
                const unsigned tag = gstep + 1;
                const unsigned slot_off = (gstep & 1) * (unsigned)(kC3K * kC3XS * sizeof(u64));
                // the lane's four columns are the own states of wave ci: bring them to the largest of the waves' exponents
                const int4 ek0 = *(const int4*)&ctl_s[8], ek1 = *(const int4*)&ctl_s[12];
                const int ekmax = max(max(max(ek0.x, ek0.y), max(ek0.z, ek0.w)), max(max(ek1.x, ek1.y), max(ek1.z, ek1.w)));
                const int ekc = ctl_s[8 + g.ci];
                const float4 ov4 = *(const float4*)&own_s[4 * g.ci];
                float ov[4] = {ov4.x, ov4.y, ov4.z, ov4.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) ov[c] = __builtin_ldexpf(ov[c], ekc - ekmax);
                float t[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float s = EP[B_].e[j][0] * ov[0];
#pragma unroll
                    for (int c = 1; c < 4; ++c) s = fmaf(EP[B_].e[j][c], ov[c], s);
                    t[j] = s;
                }
                // the eight lanes of a row: the four of a quad, then the row's two quads (the total ends in the
                // upper quad's lanes)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    t[j] += dpp_f<0xB1>(0.f, t[j]);
                    t[j] += dpp_f<0x4E>(0.f, t[j]);
                    t[j] += dpp_f<0x114>(0.f, t[j]);
                }
                if (g.ci == 4) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) rowp_s[32 * wave + 8 * j + g.rg] = t[j];
                }
                // odd elements: the own states' empty-label arcs (lanes 0..4) and the start state's label arcs into the
                // own states (lanes 8..11, added up over the four); their exponent is the wave's own
                const float mo = own_s[oidx] * EP[B_].m;
                float zt = mo;
                zt += dpp_f<0xB1>(0.f, zt);
                zt += dpp_f<0x4E>(0.f, zt);
                const int tw = ekmax + sP[B_], tb = ek + sP[B_];
                if (lane < 8) bl_s[8 * wave + lane] = mo;
                if (lane == 8) z_s[wave] = zt;
                if (lane == 0) { ctl_s[16 + wave] = tw; ctl_s[24 + wave] = tb; }
                c2_barrier();
                const bool exch = !(GAMMA && iP == L - 1);
                if (exch && tid < 256) {
                    const int4 tw0 = *(const int4*)&ctl_s[16], tw1 = *(const int4*)&ctl_s[20];
                    const int4 tb0 = *(const int4*)&ctl_s[24], tb1 = *(const int4*)&ctl_s[28];
                    const int tmax = max(max(max(max(tw0.x, tw0.y), max(tw0.z, tw0.w)), max(max(tw1.x, tw1.y), max(tw1.z, tw1.w))),
                                         max(max(max(tb0.x, tb0.y), max(tb0.z, tb0.w)), max(max(tb1.x, tb1.y), max(tb1.z, tb1.w))));
                    // thread <-> label state tid + 1
                    float val = __builtin_ldexpf(rowp_s[tid], ctl_s[16 + prow] - tmax);
                    if (pubown) val += __builtin_ldexpf(bl_s[pubbl], ctl_s[24 + pubw] - tmax);
                    const int rel = tmax - S;
                    c3_xstore(c2_pack(val, tag, rel), xrs, voffpub, slot_off);
                    if (tid == 0) {
                        float v0 = ((__builtin_ldexpf(z_s[0], tb0.x - tmax) + __builtin_ldexpf(z_s[1], tb0.y - tmax))
                                    + (__builtin_ldexpf(z_s[2], tb0.z - tmax) + __builtin_ldexpf(z_s[3], tb0.w - tmax)))
                                   + ((__builtin_ldexpf(z_s[4], tb1.x - tmax) + __builtin_ldexpf(z_s[5], tb1.y - tmax))
                                      + (__builtin_ldexpf(z_s[6], tb1.z - tmax) + __builtin_ldexpf(z_s[7], tb1.w - tmax)));
                        if (k == 0) v0 += __builtin_ldexpf(bl_s[4], tb0.x - tmax);
                        c3_xstore(c2_pack(v0, tag, rel), xrs, (unsigned)(k * kC3XS + 256) * 8u, slot_off);
                    }
                }
                C3Look lk;
                auto marginalsP = [&]() __attribute__((always_inline)) {
                  if (GAMMA && iP >= ph1) {
                    // marginals: gamma[q][y] = a_t[q] M[q][y] b_{t+1}[y] / Z, b_{t+1} = the own states of the F-step
                    const unsigned gso = (unsigned)tP * frb;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float fq = a.scale * aP[B_][j] * c3_mscale(eP[B_][j] + tw, D, xwide);
                        float x[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) x[c] = fq * EP[B_].e[j][c] * ov[c];
                        c3_put4<ACC>(x, grs, g.voffC, gso + g.rowC0 + (unsigned)(8 * j) * pitch);
                    }
                    const float fm = a.scale * aPm[B_] * c3_mscale(ePm[B_] + tb, D, xwide);
                    c2_put<ACC>(mo * fm, grs, g.voffMc, gso);
                  }
                };
                // (the stores of both frames right behind the publish: the stretch from the gather to the publish,
                // on which every other workgroup of the group waits, then has no store of this one in its way)
                marginalsF();
                marginalsP();
                const unsigned foF2 = (unsigned)frameF(p + 2) * frb;
                prep(std::integral_constant<int, B1_>(),
                     [&](int j) __attribute__((always_inline)) {
                         if (GAMMA && met) other_piece(std::integral_constant<int, B2_>(), p + 2, j);
                     },
                     [&]() __attribute__((always_inline)) {
                         if (exch) c3_look(xrs, slot_off, voffq, voffz, lk);
                     },
                     [](int) {});
                if (!exch) {
#pragma unroll
                    for (int j = 0; j < 5; ++j) c3_load_rows_slot(EF[B2_], j, wrs, g, foF2);
                }
                if (exch) {
                    c3_gather(xrs, slot_off, voffq, voffz, tag, full_s, ctl_s, a.spin_limit, dead, lk,
                              [&]() __attribute__((always_inline)) {
#pragma unroll
                                  for (int j = 0; j < 5; ++j) c3_load_rows_slot(EF[B2_], j, wrs, g, foF2);
                              });
                    gstep += 1;
                    if (tP >= mid) c3_store_pair(full_s[g.midx], ctl_s[0], srs, g.voffS, (unsigned)tP * kC3SP);
                }
            }
            ++p;
            return true;
        };
        for (;;) {
            if (!pair(std::integral_constant<int, 0>())) break;
            if (!pair(std::integral_constant<int, 1>())) break;
            if constexpr (NS == 3) {
                if (!pair(std::integral_constant<int, 2>())) break;
            }
        }
        __syncthreads();
        if (!met) meet();
        if (xwide > kC2RangeBits) ctl_s[2] = 1;
        if (dead) ctl_s[1] = 1;
        __syncthreads();
        if (tid == 0) {
            if (ctl_s[2] && a.item_status && !bad) atomicMax(&a.item_status[b], (int)kItemRange);
            cluster_finish_item(a, b, ctl_s[1] != 0, bad, 2 * kC3K);
        }
        __syncthreads();
    }
}

// One workgroup per compute unit, two waves per SIMD: at most 256 registers per lane.
// NS: register sets of frames.  2: the P frame of a pair is requested during the pair before it (under 200
// registers: waves of another kernel fit beside this one); 3: two pairs ahead, like the F frames, so that
// its exp pass never waits for memory while the marginal stores of the second half crowd it (about 240).
template <bool GAMMA, bool ACC = false, int NS = 2>
__global__ __launch_bounds__(kC3Threads) void cluster3_kernel(ClusterArgs a)
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
    if (g.role == 0) alpha3_role<GAMMA, ACC, NS>(a, g, smem, gstep, ptag);
    else beta3_role<GAMMA, ACC, NS>(a, g, smem, gstep, ptag);
}

}  // namespace last
