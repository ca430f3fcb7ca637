// Second generation of the clustered forward-backward for the full 1-gram
// context dependency (arXiv 2304.13134, Eq. 2 / Eq. 1, Sections 4.1, 4.2.2):
// ONE exchange per TWO frames.
//
// Same decomposition as cluster_kernels.hpp (an item = 2K persistent workgroups
// on one XCD, K walking frames upwards, K downwards, meeting in the middle;
// workgroup k owns states [k*RPW, (k+1)*RPW)), but the two frames between
// exchanges are processed with two different ownerships of the weight matrix
// M_t[q][y] = exp(w_t[q][y]):
//   F-step ("from the full vector"): every workgroup knows the whole state vector
//       and produces its OWN states of the next one without communication;
//       alpha: a'[y] = sum_q a[q] M[q][y] for its own columns y (reads all rows x own columns),
//       beta : b'[q] = sum_y M[q][y] b[y] for its own rows q (reads own rows x all columns);
//   P-step ("partials"): from its own states only, every workgroup produces a
//       partial result for ALL states,
//       alpha: p_k[y] = sum_{q own} a[q] M[q][y]   (own rows x all columns),
//       beta : p_k[q] = sum_{y own} M[q][y] b[y]   (all rows x own columns),
//       publishes the C partial values, and every workgroup reads all K x C of
//       them and adds them up in the same order: the whole next vector, bit for
//       bit the same everywhere.
// Either way each element of the frame is read by exactly one workgroup, so the
// traffic is unchanged (12 B/arc with the marginals), the number of latency-bound
// exchanges is halved, and because the summed vector is complete and identical in
// every workgroup its binary exponent is taken from the data itself (no predicted
// exponent steps).  Own parts carry a per-workgroup exponent, so stored state
// vectors have one exponent per block of RPW states (Sa, Sb: [B][T+1][8]).
//
// The empty label (column 0) keeps the state: w[q][0] is an arc q -> q.  In the
// steps that read "own columns" the workgroup reads column 0 for its own rows
// separately.
//
// Arithmetic as in cluster_kernels.hpp: E = 2^(w log2 e - s) with integer shifts s from the data (per
// own column, or per row), evaluated for the NEXT pair while the exchange of the current one is in
// flight.  Exchange words are [value:32 | tag:16 | exponent:16], published with plain stores into the
// XCD's L2 and gathered with agent-scope loads (K per thread, the first look issued halfway through the
// exp pass); all waits are bounded (status 5 instead of a hang).
//
// Access patterns.  "Own rows x all columns" (alpha P-step, beta F-step) is read row-contiguous.  "All
// rows x own columns" is read three rows per instruction, 17 lanes x 8 bytes per row (alpha F-step), or
// seven rows per instruction, 9 lanes x 16 bytes per row (beta P-step).  Masks are not branches: a lane that must not store gets a buffer offset beyond the
// descriptor (dropped by the hardware's range check), and loads beyond the matrix fetch a copy of the
// last row or column, which meets a zero of the state vector in every sum.
#pragma once
#include "cluster_kernels.hpp"

namespace last {

constexpr int kC2Threads = 512;   // 8 waves = 2 per SIMD: 256 registers per lane
constexpr int kC2Waves = 8;
constexpr int kC2NQ = 33;      // rows per wave when a workgroup reads all rows: 8 * 33 >= 264
constexpr int kC2FG = 3;       // alpha F-step: row groups per wave (17 lanes each, two columns per lane)
constexpr int kC2FJ = 11;      // alpha F-step: rows per lane, kC2FG * kC2FJ = kC2NQ
constexpr int kC2Hdr = 264;    // largest number of states on this path (words of value per producer and slot)
constexpr int kC2XS = 272;     // words per producer and slot
constexpr int kC2RW = 5;       // rows per wave when a workgroup reads its own rows wave by wave: 8 * 5 >= 33
constexpr int kC2NC = 4;       // ... a lane takes four neighbouring columns; columns beyond 256 by one more instruction (see beta F-step)
constexpr int kC2PH = 17;      // alpha P-step: a thread takes one half of the (at most 33) own rows: [0, 17) or [17, 33)
constexpr int kC2PC = 256;     // columns that have a thread per half (alpha P-step) or a lane per four (beta F-step);
                               // the few beyond ("stragglers", at most 8) are taken lane-wise by single instructions
constexpr int kC2Own = 40;     // LDS slots for own states
constexpr int kC2QL = 9;       // beta P-step: lanes per row, four neighbouring own columns each (16-byte loads)
constexpr int kC2QG = 7;       // ... rows per instruction (63 lanes)
constexpr int kC2QJ = 5;       // ... instructions per lane: row slots kC2QG * j + group, 35 >= kC2NQ
// A per-lane buffer offset beyond every descriptor's size: the hardware's range check drops the lane's
// store and returns zero for its load.  Replaces branches around accesses whose mask differs per lane.
constexpr unsigned kC2Off = 0xFFFFFF00u;

// LDS map (floats / ints)
constexpr int kC2Full = 0;                          // [320] whole state vector
constexpr int kC2OwnS = kC2Full + 320;              // [40]  own states
constexpr int kC2RedN = kC2Waves * kC2FG;           // partial sums per own column (alpha F-step)
constexpr int kC2Red = kC2OwnS + kC2Own;            // [24][40] partials per wave and row group
constexpr int kC2Shc = kC2Red + kC2RedN * kC2Own;   // [2][40] shift per own column, per buffer (int, atomic maxima)
constexpr int kC2Bl = kC2Shc + 2 * kC2Own;          // [40] empty-label terms
constexpr int kC2Pacc = kC2Bl + kC2Own;             // [320] partial sums of the second half
constexpr int kC2Bo = kC2Pacc + 320;                // [40] other side's own-state values (marginals)
constexpr int kC2Ctl = kC2Bo + kC2Own;              // [32] ints
constexpr int kC2RedB = kC2Ctl + 32;                // [32] block reductions
constexpr int kC2Strag = kC2RedB + 32;              // [8] partial sums of the straggler columns
constexpr int kC2RowF = kC2Strag + 8;               // [40] beta F-step: row sums
constexpr int kC2RowS = kC2RowF + kC2Own;           // [40] beta F-step: row shifts (int)
constexpr int kC2Bt = kC2RowS + kC2Own;             // [40] beta P-step: own states times their columns' shifts
constexpr int kC2Afull = kC2Bt + kC2Own;            // [320] beta P-step: other side's vector (marginals)
constexpr int kC2R2S = 12;                          // row pitch of the per-lane partials (9 used, the rest stays zero)
constexpr int kC2Red2 = kC2Afull + 320;             // [264][12] beta P-step: partial sums per row and lane
constexpr int kC2Lds = kC2Red2 + kC2Waves * kC2NQ * kC2R2S;
static_assert(kC2Red2 % 4 == 0 && kC2R2S % 4 == 0, "16-byte reads of the per-row partials");
static_assert(kC2Red % 2 == 0 && kC2Shc % 2 == 0 && kC2Bt % 2 == 0 && kC2Own % 2 == 0, "8-byte LDS accesses");


__device__ __forceinline__ void c2_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Keeps a value computed in the shadow of the exchange where it was computed: without it the compiler
// merges the evaluation at the end of one pair with the one before the loop and moves both behind the
// exchange, onto the critical path.
template <typename T>
__device__ __forceinline__ void c2_pin(T& v)
{
    asm volatile("" : "+v"(v));
}

// The compiler follows loads without regard to the conditions they sit under: a load under a
// condition whose uses sit under the same condition still counts as possibly pending at every later
// use, and costs a wait that also covers whatever was issued in between.  Loads of this kernel are
// therefore issued on every path (a lane or wave that needs nothing gets the out-of-range offset), and
// where a path does not use a loaded value it "touches" it: a comparison that is never true, whose
// result ends in a flag nobody reads.
__device__ __forceinline__ int c2_touch(float v)
{
    return v > 3.3e38f ? 1 : 0;
}

// Wait for every vector memory load in flight (vmcnt(0); the other counters untouched).  Used on the
// rare path that reloads prefetched values: the compiler merges the pending state of that path into
// the common one, and would otherwise make the common path wait for loads it has only just issued.
__device__ __forceinline__ void c2_wait_loads()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

__device__ __forceinline__ float c2_scale(float v, int e)     // v * 2^e (zero stays zero whatever e is)
{
    return __builtin_ldexpf(v, max(e, -300));
}

// 2^(e - D) for the marginals.  e adds up the exponents of three maxima (state vector, weights, state
// vector) that need not be reached by the same arc.  The three factors it scales are held relative to
// those maxima in float32, so whatever lies more than 2^126 below its maximum has already become zero:
// harmless in every sum, but an arc can make up for a small state value by a large weight, and its marginal
// is then lost.  With e - D <= kC2RangeBits such a lost marginal is below 2^(kC2RangeBits - 126); beyond,
// the item is flagged (status kItemRange) and the factor is capped so that it stays finite (an infinite
// factor next to an underflowed product would give NaN).
constexpr float kC2RangeBits = 80.f;
__device__ __forceinline__ float c2_marginal_scale(int e, double D2, int* ctl_s)
{
    const float x = (float)((double)e - D2);
    if (x > kC2RangeBits) ctl_s[11] = 1;
    return fast_exp2(fminf(x, 126.f));
}
// (the same with the largest exponent kept in a register of the caller, looked at when the item ends:
// cheaper where the caller has the register to spare)
__device__ __forceinline__ float c2_marginal_scale(int e, double D2, float& xmax)
{
    const float x = (float)((double)e - D2);
    xmax = fmaxf(xmax, x);
    return fast_exp2(fminf(x, 126.f));
}

// Largest float of a wave for several independent values at once: floats are mapped to integers of the
// same order, and the steps take the smallest integer where a lane has no source, which lets the
// compiler fold each step into one v_max_i32 with a DPP operand.  (One chain alone is not faster this
// way, its steps wait on each other; several interleaved chains are.)
__device__ __forceinline__ int c2_fkey(float x)
{
    const int b = __float_as_int(x);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float c2_fkey_inv(int k)
{
    return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}
__device__ __forceinline__ int c2_wave_max_key(int v)
{
    constexpr int kMin = -2147483647 - 1;
    v = max(v, dpp_i<0x111>(kMin, v));
    v = max(v, dpp_i<0x112>(kMin, v));
    v = max(v, dpp_i<0x114>(kMin, v));
    v = max(v, dpp_i<0x118>(kMin, v));
    v = max(v, dpp_i<0x142, 0xa>(kMin, v));
    v = max(v, dpp_i<0x143, 0xc>(kMin, v));
    return __builtin_amdgcn_readlane(v, 63);
}

// Exchange word of this kernel: [value:32 | tag:16 | exponent:16].  The exponent is the producer's,
// relative to the exponent of the vector both sides already share (the one the pair started from), so
// that it fits 16 bits whatever the length of the sequence; it is the same in all words of a producer.
// A slot is rewritten every second exchange, so 16 bits of the step number identify a word.
__device__ __forceinline__ u64 c2_pack(float v, unsigned tag, int rel)
{
    return (u64)__float_as_uint(v) | ((u64)((tag & 0xFFFFu) << 16 | ((unsigned)rel & 0xFFFFu)) << 32);
}

// Gathering one exchange slot: all K x C partial values, added up in producer order relative to the
// largest exponent; the vector ends in full_s, its exponent in ctl_s[0].
// The first look is issued before the exp pass of the next pair (c2_gather_look) and examined after
// it (c2_gather): by then the words have usually arrived and the round trip to the L2 cache is hidden.
struct C2Look {
    u64 wv[kClMaxK];
};

// (Threads beyond the last state read the last state's words and discard the result: loads and their
// uses sit on every path, see c2_touch.)
// FULL: K is the largest number of producers (the common case at 257 states): no test per word.
template <bool FULL>
__device__ __forceinline__ void c2_gather_look(const u64* xs, int K, int C, C2Look& lk)
{
    const int q = min((int)threadIdx.x, C - 1);
#pragma unroll
    for (int kk = 0; kk < kClMaxK; ++kk)
        if (FULL || kk < K) lk.wv[kk] = xload(xs + (size_t)kk * kC2XS + q);
}

// Every thread calls; ends with a workgroup barrier.  `after_poll` runs once all words are there, before
// they are added up: the place for memory requests that should not stand between the polls and their data.
template <bool FULL, typename AfterPoll>
__device__ __forceinline__ void c2_gather(const u64* xs, int K, int C, unsigned tag, float* full_s,
                                            int* ctl_s, int limit, int& dead, C2Look& lk, AfterPoll&& after_poll)
{
    const int tid = threadIdx.x;
    const int S0 = ctl_s[0];           // exponent the producers' exponents are relative to
    float v = 0.f;
    int hr = 0;
    {
        int n = 0;
        for (;;) {
            // all K tags right: no bit differs in the upper halves of the words' high parts
            const unsigned tagw = (tag & 0xFFFFu) << 16;
            unsigned diff = 0;
#pragma unroll
            for (int kk = 0; kk < kClMaxK; ++kk)
                if (FULL || kk < K) diff |= (unsigned)(lk.wv[kk] >> 32) ^ tagw;
            const bool ok = (diff >> 16) == 0;
            if (ok || dead) break;
            if (++n > limit) { dead = 1; break; }
            __builtin_amdgcn_s_sleep(1);
            c2_gather_look<FULL>(xs, K, C, lk);
        }
        after_poll();
        int href = -(1 << 30);
#pragma unroll
        for (int kk = 0; kk < kClMaxK; ++kk)
            if (FULL || kk < K) href = max(href, (int)(short)(unsigned short)(lk.wv[kk] >> 32));
#pragma unroll
        for (int kk = 0; kk < kClMaxK; ++kk)
            if (FULL || kk < K)
                v += __builtin_ldexpf(__uint_as_float((unsigned)lk.wv[kk]),
                                      (int)(short)(unsigned short)(lk.wv[kk] >> 32) - href);      // (16-bit exponents: in [-65535, 0])
        hr = href;
        if (tid >= C) v = 0.f;
    }
    // renormalise by the largest magnitude actually present, so that mantissas do not drift.  The values
    // are sums of products of non-negative numbers: their bit patterns order like integers, and the
    // exponent is taken once, from the largest.
    const int mub = wave_max_dpp(__float_as_int(v));
    if ((tid & 63) == 0) ctl_s[24 + (tid >> 6)] = mub;
    if (dead) ctl_s[8] = 1;
    c2_barrier();
    const int4 m0 = *(const int4*)&ctl_s[24], m1 = *(const int4*)&ctl_s[28];
    const int mxb = max(max(max(m0.x, m0.y), max(m0.z, m0.w)), max(max(m1.x, m1.y), max(m1.z, m1.w)));
    const int mx = mxb > 0 ? float_exponent(__int_as_float(mxb)) : 0;
    if (tid < C) full_s[tid] = c2_scale(v, -mx);
    if (tid == 0) ctl_s[0] = S0 + hr + mx;
    c2_barrier();
}
// D = log2 sum_q a_mid[q] b_mid[q] with one exponent per block of RPW states on either side
__device__ __forceinline__ double c2_meeting(const float* ah, const float* bh, const int* Sa, const int* Sb,
                                             int C, int RPW, int K, float* red)
{
    int xmax = -(1 << 30);
    for (int k = 0; k < K; ++k) xmax = max(xmax, Sa[k] + Sb[k]);
    float part = 0.f;
    for (int q = threadIdx.x; q < C; q += blockDim.x) {
        const int k = q / RPW;
        part += c2_scale(ah[q] * bh[q], Sa[k] + Sb[k] - xmax);
    }
    const float tot = block_sum(part, red);
    return (double)xmax + (double)__log2f(tot);
}

// 8-byte buffer accesses (two neighbouring floats, 4-byte aligned)
__device__ __forceinline__ float2 buf_load2(buf_t r, unsigned voff, unsigned soff)
{
    const auto v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0);
    static_assert(sizeof(v) == sizeof(float2), "8-byte buffer load");
    return __builtin_bit_cast(float2, v);
}
__device__ __forceinline__ void buf_store2(float x, float y, buf_t r, unsigned voff, unsigned soff)
{
    typedef decltype(__builtin_amdgcn_raw_buffer_load_b64(r, 0, 0, 0)) b64_t;
    float2 f;
    f.x = x; f.y = y;
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(b64_t, f), r, (int)voff, (int)soff, 0);
}

// 16-byte buffer accesses (four neighbouring floats, 4-byte aligned)
__device__ __forceinline__ float4 buf_load4(buf_t r, unsigned voff, unsigned soff)
{
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
    static_assert(sizeof(v) == sizeof(float4), "16-byte buffer load");
    return __builtin_bit_cast(float4, v);
}
// Writing marginals: overwrite, or (ACC) add to what the gradient tensor holds.  A lane with the out-of-range
// offset reads zero and its store is dropped.  Overwriting, the columns that two lanes have in common (see
// c2_pair, c2_quad) are simply written twice with the same value; adding, each element is added by the one
// lane that counts it (ok0, ok1), four bytes at a time.
template <bool ACC>
__device__ __forceinline__ void c2_put(float x, buf_t r, unsigned voff, unsigned soff)
{
    if constexpr (ACC) x += buf_load(r, voff, soff);
    buf_store(x, r, voff, soff);
}
template <bool ACC>
__device__ __forceinline__ void c2_put2(float x, float y, buf_t r, unsigned voff, unsigned soff, bool ok0, bool ok1)
{
    if constexpr (ACC) {
        c2_put<true>(x, r, ok0 ? voff : kC2Off, soff);
        c2_put<true>(y, r, ok1 ? voff + 4u : kC2Off, soff);
    } else {
        buf_store2(x, y, r, voff, soff);
    }
}

// 16-byte stores.  With a scalar offset the compiler leaves no wait state between such a store and the next
// instruction that overwrites its data registers, and on this chip lanes of the store were then seen to
// pick up the new contents: the store sits in an asm statement together with its wait states.  It pays:
// the address path takes a vector memory instruction lane by lane, whatever its width, so four floats per
// lane cost what two do.  (Adding to the gradient tensor stays at load - add - store of eight bytes.)
typedef float c2_v4f __attribute__((ext_vector_type(4)));
template <bool ACC>
__device__ __forceinline__ void c2_put4(float x0, float x1, float x2, float x3, buf_t r, unsigned voff, unsigned soff,
                                        bool ok0, bool ok1, bool ok2, bool ok3)
{
    if constexpr (ACC) {
        c2_put2<true>(x0, x1, r, voff, soff, ok0, ok1);
        c2_put2<true>(x2, x3, r, voff + 8u, soff, ok2, ok3);
    } else {
        c2_v4f d;
        d.x = x0; d.y = x1; d.z = x2; d.w = x3;
        asm volatile("buffer_store_dwordx4 %0, %1, %2, %3 offen\n\ts_nop 2" :: "v"(d), "v"(voff), "s"(r), "s"(soff));
    }
}

// Lane -> pair of neighbouring own columns for the "all rows x own columns" frames.  Every lane with
// columns stores 8 bytes per row: the pairs start behind the column that takes no label arcs (column 0 of
// the first workgroup), and an odd number of columns ends in a pair that overlaps its predecessor by one
// column (dup0: stored twice with the same value, counted once).  Only a workgroup with a single label
// column has a lane with one column (single).
struct C2Pair {
    int c0;            // first own column of the lane (second: c0 + 1)
    bool act, dup0, single;
};
__device__ __forceinline__ C2Pair c2_pair(int ci, bool in_group, int r0, int nr)
{
    C2Pair p;
    const int cbase = r0 == 0 ? 1 : 0;
    const int ncols = max(nr - cbase, 0);
    const int np = (ncols + 1) / 2;
    p.act = in_group && ci < np;
    p.c0 = cbase + 2 * min(ci, max(np - 1, 0));
    p.dup0 = false;
    p.single = false;
    if (p.c0 + 1 >= nr) {
        if (ncols >= 2) { p.c0 = nr - 2; p.dup0 = true; }
        else p.single = true;
    }
    return p;
}

// Lane -> four neighbouring own columns (beta P-step).  The quads start behind the column that takes no
// label arcs; the last quad is moved back so that it ends with the last own column, and the ndup columns
// it then has in common with its predecessor are stored twice with the same value and counted once.
// (The workgroup has at least four such columns.)
struct C2Quad {
    int c0;            // first own column of the lane
    int ndup;          // leading columns that belong to the lane before
    bool act;
};
__device__ __forceinline__ C2Quad c2_quad(int ci, bool in_group, int r0, int nr)
{
    C2Quad q;
    const int cbase = r0 == 0 ? 1 : 0;
    const int ncols = max(nr - cbase, 4);
    const int nq = (ncols + 3) / 4;
    q.act = in_group && ci < nq;
    const int want = cbase + 4 * min(ci, nq - 1);
    q.c0 = max(min(want, nr - 4), 0);
    q.ndup = want - q.c0;
    return q;
}

// ------------------------------------------------------------------ alpha role
template <bool GAMMA, bool ACC, bool FULL>
__device__ __forceinline__ void alpha2_role(const ClusterArgs& a, const ClusterGeom& g, float* smem,
                                            unsigned& gstep, unsigned& ptag)
{
    float* full_s = smem + kC2Full;
    float* own_s = smem + kC2OwnS;
    float* red_s = smem + kC2Red;
    int* shc_s = (int*)(smem + kC2Shc);
    float* bl_s = smem + kC2Bl;
    float* pacc_s = smem + kC2Pacc;
    float* bo_s = smem + kC2Bo;
    int* ctl_s = (int*)(smem + kC2Ctl);       // [0] exponent of full_s, [1] exponent of own_s, [8] timeout
    float* redb = smem + kC2RedB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int C = a.C, K = a.K, RPW = a.RPW;
    // P-step: thread <-> column cP = 64 (wave & 3) + lane and half hP = wave >> 2 of the own rows;
    // straggler column 256 + sS on wave 7 - sS, lane <-> own row
    float* strag_s = smem + kC2Strag;
    const int hP = wave >> 2;
    const int cP = ((wave & 3) << 6) + lane;
    const bool colok = cP < C;
    const int rP0 = kC2PH * hP;
    const int nst = max(C - kC2PC, 0);
    const int sS = kC2Waves - 1 - wave;
    const bool hasS = sS < nst;
    const int cS = kC2PC + sS;
    // F-step: wave <-> rows [33 wave, 33 wave + 33); inside the wave three groups of 17 lanes take every
    // third row, and a lane takes two neighbouring own columns (8-byte accesses): row 33 wave + 3 j + gq,
    // columns r0 + 2 ci, r0 + 2 ci + 1.  Lanes 51..63 idle.  The sums over rows end in wave 0, lane <-> own column.
    const int gq = lane / 17, ci = lane - 17 * gq;
    const C2Pair pr = c2_pair(ci, lane < 17 * kC2FG, g.r0, g.nr);    // (state 0 receives no label arcs)
    const bool lact = pr.act;
    const int c0 = pr.c0;
    const bool v0ok = lact && !pr.dup0;                 // columns this lane adds up: the overlap only once
    const bool v1ok = lact && !pr.single;
    const bool need1 = g.nr - (g.r0 == 0 ? 1 : 0) == 1;  // (whole workgroup) one label column: 4-byte stores
    const int qF0 = kC2NQ * wave + gq;                  // first row of this lane
    const int jlim = lact ? (C - qF0 + kC2FG - 1) / kC2FG : 0;   // rows j < jlim exist
    const int slotF = (wave * kC2FG + min(gq, kC2FG - 1)) * kC2Own + c0;
    const bool fok = lane < g.nr;                       // wave 0: lane <-> own column
    const int yF = min(g.r0 + lane, C - 1);

    for (int b = g.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : mid;
        const size_t fr = (size_t)C * C;
        const unsigned frb = (unsigned)(fr * sizeof(float));
        const unsigned pitch = (unsigned)(C * (int)sizeof(float));
        float* ah = a.ahat + (size_t)b * (a.T + 1) * C;
        const float* bh = a.bhat + (size_t)b * (a.T + 1) * C;
        int* Sa = a.Sa + (size_t)b * (a.T + 1) * kClMaxK;
        const int* Sb = a.Sb + (size_t)b * (a.T + 1) * kClMaxK;
        u64* xbase = a.xa + (size_t)g.cg * 2 * kClMaxK * kC2XS;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? a.dw + (size_t)b * a.T * fr : a.w, GAMMA ? (unsigned)a.T * frb : 0u);
        const buf_t brs = make_buf(bh, (unsigned)(a.T + 1) * pitch);
        const buf_t sbrs = make_buf(Sb, (unsigned)(a.T + 1) * (unsigned)(kClMaxK * sizeof(int)));
        const unsigned yoff = (unsigned)(yF * (int)sizeof(float));
        const unsigned koff = (unsigned)((lane & 7) * (int)sizeof(int));
        const unsigned coffP = (unsigned)(min(cP, C - 1) * (int)sizeof(float));
        const unsigned coffPm = colok ? (unsigned)(cP * (int)sizeof(float)) : kC2Off;     // nothing beyond the row
        const unsigned coffS = lane < g.nr ? (unsigned)lane * pitch + (unsigned)(cS * (int)sizeof(float)) : kC2Off;
        const unsigned soffS = (unsigned)(min(kC2PC + (lane & 7), C - 1) * (int)sizeof(float));
        const unsigned rbaseP = (unsigned)g.r0 * pitch;
        const unsigned colF = (unsigned)((g.r0 + c0) * (int)sizeof(float));
        const unsigned coffF = (unsigned)gq * pitch + colF;
        const unsigned rowF0 = (unsigned)(kC2NQ * wave) * pitch;     // scalar: first row of this wave
        const unsigned rowB = (unsigned)yF * pitch;                  // row of the own state (empty-label weight)
        const int nlast = max(n - 1, 0);

        // Offset of this lane's element pair in row j of its rows.  A row beyond the matrix is replaced by
        // the last row: what is loaded there is finite, takes part in no maximum that matters and meets a
        // zero of the state vector in every sum, so the exp pass needs no mask per element.  A lane without
        // columns of its own repeats the address of a lane that has some (no traffic of its own); its
        // elements are zeroed by its shift.  (jl: the number of rows, through a register the compiler cannot
        // see through, so that the offsets are made where they are used instead of being kept.)
        const int gqa = min(gq, kC2FG - 1);
        const unsigned cola = colF;          // (c2_pair gives a lane without columns the last pair's)
        const unsigned offA0 = (unsigned)(kC2NQ * wave + gqa) * pitch + cola;
        const unsigned offAL = (unsigned)(C - 1) * pitch + cola;
        const int jla = max((C - (kC2NQ * wave + gqa) + kC2FG - 1) / kC2FG, 0);
        auto rowcol = [&](int j, int jl) __attribute__((always_inline)) {
            return j < jl ? offA0 + (unsigned)(kC2FG * j) * pitch : offAL;
        };
        // a_0 = unit vector at the start state, exponent 0
        for (int q = tid; q < 320; q += kC2Threads) full_s[q] = q == 0 ? 1.f : 0.f;
        if (tid < kC2Own) { own_s[tid] = 0.f; bl_s[tid] = 0.f; bo_s[tid] = 0.f; }
        if (tid < 32) ctl_s[tid] = (tid == 2 || tid == 3) ? kShiftNone : 0;
        if (tid < 2 * kC2Own) shc_s[tid] = kShiftNone;
        for (int q = tid; q < kC2RedN * kC2Own; q += kC2Threads) red_s[q] = 0.f;
        if (tid < g.nr) ah[g.r0 + tid] = (g.r0 + tid == 0) ? 1.f : 0.f;
        if (tid == 0) Sa[g.k] = 0;
        __syncthreads();

        float EF0[2][kC2FJ], EF1[2][kC2FJ], EP[2][kC2PH];
        float EB[2] = {0.f, 0.f}, ES[2] = {0.f, 0.f}, bSt[2] = {0.f, 0.f};
        float EBP[2] = {0.f, 0.f};                  // wave 0: empty-label weight of the own row of this lane, P frame
        int shP[2] = {0, 0}, sigP[2] = {0, 0}, ssP[2] = {kShiftNone, kShiftNone}, sbP0[2] = {kShiftNone, kShiftNone};
        // other side's vector for the marginals
        float bF0[2] = {0.f, 0.f}, bF1[2] = {0.f, 0.f}, bFb[2] = {0.f, 0.f}, bPv[2] = {0.f, 0.f}, boP[2] = {0.f, 0.f};
        int sbF[2] = {0, 0}, sbP[2] = {0, 0};
        const int kP = min(cP, C - 1) / RPW;          // block of this thread's column
        double D2 = 0.0;
        int dead = 0;
        bool met = false;

        // state vectors of the other side for the marginals of pair p (rows t + 1 of its two frames);
        // fetched one pair ahead, and again right after the meeting for the pairs in flight
        auto other = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const int tF = min(2 * p, nlast), tP = min(2 * p + 1, nlast);
            // (32-bit offsets into buffer descriptors: 64-bit addresses per lane would cost the registers
            // this kernel does not have; a column beyond the row reads a neighbour or zero and is unused)
            const float2 bf = buf_load2(brs, colF, (unsigned)(tF + 1) * pitch);
            bF0[B_] = bf.x; bF1[B_] = bf.y;
            bFb[B_] = buf_load(brs, yoff, (unsigned)(tF + 1) * pitch);
            // block exponents: one per lane (lane & 7), picked at the point of use.  A wave-uniform
            // address would make these scalar loads, and every workgroup barrier waits for those.
            sbF[B_] = __builtin_bit_cast(int, buf_load(sbrs, koff, (unsigned)(tF + 1) * (unsigned)(kClMaxK * sizeof(int))));
            bPv[B_] = buf_load(brs, coffP, (unsigned)(tP + 1) * pitch);
            sbP[B_] = __builtin_bit_cast(int, buf_load(sbrs, koff, (unsigned)(tP + 1) * (unsigned)(kClMaxK * sizeof(int))));
            // own states of that vector, relative to the exponent of block 0 (the block of column 0,
            // whose exponent the column-0 thread uses for the empty-label arcs)
            // (only loads here: arithmetic on the loaded values would wait for every load in flight)
            boP[B_] = buf_load(brs, yoff, (unsigned)(tP + 1) * pitch);       // wave 0: own state of this lane
            bSt[B_] = buf_load(brs, nst > 0 ? soffS : kC2Off, (unsigned)(tP + 1) * pitch);   // lanes 0..7: straggler columns
        };
        // after a reload on the rare path: read every reloaded value once, so that none of them counts as
        // pending on the common path (see c2_touch)
        auto settle = [&]() __attribute__((always_inline)) {
            int t = 0;
#pragma unroll
            for (int x = 0; x < 2; ++x)
                t |= c2_touch(bF0[x]) | c2_touch(bF1[x]) | c2_touch(bFb[x]) | c2_touch(bPv[x]) | c2_touch(boP[x]) |
                     c2_touch(bSt[x]) | (sbF[x] == 0x7fffffff) | (sbP[x] == 0x7fffffff);
            if (t) ctl_s[9] = 1;          // (never; nobody reads it)
        };
        // The loads of a pair are issued in four pieces spread over the previous pair: issued in one
        // go, the whole chip would pull at the HBM limit for a moment and every wave would sit in its
        // issue slot until the burst has drained.  Lanes beyond the own columns load nothing.
        auto issueF = [&](auto BUF, int p, int j0, int j1) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned foF = (unsigned)min(2 * p, nlast) * frb;
            int jl = jla;
            c2_pin(jl);
#pragma unroll
            for (int j = 0; j < kC2FJ; ++j)
                if (j >= j0 && j < j1) {
                    const float2 x = buf_load2(wrs, rowcol(j, jl), foF);
                    EF0[B_][j] = x.x;
                    EF1[B_][j] = x.y;
                }
            if (j1 >= kC2FJ) EB[B_] = buf_load(wrs, wave == 0 && fok ? rowB : kC2Off, foF);
            if (GAMMA && j0 == 0) other(BUF, p);
        };
        auto issueP = [&](auto BUF, int p, int r0_, int r1_) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned foP = (unsigned)min(2 * p + 1, nlast) * frb;
#pragma unroll
            for (int r = 0; r < kC2PH; ++r)
                if (r >= r0_ && r < r1_)
                    EP[B_][r] = buf_load(wrs, coffPm, foP + rbaseP + (unsigned)min(rP0 + r, g.nr - 1) * pitch);
            if (r1_ >= kC2PH) ES[B_] = buf_load(wrs, hasS ? coffS : kC2Off, foP + rbaseP);
            if (r1_ >= kC2PH) EBP[B_] = buf_load(wrs, wave == 0 && fok ? rowB : kC2Off, foP);     // w[q][0], own rows
        };
        // exp pass of both frames of a pair (contains workgroup barriers)
        auto prep = [&](auto BUF, auto&& halfway) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            // F frame: one shift per own column, common to all waves and row groups
            float m0 = LAST_NEG_INF, m1 = LAST_NEG_INF;
#pragma unroll
            for (int j = 0; j < kC2FJ; ++j) {
                m0 = fmaxf(m0, EF0[B_][j]);
                m1 = fmaxf(m1, EF1[B_][j]);
            }
            // (maxima of integers through LDS atomics: the order does not matter, one barrier is enough)
            if (lane < 17 * kC2FG) {
                if (v0ok) atomicMax(&shc_s[B_ * kC2Own + c0], shift_for(m0));
                if (v1ok) atomicMax(&shc_s[B_ * kC2Own + c0 + 1], shift_for(m1));
            }
            int touched = 0;
            if (wave == 0 && lane < kC2Own) {
                if (!fok) EB[B_] = LAST_NEG_INF;
                atomicMax(&shc_s[B_ * kC2Own + lane], shift_for(EB[B_]));
            } else {
                touched |= c2_touch(EB[B_]);
            }
            // P frame: one shift per column and thread, the workgroup's largest as reference
            float mp = LAST_NEG_INF;
#pragma unroll
            // (a row beyond the own rows was loaded as a copy of the last one and meets a zero in the sums)
            for (int r = 0; r < kC2PH; ++r) mp = fmaxf(mp, EP[B_][r]);
            const int sp = colok ? shift_for(mp) : kShiftNone;
            int wm = wave_max_dpp(sp);
            int ssp = kShiftNone;
            if (hasS) {
                const float e = lane < g.nr ? ES[B_] : LAST_NEG_INF;
                ssp = shift_for(wave_max_dpp(e));
                ES[B_] = fast_exp2(fmaf(e, kLog2e, -(float)ssp));
                wm = max(wm, ssp);
            } else {
                touched |= c2_touch(ES[B_]);
            }
            c2_pin(ES[B_]);
            if (wave == 0) {
                // empty-label arcs of the own rows: lane <-> row, each with its own shift
                const int sb0 = shift_for(fok ? EBP[B_] : LAST_NEG_INF);
                EBP[B_] = fok ? fast_exp2(fmaf(EBP[B_], kLog2e, -(float)sb0)) : 0.f;
                sbP0[B_] = sb0;
                wm = max(wm, wave_max_dpp(sb0));
            } else {
                touched |= c2_touch(EBP[B_]);
            }
            c2_pin(EBP[B_]);
            if (touched) ctl_s[9] = 1;        // (never; nobody reads it)
            if (lane == 0) atomicMax(&ctl_s[2 + B_], wm);
            c2_barrier();
            // every wave is past the pair that is ending: its cells are cleared for the pass after this one
            if (wave == 1 && lane < kC2Own) shc_s[(B_ ^ 1) * kC2Own + lane] = kShiftNone;
            if (wave == 1 && lane == 0) ctl_s[2 + (B_ ^ 1)] = kShiftNone;
            halfway();
            // (a lane without a column loaded zeros: a huge shift turns them into E = 0)
            const float fsp = sp == kShiftNone ? 3.0e38f : (float)sp;
#pragma unroll
            for (int r = 0; r < kC2PH; ++r) { EP[B_][r] = fast_exp2(fmaf(EP[B_][r], kLog2e, -fsp)); c2_pin(EP[B_][r]); }
            int2 sc2;
            sc2.x = shc_s[B_ * kC2Own + c0]; sc2.y = shc_s[B_ * kC2Own + c0 + 1];
            // (a column this lane does not have: a huge shift makes its E zero; the overlapping column keeps
            // its E, which the marginals need)
            const float fs0 = lact && sc2.x != kShiftNone ? (float)sc2.x : 3.0e38f;
            const float fs1 = v1ok && sc2.y != kShiftNone ? (float)sc2.y : 3.0e38f;
#pragma unroll
            for (int j = 0; j < kC2FJ; ++j) {
                EF0[B_][j] = fast_exp2(fmaf(EF0[B_][j], kLog2e, -fs0));
                EF1[B_][j] = fast_exp2(fmaf(EF1[B_][j], kLog2e, -fs1));
                c2_pin(EF0[B_][j]); c2_pin(EF1[B_][j]);
            }
            if (wave == 0) EB[B_] = fast_exp2(fmaf(EB[B_], kLog2e, -(float)shc_s[B_ * kC2Own + min(lane, kC2Own - 1)]));
            c2_pin(EB[B_]);
            shP[B_] = sp; sigP[B_] = ctl_s[2 + B_]; ssP[B_] = ssp;
            if (GAMMA) {
                c2_pin(bSt[B_]);
                // The prefetched values of the other side have arrived with the frame.  Touching them here
                // keeps the compiler from guarding their later uses with waits counted along the shortest
                // path, which on the waves that load more would stall on loads issued in between.
                c2_pin(bF0[B_]); c2_pin(bF1[B_]); c2_pin(bFb[B_]); c2_pin(bPv[B_]); c2_pin(boP[B_]);
                c2_pin(sbF[B_]); c2_pin(sbP[B_]);
            }
        };
        auto meet = [&]() __attribute__((always_inline)) {
            if (dead) ctl_s[8] = 1;
            cluster_sync(a, g, ptag, &ctl_s[8]);
            ptag += 1;
            D2 = c2_meeting(ah + (size_t)mid * C, bh + (size_t)mid * C, Sa + (size_t)mid * kClMaxK,
                            Sb + (size_t)mid * kClMaxK, C, RPW, K, redb);
            if (g.k == 0 && tid == 0) {
                a.dist[b] = bad ? __builtin_nanf("") : (float)(D2 * 0.6931471805599453);
                if (a.item_status)
                    a.item_status[b] = bad ? kItemBadLength : (ctl_s[8] ? kItemTimeout : kItemOk);
            }
            met = true;
            __syncthreads();
        };

        issueF(std::integral_constant<int, 0>(), 0, 0, kC2NQ);
        issueP(std::integral_constant<int, 0>(), 0, 0, kC2PH);
        prep(std::integral_constant<int, 0>(), [] {});

        int p = 0;
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value;
            const int tF = 2 * p, tP = 2 * p + 1;
            if (tF >= n) return false;
            // ---------------- F-step: frame tF, all rows x own columns, from the whole vector
            if (tF == mid && !met) {
                meet();
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B_ ^ 1>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            }
            {
                const int S = ctl_s[0];
                float aq[kC2FJ];
#pragma unroll
                for (int j = 0; j < kC2FJ; ++j) aq[j] = full_s[min(qF0 + kC2FG * j, 319)];
                float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
                for (int j = 0; j < kC2FJ; ++j) {
                    ps0 = fmaf(aq[j], EF0[B_][j], ps0);
                    ps1 = fmaf(aq[j], EF1[B_][j], ps1);
                }
                if (v0ok) red_s[slotF] = ps0;
                if (v1ok) red_s[slotF + 1] = ps1;
                if (GAMMA && tF >= mid) {
                    const unsigned gso = (unsigned)tF * frb;
                    const int sbk = __builtin_amdgcn_readlane(sbF[B_], g.k);
                    {
                        // every lane with columns stores 8 bytes (see c2_pair); 4-byte stores only in a workgroup
                        // with a single label column
                        int2 sc2;
                        sc2.x = shc_s[B_ * kC2Own + c0]; sc2.y = shc_s[B_ * kC2Own + c0 + 1];
                        const float fc0 = a.scale * bF0[B_] * c2_marginal_scale(sbk + S + sc2.x, D2, ctl_s);
                        const float fc1 = a.scale * bF1[B_] * c2_marginal_scale(sbk + S + sc2.y, D2, ctl_s);
                        const unsigned off2 = (lact && !pr.single) ? coffF : kC2Off;
                        const unsigned off1 = (lact && pr.single) ? coffF : kC2Off;
                        int jl = jlim;
                        c2_pin(jl);
#pragma unroll
                        for (int j = 0; j < kC2FJ; ++j) {
                            const unsigned so = gso + rowF0 + (unsigned)(kC2FG * j) * pitch;
                            const float g0 = aq[j] * EF0[B_][j] * fc0, g1 = aq[j] * EF1[B_][j] * fc1;
                            c2_put2<ACC>(g0, g1, grs, j < jl ? off2 : kC2Off, so, v0ok, v1ok);
                            if (need1) c2_put<ACC>(g0, grs, j < jl ? off1 : kC2Off, so);
                            __builtin_amdgcn_sched_barrier(0);     // one row at a time: registers
                        }
                    }
                    if (wave == 0 && fok) {
                        const float fcb = a.scale * bFb[B_] * c2_marginal_scale(sbk + S + shc_s[B_ * kC2Own + lane], D2, ctl_s);
                        c2_put<ACC>(full_s[yF] * EB[B_] * fcb, grs, rowB, gso);
                    }
                }
                c2_barrier();
                // next pair's F frame: waves 1..7 request theirs while wave 0 adds up the columns; wave 0
                // requests its own afterwards (alone on the address path, that is quick)
                if (wave != 0) issueF(std::integral_constant<int, B_ ^ 1>(), p + 1, 0, kC2FJ);
                if (wave == 0) {
                    float v = 0.f;
                    const int shFl = shc_s[B_ * kC2Own + min(lane, kC2Own - 1)];
                    if (fok) {
                        // all partial sums are requested before the first is used (left to itself the
                        // compiler waits for every LDS read in turn to save registers: 12 round trips)
                        float pr[kC2RedN];
#pragma unroll
                        for (int x = 0; x < kC2RedN; ++x) pr[x] = red_s[x * kC2Own + lane];
                        const float ay = full_s[yF];
                        __builtin_amdgcn_sched_group_barrier(0x100, kC2RedN + 1, 0);    // the LDS reads
                        __builtin_amdgcn_sched_group_barrier(0x002, kC2RedN + 1, 0);    // then the additions
#pragma unroll
                        for (int x = 0; x < kC2RedN; ++x) v += pr[x];
                        v = fmaf(ay, EB[B_], v);
                    }
                    const int sc = (fok && v > 0.f) ? shFl + float_exponent(v) : kShiftNone;
                    const int ms = wave_max_dpp(sc);
                    const float own = (sc == kShiftNone) ? 0.f : c2_scale(v, shFl - ms);
                    if (lane < kC2Own) own_s[lane] = own;
                    const int ek = (ms == kShiftNone) ? S : S + ms;
                    if (lane == 0) ctl_s[1] = ek;
                    if (tF + 1 <= mid) {
                        if (fok) ah[(size_t)(tF + 1) * C + g.r0 + lane] = own;
                        if (lane == 0) Sa[(size_t)(tF + 1) * kClMaxK + g.k] = ek;
                    }
                    issueF(std::integral_constant<int, B_ ^ 1>(), p + 1, 0, kC2FJ);
                }
                c2_barrier();
            }
            if (tP >= n) return false;
            issueP(std::integral_constant<int, B_ ^ 1>(), p + 1, 0, 9);
            // ---------------- P-step: frame tP, own rows x all columns, partial sums for every state
            if (tP == mid && !met) {
                meet();
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B_ ^ 1>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            }
            {
                const unsigned tag = gstep + 1;
                u64* xs = xbase + (size_t)(gstep & 1) * kClMaxK * kC2XS;
                const int ek = ctl_s[1];
                float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
                for (int r = 0; r < kC2PH; ++r) {
                    if (r & 1) acc1 = fmaf(own_s[rP0 + r], EP[B_][r], acc1); else acc0 = fmaf(own_s[rP0 + r], EP[B_][r], acc0);
                }
                const int sp = shP[B_], sg = sigP[B_], ssp = ssP[B_];
                const float val = (sp == kShiftNone) ? 0.f : c2_scale(acc0 + acc1, sp - sg);
                issueP(std::integral_constant<int, B_ ^ 1>(), p + 1, 9, kC2PH);
                if (wave == 0 && lane < kC2Own)
                    bl_s[lane] = (sbP0[B_] == kShiftNone) ? 0.f : c2_scale(own_s[lane] * EBP[B_], sbP0[B_] - sg);
                if (hP == 1) pacc_s[cP] = val;                 // second half of the own rows
                if (hasS) {
                    const float sv = wave_sum_dpp(lane < g.nr ? own_s[lane] * ES[B_] : 0.f);
                    if (lane == 0) strag_s[sS] = (ssp == kShiftNone) ? 0.f : c2_scale(sv, ssp - sg);
                }
                if (GAMMA && wave == 0) {
                    const int dk = __builtin_amdgcn_readlane(sbP[B_], g.k) - __builtin_amdgcn_readlane(sbP[B_], 0);
                    // own state times the other side's value of the same state: what the empty-label arcs
                    // (column 0) are multiplied with in place of the own state alone
                    if (lane < kC2Own) bo_s[lane] = lane < g.nr ? own_s[lane] * c2_scale(boP[B_], dk) : 0.f;
                }
                c2_barrier();
                const bool exch = !(GAMMA && tP == L - 1);
                if (tid < C && exch) {
                    // threads 0..255 are the first halves of their columns; 256.. publish the stragglers
                    float pub = tid < kC2PC ? (tid == 0 ? 0.f : val + pacc_s[tid])      // column 0: the empty label
                                            : strag_s[tid - kC2PC];
                    if (tid >= g.r0 && tid < g.r0 + g.nr) pub += bl_s[tid - g.r0];
                    xpublish(xs + (size_t)g.k * kC2XS + tid, c2_pack(pub, tag, (sg == kShiftNone ? ek : ek + sg) - ctl_s[0]));
                }
                if (GAMMA && tP >= mid) {
                    const int sbk = __shfl(sbP[B_], kP, 64);       // every lane takes part
                    const unsigned gso = (unsigned)tP * frb + rbaseP;
                    {
                        const float fy = (sp == kShiftNone) ? 0.f : a.scale * c2_marginal_scale(sbk + sp + ek, D2, ctl_s) * (cP == 0 ? 1.f : bPv[B_]);
                        // the empty label (column 0) returns to the row's own state: its thread reads the
                        // products instead of the own states; all reads first, then the stores
                        const float* osrc = (cP == 0 ? bo_s : own_s) + rP0;
                        float ov[kC2PH];
#pragma unroll
                        for (int r = 0; r < kC2PH; ++r) ov[r] = osrc[r];
#pragma unroll
                        for (int r = 0; r < kC2PH; ++r)
                            c2_put<ACC>(ov[r] * EP[B_][r] * fy, grs, rP0 + r < g.nr ? coffPm : kC2Off,
                                      gso + (unsigned)(rP0 + r) * pitch);
                    }
                    if (hasS) {
                        const int sbkS = __builtin_amdgcn_readlane(sbP[B_], cS / RPW);
                        const float bS = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bSt[B_]), sS));
                        const float fyS = (ssp == kShiftNone) ? 0.f
                                          : a.scale * bS * c2_marginal_scale(sbkS + ssp + ek, D2, ctl_s);
                        c2_put<ACC>(own_s[min(lane, kC2Own - 1)] * ES[B_] * fyS, grs, coffS, gso);
                    }
                }
                // first look at the exchange halfway through the exp pass: early enough for the round trip to
                // the L2 cache to end with the pass, late enough for the other workgroups' words to be there
                C2Look lk;
                prep(std::integral_constant<int, B_ ^ 1>(), [&]() __attribute__((always_inline)) { if (exch) c2_gather_look<FULL>(xs, K, C, lk); });
                if (exch) {
                    c2_gather<FULL>(xs, K, C, tag, full_s, ctl_s, a.spin_limit, dead, lk, [] {});
                    gstep += 1;
                    if (tP + 1 <= mid && wave == 6) {      // (a wave with no other special duty)
                        if (lane < g.nr) ah[(size_t)(tP + 1) * C + g.r0 + lane] = full_s[g.r0 + lane];
                        if (lane == 0) Sa[(size_t)(tP + 1) * kClMaxK + g.k] = ctl_s[0];
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
        if (tid == 0 && ctl_s[11] && a.item_status && !bad) atomicMax(&a.item_status[b], (int)kItemRange);
        if (tid == 0) cluster_finish_item(a, b, ctl_s[8] != 0 || dead != 0, bad, 2 * a.K);
        __syncthreads();
    }
}

// ------------------------------------------------------------------- beta role
template <bool GAMMA, bool ACC, bool FULL>
__device__ __forceinline__ void beta2_role(const ClusterArgs& a, const ClusterGeom& g, float* smem,
                                           unsigned& gstep, unsigned& ptag)
{
    float* full_s = smem + kC2Full;
    float* own_s = smem + kC2OwnS;
    float* red_s = smem + kC2RowF;            // [40] row sums of the F-step
    int* shr_s = (int*)(smem + kC2RowS);      // [40] their shifts
    int* shc_s = (int*)(smem + kC2Shc);
    float* bl_s = smem + kC2Bl;
    float* bt_s = smem + kC2Bt;
    float* afull_s = smem + kC2Afull;
    float* red2_s = smem + kC2Red2;
    int* ctl_s = (int*)(smem + kC2Ctl);
    float* redb = smem + kC2RedB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int C = a.C, K = a.K, RPW = a.RPW;
    // F-step: wave <-> own rows wave, wave + 8, ..., lane <-> four neighbouring columns cb4 .. cb4 + 3 of the
    // first 256 (one 16-byte access per row); the columns beyond (at most 8) of all rows of the wave by one
    // more instruction: lane <-> (row lane & 7, column 256 + (lane >> 3)).  Where the row ends inside or before
    // a lane's four columns the lane takes the last four of the row instead: what it has in common with its
    // predecessors enters no sum (their entry of the state vector is replaced by zero) and is stored twice
    // with the same value, or not at all by a lane that lies wholly beyond the row.
    int nrw = (g.nr - wave + kC2Waves - 1) / kC2Waves;
    if (nrw < 0) nrw = 0;
    const int nstF = max(C - kC2PC, 0);
    const int rS = lane & 7, sI = lane >> 3;
    const bool validS = rS < nrw && rS < kC2RW && sI < nstF;
    const int cb4 = min(4 * lane, min(C, kC2PC) - 4);      // (C >= 4 on this path)
    const bool st4 = 4 * lane < min(C, kC2PC);             // the lane has a column nobody else has
    // P-step (all rows x own columns): wave <-> rows [33 wave, 33 wave + 33); seven groups of nine lanes take
    // every seventh row (row slot 7 j + group, j < 5; slots 33 and 34 are unused), a lane four neighbouring
    // own columns (16-byte loads and stores).  One shift per own column; the lanes' partial sums of a row
    // meet in LDS, where thread <-> row qT adds them up and publishes.
    const int gq = min(lane / kC2QL, kC2QG - 1), ci = lane - kC2QL * (lane / kC2QL);
    const C2Quad qd = c2_quad(ci, lane < kC2QL * kC2QG, g.r0, g.nr);    // (column 0 is the empty label)
    const bool lact = qd.act;
    const int c0 = qd.c0;
    bool vok[4];                                        // columns this lane adds up: the overlap only once
#pragma unroll
    for (int k = 0; k < 4; ++k) vok[k] = lact && k >= qd.ndup;
    const int qF0 = kC2NQ * wave + gq;                  // first row of this lane
    // rows j < jlim exist: inside the wave's 33 and inside the matrix
    const int jlim = lact ? max(min((kC2NQ - gq + kC2QG - 1) / kC2QG, (C - qF0 + kC2QG - 1) / kC2QG), 0) : 0;
    const bool slot4 = lane < kC2QL * kC2QG && gq < kC2NQ - kC2QG * (kC2QJ - 1);   // the lane's fifth row slot is one of the wave's
    const bool fok = lane < g.nr;                       // wave 0: lane <-> own state (empty-label arcs)
    const int yF = min(g.r0 + lane, C - 1);
    const int qT = min(tid, C - 1);
    const bool rowok = tid < C;
    const bool rowown = rowok && tid >= g.r0 && tid < g.r0 + g.nr;

    for (int b = g.cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int mid = L / 2;
        const int n = GAMMA ? L : L - mid;
        const int ph1 = L - mid;                      // step at which the state index reaches mid
        const size_t fr = (size_t)C * C;
        const unsigned frb = (unsigned)(fr * sizeof(float));
        const unsigned pitch = (unsigned)(C * (int)sizeof(float));
        const float* wi = a.w + (size_t)b * a.T * fr;
        float* gi = GAMMA ? a.dw + (size_t)b * a.T * fr : nullptr;
        const float* ah = a.ahat + (size_t)b * (a.T + 1) * C;
        float* bh = a.bhat + (size_t)b * (a.T + 1) * C;
        const int* Sa = a.Sa + (size_t)b * (a.T + 1) * kClMaxK;
        int* Sb = a.Sb + (size_t)b * (a.T + 1) * kClMaxK;
        u64* xbase = a.xb + (size_t)g.cg * 2 * kClMaxK * kC2XS;
        const buf_t wrs = make_buf(wi, (unsigned)a.T * frb);
        const buf_t grs = make_buf(GAMMA ? (const float*)gi : wi, GAMMA ? (unsigned)a.T * frb : 0u);
        const unsigned coff4 = (unsigned)(cb4 * (int)sizeof(float));
        const unsigned coff4s = st4 ? coff4 : kC2Off;
        auto roff = [&](int ri) __attribute__((always_inline)) {              // scalar
            return (unsigned)(g.r0 + min(wave + ri * kC2Waves, g.nr - 1)) * pitch;
        };
        const int nlast = max(n - 1, 0);
        // the other side's vectors through 32-bit offsets (registers)
        const buf_t ars = make_buf(ah, (unsigned)(a.T + 1) * pitch);
        const buf_t sars = make_buf(Sa, (unsigned)(a.T + 1) * (unsigned)(kClMaxK * sizeof(int)));
        const unsigned koff = (unsigned)((lane & 7) * (int)sizeof(int));
        // lanes 0..4 of a wave: the wave's own rows of the F-step
        const unsigned aoffF = (unsigned)((g.r0 + max(min(wave + min(lane, kC2RW - 1) * kC2Waves, g.nr - 1), 0)) * (int)sizeof(float));
        const unsigned offSt = validS ? (unsigned)(g.r0 + wave + rS * kC2Waves) * pitch + (unsigned)((kC2PC + sI) * (int)sizeof(float))
                                      : kC2Off;
        const unsigned colF = (unsigned)((g.r0 + c0) * (int)sizeof(float));
        const unsigned coffF = (unsigned)gq * pitch + colF;
        const unsigned rowF0 = (unsigned)(kC2NQ * wave) * pitch;     // scalar: first row of this wave
        const unsigned rowB = (unsigned)yF * pitch;                  // row of the own state (empty-label weight)

        // Offset of this lane's four elements in row slot j.  A slot beyond the wave's rows or beyond the
        // matrix is replaced by the last row: what is loaded there is finite, takes part in no maximum that
        // matters, and is neither added up nor stored.  A lane without columns of its own repeats the address
        // of a lane that has some (no traffic of its own); its elements are zeroed by its shift.  (jl: the
        // number of slots, through a register the compiler cannot see through, so that the offsets are made
        // where they are used instead of being kept.)
        const unsigned cola = colF;          // (c2_quad gives a lane without columns the last quad's)
        const unsigned offA0 = (unsigned)qF0 * pitch + cola;
        const unsigned offAL = (unsigned)(C - 1) * pitch + cola;
        const int jla = max(min((kC2NQ - gq + kC2QG - 1) / kC2QG, (C - qF0 + kC2QG - 1) / kC2QG), 0);
        auto rowcol = [&](int j, int jl) __attribute__((always_inline)) {
            return j < jl ? offA0 + (unsigned)(kC2QG * j) * pitch : offAL;
        };
        // b_L = 1 for every state, exponent 0
        for (int q = tid; q < 320; q += kC2Threads) full_s[q] = q < C ? 1.f : 0.f;
        if (tid < kC2Own) own_s[tid] = 0.f;
        if (tid < 32) ctl_s[tid] = 0;
        if (tid < 2 * kC2Own) shc_s[tid] = kShiftNone;
        if (tid < kC2Own) { bt_s[tid] = 0.f; bl_s[tid] = 0.f; }
        for (int q = tid; q < kC2Waves * kC2NQ * kC2R2S; q += kC2Threads) red2_s[q] = 0.f;    // (cells beyond the ninth of a row stay zero)
        if (tid < g.nr) bh[(size_t)L * C + g.r0 + tid] = 1.f;
        if (tid == 0) Sb[(size_t)L * kClMaxK + g.k] = 0;
        __syncthreads();

        float EFb[2][kC2RW][kC2NC], ESb[2] = {0.f, 0.f};
        float EQ[2][kC2QJ][4];
        float EB[2] = {0.f, 0.f};
        int srF[2][kC2RW];
        float aF[2] = {0.f, 0.f}, aP[2] = {0.f, 0.f};      // other side's vector for the marginals
        int saF[2] = {0, 0}, saP[2] = {0, 0};
        double D2 = 0.0;
        int dead = 0;
        bool met = false;
        int p = 0;                // pair counter
        float xwide = -3.0e38f;   // largest exponent of a marginal scale relative to D

        // step index i -> frame L - 1 - i; pair p = steps 2p (F) and 2p + 1 (P)
        auto frameF = [&](int p) { return max(L - 1 - min(2 * p, nlast), 0); };
        auto frameP = [&](int p) { return max(L - 1 - min(2 * p + 1, nlast), 0); };
        // state vectors of the other side for the marginals of pair p (rows t of its two frames);
        // fetched one pair ahead, and again right after the meeting for the pairs in flight
        auto other = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const int tF = frameF(p), tP = frameP(p);
            aF[B_] = buf_load(ars, aoffF, (unsigned)tF * pitch);
            // block exponents: one per lane (lane & 7), picked at the point of use.  A wave-uniform
            // address would make these scalar loads, and every workgroup barrier waits for those.
            saF[B_] = __builtin_bit_cast(int, buf_load(sars, koff, (unsigned)tF * (unsigned)(kClMaxK * sizeof(int))));
            aP[B_] = buf_load(ars, (unsigned)(qT * (int)sizeof(float)), (unsigned)tP * pitch);
            saP[B_] = __builtin_bit_cast(int, buf_load(sars, koff, (unsigned)tP * (unsigned)(kClMaxK * sizeof(int))));
        };
        // after a reload on the rare path: read every reloaded value once, so that none of them counts as
        // pending on the common path (see c2_touch)
        auto settle = [&]() __attribute__((always_inline)) {
            int t = 0;
#pragma unroll
            for (int x = 0; x < 2; ++x)
                t |= c2_touch(aF[x]) | c2_touch(aP[x]) | (saF[x] == 0x7fffffff) | (saP[x] == 0x7fffffff);
            if (t) ctl_s[9] = 1;          // (never; nobody reads it)
        };
        auto issueF = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned foF = (unsigned)frameF(p) * frb;
#pragma unroll
            for (int ri = 0; ri < kC2RW; ++ri) {
                // (a wave without a row ri loads nothing: every lane out of range)
                const float4 x = buf_load4(wrs, ri < nrw ? coff4 : kC2Off, foF + roff(ri));
                EFb[B_][ri][0] = x.x; EFb[B_][ri][1] = x.y; EFb[B_][ri][2] = x.z; EFb[B_][ri][3] = x.w;
            }
            ESb[B_] = buf_load(wrs, offSt, foF);
            if (GAMMA) other(BUF, p);
        };
        auto issueP = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned foP = (unsigned)frameP(p) * frb;
            int jl = jla;
            c2_pin(jl);
#pragma unroll
            for (int j = 0; j < kC2QJ; ++j) {
                const float4 x = buf_load4(wrs, rowcol(j, jl), foP);
                EQ[B_][j][0] = x.x; EQ[B_][j][1] = x.y; EQ[B_][j][2] = x.z; EQ[B_][j][3] = x.w;
            }
            EB[B_] = buf_load(wrs, wave == 0 && fok ? rowB : kC2Off, foP);           // w[q][0] of the own states
        };
        auto prep = [&](auto BUF, auto&& halfway) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            // F frame: one shift per own row (wave-uniform).  All five rows at once, without branches, so
            // that their cross-lane reductions overlap: a row the wave does not have holds the zeros of its
            // out-of-range loads, and what is made of them is used nowhere.
            float fsS = 3.0e38f;       // shift of the row of this lane's straggler element
            int touched = 0;
            float mxr[kC2RW];
#pragma unroll
            for (int ri = 0; ri < kC2RW; ++ri) {
                float mx = (validS && rS == ri) ? ESb[B_] : LAST_NEG_INF;
#pragma unroll
                for (int j = 0; j < kC2NC; ++j) mx = fmaxf(mx, EFb[B_][ri][j]);
                mxr[ri] = mx;
            }
            int kr[kC2RW];
#pragma unroll
            for (int ri = 0; ri < kC2RW; ++ri) kr[ri] = c2_fkey(mxr[ri]);
#pragma unroll
            for (int ri = 0; ri < kC2RW; ++ri) kr[ri] = c2_wave_max_key(kr[ri]);
#pragma unroll
            for (int ri = 0; ri < kC2RW; ++ri) mxr[ri] = c2_fkey_inv(kr[ri]);
#pragma unroll
            for (int ri = 0; ri < kC2RW; ++ri) {
                const int s = shift_for(mxr[ri]);
                srF[B_][ri] = ri < nrw ? s : kShiftNone;
                const float fs = (float)s;
                if (rS == ri) fsS = fs;
#pragma unroll
                for (int j = 0; j < kC2NC; ++j) {
                    EFb[B_][ri][j] = fast_exp2(fmaf(EFb[B_][ri][j], kLog2e, -fs));
                    c2_pin(EFb[B_][ri][j]);
                }
            }
            ESb[B_] = validS ? fast_exp2(fmaf(ESb[B_], kLog2e, -fsS)) : 0.f;
            c2_pin(ESb[B_]);
            halfway();
            // P frame: one shift per own column, common to all waves and row groups; the empty-label weight
            // of an own state q shares the shift of the column of q, whose value it multiplies
            float mq[4] = {LAST_NEG_INF, LAST_NEG_INF, LAST_NEG_INF, LAST_NEG_INF};
#pragma unroll
            for (int j = 0; j < kC2QJ; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k) mq[k] = fmaxf(mq[k], EQ[B_][j][k]);
            // (maxima of integers through LDS atomics: the order does not matter, one barrier is enough)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (vok[k]) atomicMax(&shc_s[B_ * kC2Own + c0 + k], shift_for(mq[k]));
            if (wave == 0 && lane < kC2Own) {
                if (!fok) EB[B_] = LAST_NEG_INF;
                atomicMax(&shc_s[B_ * kC2Own + lane], shift_for(EB[B_]));
            } else {
                touched |= c2_touch(EB[B_]);
            }
            if (touched) ctl_s[9] = 1;        // (never; nobody reads it)
            c2_barrier();
            // every wave is past the pair that is ending: its cells are cleared for the pass after this one
            if (wave == 1 && lane < kC2Own) shc_s[(B_ ^ 1) * kC2Own + lane] = kShiftNone;
            if (wave == 0) {
                // largest shift of the own columns: the reference of the P-step's partial sums
                const int sg = wave_max_dpp(fok ? shc_s[B_ * kC2Own + lane] : kShiftNone);
                if (lane == 0) ctl_s[2 + B_] = sg;
            }
            // (a lane without columns: a huge shift makes its E zero; the overlapping columns keep their E,
            // which the marginals need)
            float fsq[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int sc = shc_s[B_ * kC2Own + c0 + k];
                fsq[k] = lact && sc != kShiftNone ? (float)sc : 3.0e38f;
            }
#pragma unroll
            for (int j = 0; j < kC2QJ; ++j)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    EQ[B_][j][k] = fast_exp2(fmaf(EQ[B_][j][k], kLog2e, -fsq[k]));
                    c2_pin(EQ[B_][j][k]);
                }
            if (wave == 0) EB[B_] = fast_exp2(fmaf(EB[B_], kLog2e, -(float)shc_s[B_ * kC2Own + min(lane, kC2Own - 1)]));
            c2_pin(EB[B_]);
            if (GAMMA) { c2_pin(aF[B_]); c2_pin(aP[B_]); c2_pin(saF[B_]); c2_pin(saP[B_]); }
        };
        auto meet = [&]() __attribute__((always_inline)) {
            if (dead) ctl_s[8] = 1;
            cluster_sync(a, g, ptag, &ctl_s[8]);
            ptag += 1;
            D2 = c2_meeting(ah + (size_t)mid * C, bh + (size_t)mid * C, Sa + (size_t)mid * kClMaxK,
                            Sb + (size_t)mid * kClMaxK, C, RPW, K, redb);
            met = true;
            __syncthreads();
        };

        issueF(std::integral_constant<int, 0>(), 0);
        issueP(std::integral_constant<int, 0>(), 0);
        prep(std::integral_constant<int, 0>(), [] {});
        issueP(std::integral_constant<int, 1>(), 1);
        issueF(std::integral_constant<int, 1>(), 1);

        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value;
            const int iF = 2 * p, iP = 2 * p + 1;
            if (iF >= n) return false;
            // ---------------- F-step: frame tF, own rows x all columns, from the whole vector
            if (iF == ph1 && !met) {
                meet();
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B_ ^ 1>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            }
            {
                const int tF = L - 1 - iF;
                const int S = ctl_s[0];
                // bg: the columns' values; bv: the same with zero for columns that belong to a lane before
                float bg[kC2NC], bv[kC2NC];
#pragma unroll
                for (int j = 0; j < kC2NC; ++j) {
                    bg[j] = full_s[cb4 + j];
                    bv[j] = cb4 + j >= 4 * lane ? bg[j] : 0.f;
                }
                // straggler element of this lane times its column's value; it joins the sum of its row
                const float bS = full_s[min(kC2PC + sI, 319)];
                const float sprod = ESb[B_] * bS;
                float facS = 0.f;
                // all five rows at once, without branches: the cross-lane sums overlap (a row the wave does
                // not have gives a sum that is not written)
                float brow[kC2RW], tot[kC2RW];
#pragma unroll
                for (int ri = 0; ri < kC2RW; ++ri) brow[ri] = full_s[g.r0 + max(min(wave + ri * kC2Waves, g.nr - 1), 0)];
#pragma unroll
                for (int ri = 0; ri < kC2RW; ++ri) {
                    // the empty label (column 0) returns to the row's own state
                    float acc = EFb[B_][ri][0] * (lane == 0 ? brow[ri] : bv[0]);
#pragma unroll
                    for (int j = 1; j < kC2NC; ++j) acc = fmaf(EFb[B_][ri][j], bv[j], acc);
                    if (nstF > 0) acc += rS == ri ? sprod : 0.f;
                    tot[ri] = acc;
                }
#pragma unroll
                for (int ri = 0; ri < kC2RW; ++ri) tot[ri] = wave_sum_dpp(tot[ri]);
#pragma unroll
                for (int ri = 0; ri < kC2RW; ++ri) {
                    const int rloc = wave + ri * kC2Waves;
                    if (lane == 0 && ri < nrw) {
                        red_s[rloc] = tot[ri];
                        shr_s[rloc] = srF[B_][ri];
                    }
                }
                if (GAMMA && iF >= ph1) {
#pragma unroll
                    for (int ri = 0; ri < kC2RW; ++ri) {
                        const float arow = __shfl(aF[B_], ri, 64);
                        const float fac = a.scale * arow *
                                          c2_marginal_scale(__builtin_amdgcn_readlane(saF[B_], g.k) + srF[B_][ri] + S, D2, xwide);
                        if (rS == ri) facS = fac;
                        const unsigned gso = (unsigned)tF * frb + roff(ri);
                        const unsigned so4 = ri < nrw ? coff4s : kC2Off;
                        c2_put4<ACC>(EFb[B_][ri][0] * (lane == 0 ? brow[ri] : bg[0]) * fac, EFb[B_][ri][1] * bg[1] * fac,
                                     EFb[B_][ri][2] * bg[2] * fac, EFb[B_][ri][3] * bg[3] * fac, grs, so4, gso,
                                     cb4 >= 4 * lane, cb4 + 1 >= 4 * lane, cb4 + 2 >= 4 * lane, cb4 + 3 >= 4 * lane);
                    }
                }
                if (GAMMA && iF >= ph1 && nstF > 0) c2_put<ACC>(sprod * facS, grs, offSt, (unsigned)tF * frb);
                c2_barrier();
                {
                    // Every wave by itself, lane <-> own state: the same values from the same inputs, written
                    // to the same cells; a wave reads them only after its own writes, so no second barrier.
                    const bool ok = lane < g.nr;
                    const float v = ok ? red_s[lane] : 0.f;
                    const int sc = (ok && v > 0.f) ? shr_s[lane] + float_exponent(v) : kShiftNone;
                    const int ms = wave_max_dpp(sc);
                    const float own = (sc == kShiftNone) ? 0.f : c2_scale(v, shr_s[lane] - ms);
                    if (lane < kC2Own) {
                        own_s[lane] = own;
                        // for the P-step: own states times 2^(shift of their column - largest shift)
                        bt_s[lane] = c2_scale(own, shc_s[B_ * kC2Own + lane] - ctl_s[2 + B_]);
                    }
                    const int ek = (ms == kShiftNone) ? S : S + ms;
                    if (lane == 0) ctl_s[1] = ek;
                    if (wave == 0 && tF >= mid) {
                        if (ok) bh[(size_t)tF * C + g.r0 + lane] = own;
                        if (lane == 0) Sb[(size_t)tF * kClMaxK + g.k] = ek;
                    }
                }
            }
            if (iP >= n) return false;
            // ---------------- P-step: frame tP, all rows x own columns, partial sums for every state
            if (iP == ph1 && !met) {
                meet();
                if (GAMMA) {
                    other(std::integral_constant<int, B_>(), p);
                    other(std::integral_constant<int, B_ ^ 1>(), p + 1);
                    c2_wait_loads();
                    settle();
                }
            }
            {
                const int tP = L - 1 - iP;
                const unsigned tag = gstep + 1;
                u64* xs = xbase + (size_t)(gstep & 1) * kClMaxK * kC2XS;
                const int ek = ctl_s[1];
                const int sg = ctl_s[2 + B_];
                const bool exch = !(GAMMA && iP == L - 1);
                // b'[q] = sum over the own label columns of M[q][y] b[y]  (+ M[q][0] b[q] for an own state):
                // every lane its two columns of its eleven rows, then thread <-> row over the lanes' parts
                {
                    float bt[4];                    // (an overlapping column is counted by its other lane)
#pragma unroll
                    for (int k = 0; k < 4; ++k) bt[k] = vok[k] ? bt_s[c0 + k] : 0.f;
#pragma unroll
                    for (int j = 0; j < kC2QJ; ++j) {
                        float pj = EQ[B_][j][0] * bt[0];
#pragma unroll
                        for (int k = 1; k < 4; ++k) pj = fmaf(EQ[B_][j][k], bt[k], pj);
                        if (j < kC2QJ - 1 ? lane < kC2QL * kC2QG : slot4) red2_s[(qF0 + kC2QG * j) * kC2R2S + ci] = pj;
                    }
                    if (wave == 0 && lane < kC2Own) bl_s[lane] = EB[B_] * bt_s[lane];
                }
                int samax = 0;
                if (GAMMA && iP >= ph1) {
                    // the other side's vector for the marginals, all blocks on the largest block exponent
                    const int sak = __shfl(saP[B_], qT / RPW, 64);
                    samax = wave_max_dpp(lane < K ? saP[B_] : -(1 << 30));
                    if (tid < 320) afull_s[tid] = rowok ? c2_scale(aP[B_], sak - samax) : 0.f;
                }
                c2_barrier();
                if (rowok && exch) {
                    const float4* rp4 = (const float4*)&red2_s[tid * kC2R2S];
                    const float4 x0 = rp4[0], x1 = rp4[1], x2 = rp4[2];
                    float pub = ((x0.x + x0.y) + (x0.z + x0.w)) + ((x1.x + x1.y) + (x1.z + x1.w)) + ((x2.x + x2.y) + (x2.z + x2.w));
                    if (rowown) pub += bl_s[tid - g.r0];
                    xpublish(xs + (size_t)g.k * kC2XS + tid, c2_pack(pub, tag, (sg == kShiftNone ? ek : ek + sg) - ctl_s[0]));
                }
                if (GAMMA && iP >= ph1) {
                    // marginals: gamma[q][y] = a_t[q] M[q][y] b_{t+1}[y] / Z
                    const unsigned gso = (unsigned)tP * frb;
                    float fq[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        fq[k] = a.scale * own_s[c0 + k] *
                                c2_marginal_scale(shc_s[B_ * kC2Own + c0 + k] + ek + samax, D2, xwide);
                    const unsigned offq = lact ? coffF : kC2Off;
                    int jl = jlim;
                    c2_pin(jl);
                    float aq[kC2QJ];
#pragma unroll
                    for (int j = 0; j < kC2QJ; ++j) aq[j] = afull_s[min(qF0 + kC2QG * j, 319)];
#pragma unroll
                    for (int j = 0; j < kC2QJ; ++j) {
                        const unsigned so = gso + rowF0 + (unsigned)(kC2QG * j) * pitch;
                        const unsigned oj = j < jl ? offq : kC2Off;
                        c2_put4<ACC>(aq[j] * EQ[B_][j][0] * fq[0], aq[j] * EQ[B_][j][1] * fq[1], aq[j] * EQ[B_][j][2] * fq[2],
                                     aq[j] * EQ[B_][j][3] * fq[3], grs, oj, so, vok[0], vok[1], vok[2], vok[3]);
                        __builtin_amdgcn_sched_barrier(0);     // one row at a time: registers
                    }
                    if (wave == 0 && fok) {
                        // empty-label arc of the own state q: a_t[q] M[q][0] b_{t+1}[q]
                        const float fb = a.scale * own_s[lane] *
                                         c2_marginal_scale(shc_s[B_ * kC2Own + lane] + ek + samax, D2, xwide);
                        c2_put<ACC>(afull_s[yF] * EB[B_] * fb, grs, rowB, gso);
                    }
                }
                // the P frame of the pair after the next, into the registers this P-step has finished with
                if (wave < 4) issueP(std::integral_constant<int, B_>(), p + 2);
                // first look at the exchange halfway through the exp pass: early enough for the round trip to
                // the L2 cache to end with the pass, late enough for the other workgroups' words to be there
                C2Look lk;
                prep(std::integral_constant<int, B_ ^ 1>(), [&]() __attribute__((always_inline)) {
                    if (wave >= 4) issueP(std::integral_constant<int, B_>(), p + 2);
                    if (exch) c2_gather_look<FULL>(xs, K, C, lk);
                });
                // The F frame of the pair after the next goes into the registers this pair's F-step has
                // finished with; requested once the exchanged words are there, the requests pass the address
                // path while the words are added up.
                if (!exch) issueF(std::integral_constant<int, B_>(), p + 2);
                if (exch) {
                    c2_gather<FULL>(xs, K, C, tag, full_s, ctl_s, a.spin_limit, dead, lk,
                              [&]() __attribute__((always_inline)) { issueF(std::integral_constant<int, B_>(), p + 2); });
                    gstep += 1;
                    if (tP >= mid && wave == 6) {          // (a wave with no other special duty)
                        if (lane < g.nr) bh[(size_t)tP * C + g.r0 + lane] = full_s[g.r0 + lane];
                        if (lane == 0) Sb[(size_t)tP * kClMaxK + g.k] = ctl_s[0];
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
        __syncthreads();
        if (tid == 0 && ctl_s[11] && a.item_status && !bad) atomicMax(&a.item_status[b], (int)kItemRange);
        if (tid == 0) cluster_finish_item(a, b, ctl_s[8] != 0 || dead != 0, bad, 2 * a.K);
        __syncthreads();
    }
}

// FULL: a.K == kClMaxK, known when the kernel is chosen (no test per exchanged word)
template <bool GAMMA, bool ACC = false, bool FULL = false>
__global__ __launch_bounds__(kC2Threads) void cluster2_kernel(ClusterArgs a)
{
    __shared__ __align__(16) float smem[kC2Lds];
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
    if (GAMMA && !ACC) cluster_zero_padding(a, g);      // (adding leaves frames beyond the length alone)
    if (g.role == 0) alpha2_role<GAMMA, ACC, FULL>(a, g, smem, gstep, ptag);
    else beta2_role<GAMMA, ACC, FULL>(a, g, smem, gstep, ptag);
}

}  // namespace last
