// Clustered tropical recursion with arg-max backpointers for the full 1-gram context
// dependency (arXiv 2304.13134, Section 4.2.3 on the lattice of Sections 3 and 4.1): the
// shortest-path counterpart of cluster2_kernels.hpp.
//
// An item is walked forwards by K persistent workgroups on one XCD; workgroup k owns states
// [k*RPW, (k+1)*RPW).  Frames are taken in pairs with ONE exchange per pair, exactly as in the
// log-semiring kernel:
//   F-step: from the whole score vector every workgroup computes the scores and backpointers of
//           its OWN states of the next frame (all rows x own columns), no communication;
//   P-step: from its own states it computes, for ALL states of the frame after, the best arc
//           leaving an own state (own rows x all columns), publishes (score, arc) per state, and
//           every workgroup takes the best over the K published candidates.
// There is no rescaling and no exp: a candidate is one float32 add a[q] + w[q][y], comparisons are
// exact, ties go to the lowest flat arc index q*(V+1)+y.  (max, then lowest index) is associative
// and commutative, so splitting the candidates of a state over lanes, waves and workgroups gives
// bit for bit the scores and backpointers of the one-workgroup kernels (solo_viterbi).
//
// Exchange word: [score:32 | tag:15 | arc:17]; arc = 0x1FFFF means "no finite candidate".
// bp [B][T][C] (may be null): flat index of the best arc into state d at frame t, -1 if none.
#pragma once
#include "cluster2_kernels.hpp"

namespace last {

struct ClusterVArgs {
    const float* w;
    const int* len;
    int* bp;
    int* final_state;
    float* score;
    int* item_status;
    u64* xa;
    u64* fin;            // [B][2], cleared to ~0: workgroups through with the item, time-out mark
    int B, T, C, K, RPW, ncl;
    int spin_limit;
};

constexpr int kVNone = 0x1FFFF;

// LDS map (floats / ints)
constexpr int kV2Full = 0;                              // [320] scores of the whole vector
constexpr int kV2Own = kV2Full + 320;                   // [40] scores of the own states
constexpr int kV2RedV = kV2Own + kC2Own;                // [24][40] F-step: best score per wave and row group
constexpr int kV2RedI = kV2RedV + kC2RedN * kC2Own;     // [24][40] ... and its arc
constexpr int kV2BlV = kV2RedI + kC2RedN * kC2Own;      // [40] P-step: empty-label candidates of the own states
constexpr int kV2BlI = kV2BlV + kC2Own;                 // [40]
constexpr int kV2PaV = kV2BlI + kC2Own;                 // [320] P-step: second half of the own rows
constexpr int kV2PaI = kV2PaV + 320;                    // [320]
constexpr int kV2StV = kV2PaI + 320;                    // [8] P-step: columns beyond 256
constexpr int kV2StI = kV2StV + 8;                      // [8]
constexpr int kV2Ctl = kV2StI + 8;                      // [32] ints: [8] timeout
constexpr int kV2RedB = kV2Ctl + 32;                    // [64] final reduction
constexpr int kV2Lds = kV2RedB + 64;
static_assert(kV2RedV % 2 == 0 && kV2RedI % 2 == 0, "8-byte LDS accesses");

// same rule as trop_acc, with the 17-bit "none" as the starting arc
__device__ __forceinline__ void v2_acc(float v, int flat, float& best, int& bflat)
{
    if (v > best || (v == best && v != LAST_NEG_INF && flat < bflat)) { best = v; bflat = flat; }
}

__device__ __forceinline__ u64 v2_pack(float v, unsigned tag, int flat)
{
    return (u64)__float_as_uint(v) | ((u64)(((tag & 0x7FFFu) << 17) | ((unsigned)flat & 0x1FFFFu)) << 32);
}

// Many candidates at once, in two sweeps: the highest score first (one max per candidate), then the lowest
// arc among the candidates that have it (one min per candidate) -- what v2_acc gives pair by pair, at a
// third of the instructions and without its chain of dependent selects.
__device__ __forceinline__ int v2_keep(float v, int flat, float best)
{
    return (v == best && v != LAST_NEG_INF) ? flat : kVNone;
}

// The same inside one thread's scan, whose candidates come in increasing arc order: a tie keeps the
// earlier, lower arc, and a candidate of -inf never beats the initial -inf.
__device__ __forceinline__ void v2_scan(float v, int flat, float& best, int& bflat)
{
    const bool up = v > best;
    best = up ? v : best;
    bflat = up ? flat : bflat;
}

// best (score, arc) of a wave, in every lane
__device__ __forceinline__ void v2_wave_best(float& v, int& f)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64);
        const int of = __shfl_xor(f, o, 64);
        v2_acc(ov, of, v, f);
    }
}

// Gather one exchange slot: best of the K published candidates per state.  Every thread calls;
// ends with a workgroup barrier.  Returns the winning arc of state tid (kVNone if none).
// FULL: K is the largest number of producers, known when the kernel is chosen (no test per word).
template <bool FULL>
__device__ __forceinline__ int v2_gather(const u64* xs, int K, int C, unsigned tag, float* full_s,
                                         int* ctl_s, int limit, int& dead)
{
    const int tid = threadIdx.x;
    int bf = kVNone;
    if (tid < C) {
        u64 wv[kClMaxK];
        int n = 0;
        for (;;) {
#pragma unroll
            for (int kk = 0; kk < kClMaxK; ++kk)
                if (FULL || kk < K) wv[kk] = xload(xs + (size_t)kk * kC2XS + tid);
            // all K tags right: no bit differs in the tag fields (the upper 15 bits of the words)
            const unsigned tagw = (tag & 0x7FFFu) << 17;
            unsigned diff = 0;
#pragma unroll
            for (int kk = 0; kk < kClMaxK; ++kk)
                if (FULL || kk < K) diff |= (unsigned)(wv[kk] >> 32) ^ tagw;
            const bool ok = (diff >> 17) == 0;
            if (ok || dead) break;
            if (++n > limit) { dead = 1; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        float best = LAST_NEG_INF;
#pragma unroll
        for (int kk = 0; kk < kClMaxK; ++kk)
            if (FULL || kk < K) best = fmaxf(best, __uint_as_float((unsigned)wv[kk]));
#pragma unroll
        for (int kk = 0; kk < kClMaxK; ++kk)
            if (FULL || kk < K) bf = min(bf, v2_keep(__uint_as_float((unsigned)wv[kk]), (int)((wv[kk] >> 32) & 0x1FFFFu), best));
        full_s[tid] = dead ? LAST_NEG_INF : best;
    }
    if (dead) ctl_s[8] = 1;
    c2_barrier();
    return bf;
}

template <bool BP, bool FULL = false>
__global__ __launch_bounds__(kC2Threads) void cluster2v_kernel(ClusterVArgs a)
{
    __shared__ __align__(16) float smem[kV2Lds];
    float* full_s = smem + kV2Full;
    float* own_s = smem + kV2Own;
    float* redv_s = smem + kV2RedV;
    int* redi_s = (int*)(smem + kV2RedI);
    float* blv_s = smem + kV2BlV;
    int* bli_s = (int*)(smem + kV2BlI);
    float* pav_s = smem + kV2PaV;
    int* pai_s = (int*)(smem + kV2PaI);
    float* stv_s = smem + kV2StV;
    int* sti_s = (int*)(smem + kV2StI);
    int* ctl_s = (int*)(smem + kV2Ctl);
    float* rbv_s = smem + kV2RedB;
    int* rbi_s = (int*)(smem + kV2RedB + 32);

    const int id = blockIdx.x;
    const int x = id & 7, slot = id >> 3;
    const int cl = slot / a.K, k = slot - cl * a.K;
    const int cg = x + 8 * cl;
    const int C = a.C, K = a.K, V1 = a.C;          // full 1-gram context: C = V + 1
    int r0 = k * a.RPW;
    int nr = min(a.RPW, C - r0);
    if (nr < 0) nr = 0;
    if (r0 > C) r0 = C;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // P-step: thread <-> column cP = 64 (wave & 3) + lane and half hP = wave >> 2 of the own rows;
    // straggler column 256 + sS on wave 7 - sS, lane <-> own row
    const int hP = wave >> 2;
    const int cP = ((wave & 3) << 6) + lane;
    const bool colok = cP < C;
    const int rP0 = kC2PH * hP;
    const int nst = max(C - kC2PC, 0);
    const int sS = kC2Waves - 1 - wave;
    const bool hasS = sS < nst;
    const int cS = kC2PC + sS;
    // F-step: wave <-> rows [33 wave, 33 wave + 33), three groups of 17 lanes take every third row,
    // a lane two neighbouring own columns
    const int gq = lane / 17, ci = lane - 17 * gq;
    const bool lact = lane < 17 * kC2FG && 2 * ci < nr;
    const bool v0ok = lact && r0 + 2 * ci != 0;      // state 0 receives no label arcs
    const bool v1ok = lact && 2 * ci + 1 < nr;
    const int qF0 = kC2NQ * wave + gq;
    const int slotF = (wave * kC2FG + min(gq, kC2FG - 1)) * kC2Own + 2 * ci;
    const bool fok = lane < nr;                       // wave 0: lane <-> own state
    const int yF = min(r0 + lane, C - 1);
    unsigned gstep = 0;

    for (int b = cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const size_t fr = (size_t)C * C;
        const unsigned frb = (unsigned)(fr * sizeof(float));
        const unsigned pitch = (unsigned)(C * (int)sizeof(float));
        u64* xbase = a.xa + (size_t)cg * 2 * kClMaxK * kC2XS;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        int* bpi = BP ? a.bp + (size_t)b * a.T * C : nullptr;
        const unsigned coffPm = colok ? (unsigned)(cP * (int)sizeof(float)) : kC2Off;
        const unsigned coffS = lane < nr ? (unsigned)lane * pitch + (unsigned)(cS * (int)sizeof(float)) : kC2Off;
        const unsigned rbaseP = (unsigned)r0 * pitch;
        const unsigned rowB = (unsigned)yF * pitch;                  // row of the own state (empty-label weight)
        const int nlast = max(L - 1, 0);
        // F loads: a row beyond the matrix repeats the last one (its score is -inf), a lane without own
        // columns repeats the address of one that has some (its result is discarded)
        const int gqa = min(gq, kC2FG - 1), cia = min(gq < kC2FG ? ci : 16, max(nr - 1, 0) / 2);
        const unsigned cola = (unsigned)((r0 + 2 * cia) * (int)sizeof(float));
        const unsigned offA0 = (unsigned)(kC2NQ * wave + gqa) * pitch + cola;
        const unsigned offAL = (unsigned)(C - 1) * pitch + cola;
        const int jla = max((C - (kC2NQ * wave + gqa) + kC2FG - 1) / kC2FG, 0);

        // start: score 0 at the start state, -inf elsewhere (and beyond the last state)
        for (int q = tid; q < 320; q += kC2Threads) full_s[q] = q == 0 ? 0.f : LAST_NEG_INF;
        if (tid < kC2Own) own_s[tid] = LAST_NEG_INF;
        if (tid < 32) ctl_s[tid] = 0;
        __syncthreads();

        float EF0[2][kC2FJ], EF1[2][kC2FJ], EP[2][kC2PH];
        float EB[2] = {0.f, 0.f}, ES[2] = {0.f, 0.f}, EBP[2] = {0.f, 0.f};
        int dead = 0;

        auto issueF = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned foF = (unsigned)min(2 * p, nlast) * frb;
            int jl = jla;
            c2_pin(jl);          // offsets are made where they are used, not kept in registers
#pragma unroll
            for (int j = 0; j < kC2FJ; ++j) {
                const float2 v = buf_load2(wrs, j < jl ? offA0 + (unsigned)(kC2FG * j) * pitch : offAL, foF);
                EF0[B_][j] = v.x;
                EF1[B_][j] = v.y;
            }
            if (wave == 0) EB[B_] = buf_load(wrs, fok ? rowB : kC2Off, foF);
        };
        auto issueP = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            const unsigned foP = (unsigned)min(2 * p + 1, nlast) * frb;
#pragma unroll
            for (int r = 0; r < kC2PH; ++r)
                EP[B_][r] = buf_load(wrs, coffPm, foP + rbaseP + (unsigned)min(rP0 + r, max(nr - 1, 0)) * pitch);
            if (hasS) ES[B_] = buf_load(wrs, coffS, foP + rbaseP);
            if (wave == 0) EBP[B_] = buf_load(wrs, fok ? rowB : kC2Off, foP);
        };

        issueF(std::integral_constant<int, 0>(), 0);
        issueP(std::integral_constant<int, 0>(), 0);

        int p = 0;
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value;
            const int tF = 2 * p, tP = 2 * p + 1;
            if (tF >= L) return false;
            // ---------------- F-step: frame tF, all rows x own columns, from the whole vector
            {
                float b0 = LAST_NEG_INF, b1 = LAST_NEG_INF;
                int f0 = kVNone, f1 = kVNone;
                const int y0 = r0 + 2 * ci;
#pragma unroll
                for (int j = 0; j < kC2FJ; ++j) {
                    const int q = qF0 + kC2FG * j;
                    const float aq = full_s[min(q, 319)];            // -inf beyond the last state
                    v2_scan(__fadd_rn(aq, EF0[B_][j]), q * V1 + y0, b0, f0);         // (q increases with j)
                    v2_scan(__fadd_rn(aq, EF1[B_][j]), q * V1 + y0 + 1, b1, f1);
                }
                if (!v0ok) { b0 = LAST_NEG_INF; f0 = kVNone; }
                if (!v1ok) { b1 = LAST_NEG_INF; f1 = kVNone; }
                if (lane < 17 * kC2FG) {
                    float2 pv; int2 pi;
                    pv.x = b0; pv.y = b1; pi.x = f0; pi.y = f1;
                    *(float2*)&redv_s[slotF] = pv;
                    *(int2*)&redi_s[slotF] = pi;
                }
                issueF(std::integral_constant<int, B_ ^ 1>(), p + 1);
                c2_barrier();
                if (wave == 0) {
                    float best = LAST_NEG_INF;
                    int bf = kVNone;
                    if (fok) {
                        float rv[kC2RedN];
#pragma unroll
                        for (int x2 = 0; x2 < kC2RedN; ++x2) rv[x2] = redv_s[x2 * kC2Own + lane];
                        // the empty label keeps the state
                        const float ev = __fadd_rn(full_s[yF], EB[B_]);
                        best = ev;
#pragma unroll
                        for (int x2 = 0; x2 < kC2RedN; ++x2) best = fmaxf(best, rv[x2]);
                        bf = v2_keep(ev, yF * V1, best);
#pragma unroll
                        for (int x2 = 0; x2 < kC2RedN; ++x2) bf = min(bf, v2_keep(rv[x2], redi_s[x2 * kC2Own + lane], best));
                        if (BP) bpi[(size_t)tF * C + r0 + lane] = bf == kVNone ? -1 : bf;
                    }
                    if (lane < kC2Own) own_s[lane] = best;
                }
                c2_barrier();
            }
            if (tP >= L) return false;
            // ---------------- P-step: frame tP, own rows x all columns, best candidate for every state
            {
                const unsigned tag = gstep + 1;
                u64* xs = xbase + (size_t)(gstep & 1) * kClMaxK * kC2XS;
                float bv = LAST_NEG_INF;
                int bfv = kVNone;
#pragma unroll
                for (int r = 0; r < kC2PH; ++r)      // (rows beyond the own ones have score -inf)
                    v2_scan(__fadd_rn(own_s[rP0 + r], EP[B_][r]), (r0 + rP0 + r) * V1 + cP, bv, bfv);
                if (!colok || cP == 0) { bv = LAST_NEG_INF; bfv = kVNone; }     // column 0 is the empty label
                if (wave == 0 && lane < kC2Own) {
                    // the empty label keeps the state: candidates of the own states, lane <-> state
                    blv_s[lane] = fok ? __fadd_rn(own_s[lane], EBP[B_]) : LAST_NEG_INF;
                    bli_s[lane] = (r0 + lane) * V1;
                }
                if (hP == 1) { pav_s[cP] = bv; pai_s[cP] = bfv; }
                if (hasS) {
                    float sv = lane < nr ? __fadd_rn(own_s[lane], ES[B_]) : LAST_NEG_INF;
                    int sf = (r0 + lane) * V1 + cS;
                    if (!(sv > LAST_NEG_INF)) { sv = LAST_NEG_INF; sf = kVNone; }
                    v2_wave_best(sv, sf);
                    if (lane == 0) { stv_s[sS] = sv; sti_s[sS] = sf; }
                }
                issueP(std::integral_constant<int, B_ ^ 1>(), p + 1);
                c2_barrier();
                if (tid < C) {
                    // threads 0..255 are the first halves of their columns; 256.. publish the stragglers
                    float pv = LAST_NEG_INF;
                    int pf = kVNone;
                    if (tid < kC2PC) {
                        pv = bv; pf = bfv;
                        v2_acc(pav_s[tid], pai_s[tid], pv, pf);
                    } else {
                        v2_acc(stv_s[tid - kC2PC], sti_s[tid - kC2PC], pv, pf);
                    }
                    if (tid >= r0 && tid < r0 + nr) v2_acc(blv_s[tid - r0], bli_s[tid - r0], pv, pf);
                    xpublish(xs + (size_t)k * kC2XS + tid, v2_pack(pv, tag, pf));
                }
                const int bf = v2_gather<FULL>(xs, K, C, tag, full_s, ctl_s, a.spin_limit, dead);
                gstep += 1;
                if (BP && tid >= r0 && tid < r0 + nr) bpi[(size_t)tP * C + tid] = bf == kVNone ? -1 : bf;
            }
            ++p;
            return true;
        };
        for (;;) {
            if (!pair(std::integral_constant<int, 0>())) break;
            if (!pair(std::integral_constant<int, 1>())) break;
        }
        __syncthreads();
        if (L & 1) {
            // the last frame was an F-step: the own scores of every workgroup make up the final vector
            const unsigned tag = gstep + 1;
            u64* xs = xbase + (size_t)(gstep & 1) * kClMaxK * kC2XS;
            if (tid < C) {
                const bool own = tid >= r0 && tid < r0 + nr;
                xpublish(xs + (size_t)k * kC2XS + tid, v2_pack(own ? own_s[tid - r0] : LAST_NEG_INF, tag, kVNone));
            }
            v2_gather<FULL>(xs, K, C, tag, full_s, ctl_s, a.spin_limit, dead);
            gstep += 1;
        }
        // best final state, lowest index among equals (every workgroup has the whole vector; the first writes)
        if (k == 0) {
            float best = tid < C ? full_s[tid] : LAST_NEG_INF;
            int bidx = tid < C ? tid : 0x7fffffff;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(best, o, 64);
                const int oi = __shfl_xor(bidx, o, 64);
                if (ov > best || (ov == best && oi < bidx)) { best = ov; bidx = oi; }
            }
            if (lane == 0) { rbv_s[wave] = best; rbi_s[wave] = bidx; }
            __syncthreads();
            if (tid == 0) {
                for (int w2 = 1; w2 < kC2Waves; ++w2)
                    if (rbv_s[w2] > best || (rbv_s[w2] == best && rbi_s[w2] < bidx)) { best = rbv_s[w2]; bidx = rbi_s[w2]; }
                const bool tmo = ctl_s[8] != 0 || dead;
                a.score[b] = (bad || tmo) ? __builtin_nanf("") : best;
                if (a.final_state) a.final_state[b] = (bad || tmo) ? -1 : bidx;
                if (a.item_status) a.item_status[b] = bad ? kItemBadLength : (tmo ? kItemTimeout : kItemOk);
            }
        }
        __syncthreads();
        // a time-out of any workgroup voids the item: the last workgroup through looks at the mark
        if (tid == 0) {
            u64* fin = a.fin + (size_t)b * 2;
            if (ctl_s[8] != 0 || dead) __hip_atomic_store(fin + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __threadfence();
            const u64 old = __hip_atomic_fetch_add(fin, 1ull, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            if (old == (u64)(K - 2)) {
                __threadfence();
                if (__hip_atomic_load(fin + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != ~0ull && !bad) {
                    __hip_atomic_store(a.score + b, __builtin_nanf(""), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (a.final_state)
                        __hip_atomic_store(a.final_state + b, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (a.item_status)
                        __hip_atomic_store(a.item_status + b, (int)kItemTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace last
