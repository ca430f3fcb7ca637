// Clustered tropical recursion with arg-max backpointers for the full 1-gram context dependency with
// exactly 256 labels (C = 257 states; arXiv 2304.13134, Section 4.2.3 on the lattice of Sections 3 and
// 4.1): the shortest-path counterpart of cluster3_kernels.hpp, with that kernel's cut of the work.
//
// An item is walked forwards by K = 8 workgroups of eight waves on one XCD, frames in pairs with ONE
// exchange per pair (F-step: whole score vector -> own states, no communication; P-step: own states ->
// best arc out of an own state for every state, published and gathered).  Wave w of workgroup k
// ("sub-owner" u = 8 k + w) owns the four label states 1 + 4 u .. 4 + 4 u; the start state 0 is a fifth
// state of sub-owner 0.  Every weight is fetched with a 16-byte load by exactly one lane (see c3_geom
// and the access patterns at the top of cluster3_kernels.hpp): the address path of a compute unit takes
// a vector memory instruction lane by lane whatever its width, and the one-workgroup-wide reductions of
// the older kernel (one wave adding up 24 partial results per state) were most of its time.
//   * Candidates are one float32 add a[q] + w[q][y]; "highest score, then lowest flat arc index
//     q (V + 1) + y" is associative and commutative, so the split over lanes, waves and workgroups gives
//     bit for bit the scores and backpointers of the one-workgroup kernels.  Inside a lane candidates are
//     scanned in increasing arc order; between lanes, waves and workgroups (score, arc) pairs are combined.
//   * F-step: a lane scans four rows for each of its four columns; the eight lanes that share the columns
//     meet through one DPP shift and two lane swaps; the eight waves' results go through LDS (32 columns x
//     8 waves), and lane j < 4 of wave w combines those of its own state 4 w + j with the state's
//     empty-label arc and the start state's label arc.
//   * P-step: a lane scans the wave's own rows (five for sub-owner 0) for its four columns; the waves'
//     results go through LDS (8 x 256), thread y - 1 combines them for label state y and publishes
//     [score:32 | tag:15 | arc:17]; the start state's word is sent by thread 0.
//   * Gather: a quad of lanes shares two neighbouring states and splits the eight producers, two 16-byte
//     loads per lane, two DPP swaps; state 256 has its eight words on eight lanes.  The owner of a state
//     writes its backpointer.
//   * Weights travel two pairs ahead in three register sets; the requests leave right after the exchange
//     has been seen complete, because a wave's loads return in order and a look at the exchange must not
//     queue behind them.
// bp [B][T][C] (may be null): flat index of the best arc into state d at frame t, -1 if none.
#pragma once
#include "cluster2v_kernels.hpp"
#include "cluster3_kernels.hpp"

namespace last {

constexpr int kV3K = 8;                       // workgroups per item
constexpr int kV3C = kC3C;                    // 257 states
constexpr int kV3V1 = kC3C;                   // labels including the empty one (full 1-gram context: C = V + 1)
constexpr int kV3XS = kC3XS;                  // exchange words per producer and slot (257 used)

// LDS map (floats / ints)
constexpr int kV3Full = 0;                    // [272] scores of the whole vector, state q at q
constexpr int kV3RedV = kV3Full + 272;        // [32][8] F-step: best score per own column and wave
constexpr int kV3RedI = kV3RedV + 256;        // [32][8] ... and its arc
constexpr int kV3PaV = kV3RedI + 256;         // [8][256] P-step: best score per wave and label state
constexpr int kV3PaI = kV3PaV + 2048;         // [8][256]
constexpr int kV3BlV = kV3PaI + 2048;         // [8][8] empty-label candidates of the own states (per wave: 4 states, the start state)
constexpr int kV3BlI = kV3BlV + 64;           // [8][8]
constexpr int kV3OwnS = kV3BlI + 64;          // [8][8] scores of the own states after an F-step
constexpr int kV3Ctl = kV3OwnS + 64;          // [32] ints: [8] timeout
constexpr int kV3RedB = kV3Ctl + 32;          // [64] final reduction
constexpr int kV3Lds = kV3RedB + 64;
static_assert(kV3RedV % 4 == 0 && kV3RedI % 4 == 0 && kV3PaV % 4 == 0 && kV3PaI % 4 == 0, "16-byte LDS accesses");

// Combining (score, arc) candidates in two sweeps: first the highest score (one max per step), then, among
// the candidates that have it, the lowest arc (one min per step).  The result is the one of "higher score,
// then lower arc" applied pair by pair, at a fraction of the instructions.
//   arc of a candidate for the second sweep: its own if it has the best score, else none.  Every candidate
//   of score -inf carries the arc "none" (a scan never leaves its initial -inf for another -inf, published
//   words and the odd candidates are made so), which is why equal scores of -inf need no test of their own.
__device__ __forceinline__ int v3_keep(float v, int f, float best)
{
    return v == best ? f : kVNone;
}
// larger of two floats in one instruction (fmaxf costs one more per operand the compiler cannot prove
// quiet: values out of lane swaps, shifts and memory)
__device__ __forceinline__ float v3_fmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// maximum / minimum with the partner the two lane-swap instructions reach (rows of 16 lanes, halves of the wave)
__device__ __forceinline__ float v3_max_swap16(float v)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return v3_fmax(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float v3_max_swap32(float v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return v3_fmax(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ int v3_min_swap16(int f)
{
    const auto r = __builtin_amdgcn_permlane16_swap((unsigned)f, (unsigned)f, false, false);
    return min((int)r[0], (int)r[1]);
}
__device__ __forceinline__ int v3_min_swap32(int f)
{
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)f, (unsigned)f, false, false);
    return min((int)r[0], (int)r[1]);
}
// Four values per lane (one per column), to be combined over the wave's four rows of sixteen lanes, lane by
// lane: two columns share one swap (the odd rows of one against the even rows of the other), so that three
// swaps and three operations leave column r's result in row r, at the lane's place in the row.
__device__ __forceinline__ float v3_rows_max4(const float (&x)[4])
{
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x[0]), __float_as_uint(x[1]), false, false);
    const auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x[2]), __float_as_uint(x[3]), false, false);
    const float p = v3_fmax(__uint_as_float(a[0]), __uint_as_float(a[1]));      // rows: columns 0 1 0 1, of rows 0+1, 0+1, 2+3, 2+3
    const float q = v3_fmax(__uint_as_float(b[0]), __uint_as_float(b[1]));      //       columns 2 3 2 3
    const auto c = __builtin_amdgcn_permlane32_swap(__float_as_uint(p), __float_as_uint(q), false, false);
    return v3_fmax(__uint_as_float(c[0]), __uint_as_float(c[1]));               // rows: columns 0 1 2 3
}
__device__ __forceinline__ int v3_rows_min4(const int (&x)[4])
{
    const auto a = __builtin_amdgcn_permlane16_swap((unsigned)x[0], (unsigned)x[1], false, false);
    const auto b = __builtin_amdgcn_permlane16_swap((unsigned)x[2], (unsigned)x[3], false, false);
    const int p = min((int)a[0], (int)a[1]);
    const int q = min((int)b[0], (int)b[1]);
    const auto c = __builtin_amdgcn_permlane32_swap((unsigned)p, (unsigned)q, false, false);
    return min((int)c[0], (int)c[1]);
}
// ... and back: row r's value to every row, as column r's
__device__ __forceinline__ void v3_rows_spread4(float r, float (&m)[4])
{
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(r), __float_as_uint(r), false, false);   // rows 0 1 0 1 | 2 3 2 3
    const auto lo = __builtin_amdgcn_permlane16_swap(h[0], h[0], false, false);                               // rows 0 0 0 0 | 1 1 1 1
    const auto hi = __builtin_amdgcn_permlane16_swap(h[1], h[1], false, false);                               // rows 2 2 2 2 | 3 3 3 3
    m[0] = __uint_as_float(lo[0]);
    m[1] = __uint_as_float(lo[1]);
    m[2] = __uint_as_float(hi[0]);
    m[3] = __uint_as_float(hi[1]);
}
__device__ __forceinline__ float v3_word_score(unsigned lo) { return __uint_as_float(lo); }
__device__ __forceinline__ int v3_word_arc(unsigned hi) { return (int)(hi & 0x1FFFFu); }

// One exchange slot as a thread sees it (see C3Look): two neighbouring states from two of the eight
// producers, and one of the eight words of state 256.
__device__ __forceinline__ void v3_look(buf_t xrs, unsigned slot_off, unsigned voffq, unsigned voffz, C3Look& lk)
{
    lk.q[0] = c3_xload4(xrs, voffq, slot_off);
    lk.q[1] = c3_xload4(xrs, voffq, slot_off + (unsigned)(kV3XS * 8));
    lk.z = c3_xload2(xrs, voffz, slot_off);           // (lanes 0..7 of wave 0; out of range elsewhere)
}

// Gathering one exchange slot: the best of the eight published candidates of every state into full_s;
// the backpointer of the thread's state (lanes 0 and 1 of a quad: state 2 (tid / 4) + (tid & 1)) comes back
// in bp_q, that of state 256 (thread 0) in bp_z, -1 if there is none: the caller stores those of the states
// its workgroup owns, later, where a store is in nobody's way.  Every thread calls; ends with a workgroup
// barrier.  `after_poll` runs once all words are there.
template <typename AfterPoll>
__device__ __forceinline__ void v3_gather(buf_t xrs, unsigned slot_off, unsigned voffq, unsigned voffz, unsigned tag,
                                          float* full_s, int* ctl_s, int limit, int& dead, int& bp_q, int& bp_z,
                                          AfterPoll&& after_poll)
{
    const int tid = threadIdx.x;
    C3Look lk;
    v3_look(xrs, slot_off, voffq, voffz, lk);
    const unsigned tagw = (tag & 0x7FFFu) << 17;
    int n = 0;
    for (;;) {
        const unsigned zdiff = tid < 8 ? lk.z.y ^ tagw : 0u;
        const unsigned diff = zdiff | (lk.q[0].y ^ tagw) | (lk.q[0].w ^ tagw) | (lk.q[1].y ^ tagw) | (lk.q[1].w ^ tagw);
        if ((diff >> 17) == 0 || dead) break;
        if (++n > limit) { dead = 1; break; }
        __builtin_amdgcn_s_sleep(1);
        v3_look(xrs, slot_off, voffq, voffz, lk);
    }
    after_poll();
    // two producers of the two states of the quad, the other six through the quad's lanes (both swaps are
    // symmetric: every lane of the quad ends up with the same values)
    const float a0 = v3_word_score(lk.q[0].x), a1 = v3_word_score(lk.q[1].x);
    const float b0 = v3_word_score(lk.q[0].z), b1 = v3_word_score(lk.q[1].z);
    float vlo = v3_fmax(a0, a1), vhi = v3_fmax(b0, b1);
    vlo = v3_fmax(vlo, dpp_f<0xB1>(vlo, vlo));
    vhi = v3_fmax(vhi, dpp_f<0xB1>(vhi, vhi));
    vlo = v3_fmax(vlo, dpp_f<0x4E>(vlo, vlo));
    vhi = v3_fmax(vhi, dpp_f<0x4E>(vhi, vhi));
    int flo = min(v3_keep(a0, v3_word_arc(lk.q[0].y), vlo), v3_keep(a1, v3_word_arc(lk.q[1].y), vlo));
    int fhi = min(v3_keep(b0, v3_word_arc(lk.q[0].w), vhi), v3_keep(b1, v3_word_arc(lk.q[1].w), vhi));
    flo = min(flo, dpp_i<0xB1>(flo, flo));
    fhi = min(fhi, dpp_i<0xB1>(fhi, fhi));
    flo = min(flo, dpp_i<0x4E>(flo, flo));
    fhi = min(fhi, dpp_i<0x4E>(fhi, fhi));
    // state 256 (wave 0): lane l < 8 holds producer l's word; lanes 0..3 end up with the result
    const float wz = tid < 8 ? v3_word_score(lk.z.x) : LAST_NEG_INF;
    float vz = wz;
    int fz = kVNone;
    if (tid < 64) {
        vz = v3_fmax(vz, dpp_f<0xB1>(vz, vz));
        vz = v3_fmax(vz, dpp_f<0x4E>(vz, vz));
        vz = v3_fmax(vz, dpp_f<0x104>(LAST_NEG_INF, vz));                   // lanes 0..3 take lanes 4..7
        const float vzall = v3_fmax(vz, dpp_f<0x114>(LAST_NEG_INF, vz));    // ... and lanes 4..7 take lanes 0..3
        fz = tid < 8 ? v3_keep(wz, v3_word_arc(lk.z.y), vzall) : kVNone;
        fz = min(fz, dpp_i<0xB1>(fz, fz));
        fz = min(fz, dpp_i<0x4E>(fz, fz));
        fz = min(fz, dpp_i<0x104>(kVNone, fz));
        vz = vzall;
    }
    // lanes 0 and 1 of a quad write its two states
    if ((tid & 2) == 0) {
        const int s = 2 * (tid >> 2) + (tid & 1);
        const float v = (tid & 1) ? vhi : vlo;
        const int f = (tid & 1) ? fhi : flo;
        full_s[s] = dead ? LAST_NEG_INF : v;
        bp_q = (f == kVNone || dead) ? -1 : f;
    }
    if (tid == 0) {
        full_s[256] = dead ? LAST_NEG_INF : vz;
        bp_z = (fz == kVNone || dead) ? -1 : fz;
    }
    if (dead) ctl_s[8] = 1;
    c2_barrier();
}

template <bool BP>
__global__ __launch_bounds__(kC3Threads) void cluster3v_kernel(ClusterVArgs a)
{
    __shared__ __align__(16) float smem[kV3Lds];
    constexpr int C = kV3C, V1 = kV3V1;
    constexpr unsigned frb = (unsigned)C * C * 4u;
    float* full_s = smem + kV3Full;
    float* redv_s = smem + kV3RedV;
    int* redi_s = (int*)(smem + kV3RedI);
    float* pav_s = smem + kV3PaV;
    int* pai_s = (int*)(smem + kV3PaI);
    float* blv_s = smem + kV3BlV;
    int* bli_s = (int*)(smem + kV3BlI);
    float* own_s = smem + kV3OwnS;
    int* ctl_s = (int*)(smem + kV3Ctl);
    float* rbv_s = smem + kV3RedB;
    int* rbi_s = (int*)(smem + kV3RedB + 32);

    const int id = blockIdx.x;
    const int x = id & 7, slot = id >> 3;
    const int cl = slot / kV3K, k = slot - cl * kV3K;
    const int cg = x + 8 * cl;
    const int tid = threadIdx.x;
    const C3Geom g = c3_geom(k);
    const int lane = g.lane, wave = g.wave;
    // gather: quad <-> two neighbouring states, its lanes <-> two producers each
    const unsigned voffq = (unsigned)((2 * (tid & 3)) * kV3XS + 2 * (tid >> 2)) * 8u;
    const unsigned voffz = tid < 8 ? (unsigned)(tid * kV3XS + 256) * 8u : kC2Off;
    // publish: threads 0..255 <-> label states 1..256
    const unsigned voffpub = tid < 256 ? (unsigned)(k * kV3XS + tid + 1) * 8u : kC2Off;
    const int pcol = tid & 255;
    const bool pubown = (pcol >> 5) == k;
    const int pubbl = 8 * ((pcol & 31) >> 2) + (pcol & 3);
    unsigned gstep = 0;

    for (int b = cg; b < a.B; b += 8 * a.ncl) {
        int L = a.len[b];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        const int nlast = max(L - 1, 0);
        const size_t fr = (size_t)C * C;
        const buf_t wrs = make_buf(a.w + (size_t)b * a.T * fr, (unsigned)a.T * frb);
        const buf_t xrs = make_buf(a.xa + (size_t)cg * 2 * kV3K * kV3XS, (unsigned)(2 * kV3K * kV3XS * sizeof(u64)));
        int* bpi = BP ? a.bp + (size_t)b * a.T * C : nullptr;

        // start: score 0 at the start state, -inf elsewhere
        if (tid < 272) full_s[tid] = tid == 0 ? 0.f : LAST_NEG_INF;
        if (tid < 64) { own_s[tid] = LAST_NEG_INF; blv_s[tid] = LAST_NEG_INF; bli_s[tid] = kVNone; }
        if (tid < 32) ctl_s[tid] = 0;
        __syncthreads();

        C3Frame EF[3], EP[3];
        int dead = 0;
        auto issue = [&](auto BUF, int p) __attribute__((always_inline)) {
            constexpr int B_ = decltype(BUF)::value;
            c3_load_cols(EF[B_], wrs, g, (unsigned)min(2 * p, nlast) * frb);
            c3_load_rows(EP[B_], wrs, g, (unsigned)min(2 * p + 1, nlast) * frb);
        };
        issue(std::integral_constant<int, 0>(), 0);
        issue(std::integral_constant<int, 1>(), 1);

        int p = 0;
        float own = LAST_NEG_INF;      // lanes 0..3: the wave's own states, lane 4: the start state (sub-owner 0)
        // backpointers out of the last gather, stored behind the next publish (or when the item ends)
        const int gs = 2 * (tid >> 2) + (tid & 1);
        const bool gmine = (tid & 2) == 0 && (gs == 0 ? k == 0 : ((gs - 1) >> 5) == k);
        int pend_q = -1, pend_z = -1, pend_t = -1;
        auto store_pending = [&]() __attribute__((always_inline)) {
            if (BP && pend_t >= 0) {
                if (gmine) bpi[(size_t)pend_t * C + gs] = pend_q;
                if (tid == 0 && k == kV3K - 1) bpi[(size_t)pend_t * C + 256] = pend_z;
            }
            pend_t = -1;
        };
        auto pair = [&](auto BUF) __attribute__((always_inline)) -> bool {
            constexpr int B_ = decltype(BUF)::value;
            constexpr int B2_ = (B_ + 2) % 3;
            const int tF = 2 * p, tP = 2 * p + 1;
            if (tF >= L) return false;
            int fbp = kVNone;           // backpointer of the own state (lanes 0..3, lane 4: the start state's): stored behind the publish
            // ---------------- F-step: frame tF, all rows x own columns, from the whole vector
            {
                float best[4];
                int arc[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) { best[c] = LAST_NEG_INF; arc[c] = kVNone; }
                const int y0 = 1 + 32 * k + 4 * g.ci;
                const unsigned foF2 = (unsigned)min(2 * p + 4, nlast) * frb, foP2 = (unsigned)min(2 * p + 5, nlast) * frb;
#pragma unroll
                for (int j = 0; j < 4; ++j) {                  // (the row index increases with j)
                    const int q = 1 + 32 * wave + 8 * j + g.rg;
                    const float aq = full_s[q];
#pragma unroll
                    for (int c = 0; c < 4; ++c) v2_scan(__fadd_rn(aq, EF[B_].e[j][c]), q * V1 + y0 + c, best[c], arc[c]);
                    c3_load_cols_slot(EF[B2_], j, wrs, g, foF2);
                    if (j < 2) c3_load_rows_slot(EP[B2_], j, wrs, g, foP2);
                }
                c3_load_cols_slot(EF[B2_], 4, wrs, g, foF2);
                // the eight lanes with these columns: the two of a group of sixteen (a rotation by eight inside the
                // row, so both end up with the result), then the wave's four rows for all four columns at once
                float M[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) M[c] = v3_fmax(best[c], dpp_f<0x128>(best[c], best[c]));
                const float colmax = v3_rows_max4(M);          // row r: column r
                v3_rows_spread4(colmax, M);                    // every lane: all four columns
                int fk[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    fk[c] = v3_keep(best[c], arc[c], M[c]);
                    fk[c] = min(fk[c], dpp_i<0x128>(fk[c], fk[c]));
                }
                const int colarc = v3_rows_min4(fk);           // row r: column r
                if ((lane & 8) == 0) {
                    const int col = 4 * g.ci + (lane >> 4);
                    redv_s[col * 8 + wave] = colmax;
                    redi_s[col * 8 + wave] = colarc;
                }
                // odd elements: the empty-label arc of an own state (lanes 0..3; lane 4: the start state's) and
                // the start state's label arc into it (lanes 8..11, moved to lanes 0..3)
                const bool lo = lane < 4, l4 = lane == 4 && g.xR, l8 = lane >= 8 && lane < 12;
                const int ys = lo ? 1 + 4 * g.u + lane : (l8 ? 1 + 4 * g.u + lane - 8 : 0);     // the state the arc leads to
                const int qs = lo ? ys : 0;                                                    // ... and leaves
                const float mv = (g.mvC && (lo || l4 || l8)) ? __fadd_rn(full_s[qs], EF[B_].m) : LAST_NEG_INF;
                const int mf = mv > LAST_NEG_INF ? qs * V1 + (l8 ? ys : 0) : kVNone;
                const float sv = dpp_f<0x108>(LAST_NEG_INF, mv);      // lanes 0..7 take lanes 8..15
                const int sf = dpp_i<0x108>(kVNone, mf);
                c2_barrier();
                // own states: lane j < 4 combines the eight waves' results of column 4 wave + j
                float v = LAST_NEG_INF;
                int f = kVNone;
                if (lane < 4) {
                    const float4* rv = (const float4*)&redv_s[(4 * wave + lane) * 8];
                    const int4* ri = (const int4*)&redi_s[(4 * wave + lane) * 8];
                    const float4 v0 = rv[0], v1 = rv[1];
                    const int4 i0 = ri[0], i1 = ri[1];
                    v = c3_max3(c3_max3(v0.x, v0.y, v0.z), c3_max3(v0.w, v1.x, v1.y), c3_max3(v1.z, v1.w, v3_fmax(sv, mv)));
                    f = min(min(min(v3_keep(v0.x, i0.x, v), v3_keep(v0.y, i0.y, v)), min(v3_keep(v0.z, i0.z, v), v3_keep(v0.w, i0.w, v))),
                            min(min(v3_keep(v1.x, i1.x, v), v3_keep(v1.y, i1.y, v)), min(v3_keep(v1.z, i1.z, v), v3_keep(v1.w, i1.w, v))));
                    f = min(f, min(v3_keep(sv, sf, v), v3_keep(mv, mf, v)));
                } else if (l4) {
                    v = mv;
                    f = v3_keep(mv, mf, mv);
                }
                own = v;
                if (lane < 8) own_s[8 * wave + lane] = v;
                fbp = f;
            }
            auto store_fbp = [&]() __attribute__((always_inline)) {
                if (BP && (lane < 4 || (lane == 4 && g.xR))) bpi[(size_t)tF * C + (lane < 4 ? 1 + 4 * g.u + lane : 0)] = fbp == kVNone ? -1 : fbp;
            };
            if (tP >= L) { store_fbp(); store_pending(); return false; }
            // ---------------- P-step: frame tP, own rows x all columns, best candidate for every label state
            {
                const unsigned tag = gstep + 1;
                const unsigned slot_off = (gstep & 1) * (unsigned)(kV3K * kV3XS * sizeof(u64));
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(own), j));
                const float o0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(own), 4));
                float best[4];
                int arc[4];
                const int y0 = 1 + 4 * lane;
#pragma unroll
                for (int c = 0; c < 4; ++c) { best[c] = LAST_NEG_INF; arc[c] = kVNone; }
                if (g.xR) {                                    // (the start state's row comes first: lowest arcs)
#pragma unroll
                    for (int c = 0; c < 4; ++c) v2_scan(__fadd_rn(o0, EP[B_].x[c]), y0 + c, best[c], arc[c]);
                }
                const unsigned foP2 = (unsigned)min(2 * p + 5, nlast) * frb;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int q = 1 + 4 * g.u + j;
#pragma unroll
                    for (int c = 0; c < 4; ++c) v2_scan(__fadd_rn(o[j], EP[B_].e[j][c]), q * V1 + y0 + c, best[c], arc[c]);
                    if (j >= 1) c3_load_rows_slot(EP[B2_], j + 1, wrs, g, foP2);
                }
                float4 bv;
                int4 bi;
                bv.x = best[0]; bv.y = best[1]; bv.z = best[2]; bv.w = best[3];
                bi.x = arc[0]; bi.y = arc[1]; bi.z = arc[2]; bi.w = arc[3];
                *(float4*)&pav_s[wave * 256 + 4 * lane] = bv;
                *(int4*)&pai_s[wave * 256 + 4 * lane] = bi;
                // the empty label keeps the state: candidates of the own states (lane 4: the start state)
                if (lane < 8) {
                    const bool has = lane < 4 || (lane == 4 && g.xR);
                    const float cv = has ? __fadd_rn(own, EP[B_].m) : LAST_NEG_INF;
                    blv_s[8 * wave + lane] = cv;
                    bli_s[8 * wave + lane] = (has && cv > LAST_NEG_INF) ? (lane < 4 ? 1 + 4 * g.u + lane : 0) * V1 : kVNone;
                }
                c2_barrier();
                if (tid < 256) {
                    float cv[9];
#pragma unroll
                    for (int w2 = 0; w2 < 8; ++w2) cv[w2] = pav_s[256 * w2 + tid];
                    cv[8] = pubown ? blv_s[pubbl] : LAST_NEG_INF;
                    const float pv = c3_max3(c3_max3(cv[0], cv[1], cv[2]), c3_max3(cv[3], cv[4], cv[5]), c3_max3(cv[6], cv[7], cv[8]));
                    int pf = pubown ? v3_keep(cv[8], bli_s[pubbl], pv) : kVNone;
#pragma unroll
                    for (int w2 = 0; w2 < 8; ++w2) pf = min(pf, v3_keep(cv[w2], pai_s[256 * w2 + tid], pv));
                    c3_xstore(v2_pack(pv, tag, pf), xrs, voffpub, slot_off);
                    // the start state moves on by its empty-label arc only: workgroup 0 has it
                    if (tid == 0) {
                        const float zv = k == 0 ? blv_s[4] : LAST_NEG_INF;
                        c3_xstore(v2_pack(zv, tag, (k == 0 && zv > LAST_NEG_INF) ? 0 : kVNone), xrs,
                                  (unsigned)(k * kV3XS) * 8u, slot_off);
                    }
                }
                store_fbp();
                store_pending();
                v3_gather(xrs, slot_off, voffq, voffz, tag, full_s, ctl_s, a.spin_limit, dead, pend_q, pend_z, [] {});
                pend_t = tP;
                gstep += 1;
            }
            ++p;
            return true;
        };
        for (;;) {
            if (!pair(std::integral_constant<int, 0>())) break;
            if (!pair(std::integral_constant<int, 1>())) break;
            if (!pair(std::integral_constant<int, 2>())) break;
        }
        store_pending();
        __syncthreads();
        if (L & 1) {
            // the last frame was an F-step: the own scores of every workgroup make up the final vector
            const unsigned tag = gstep + 1;
            const unsigned slot_off = (gstep & 1) * (unsigned)(kV3K * kV3XS * sizeof(u64));
            if (tid < 256) {
                c3_xstore(v2_pack(pubown ? own_s[pubbl] : LAST_NEG_INF, tag, kVNone), xrs, voffpub, slot_off);
                if (tid == 0) c3_xstore(v2_pack(k == 0 ? own_s[4] : LAST_NEG_INF, tag, kVNone), xrs, (unsigned)(k * kV3XS) * 8u, slot_off);
            }
            int unused_q = -1, unused_z = -1;
            v3_gather(xrs, slot_off, voffq, voffz, tag, full_s, ctl_s, a.spin_limit, dead, unused_q, unused_z, [] {});
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
                for (int w2 = 1; w2 < kC3Waves; ++w2)
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
            if (old == (u64)(kV3K - 2)) {
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
