// Forward recursions for a context dependency given as a next-state table
// (arXiv 2304.13134, Section 3: any deterministic automaton that accepts every
// label string may serve; the table form also covers full n-gram contexts of
// size 3 and more).  One workgroup per item.
//
// A table gives the arcs by SOURCE state, so Eq. 2 is evaluated by pushing:
// a group of G lanes reads one source row of the frame (contiguous weights,
// contiguous table entries) and combines each arc into its destination state
// in LDS.  The combination is made independent of the order in which arcs
// arrive, so results are reproducible run to run:
//   log semiring : pass 1 takes the per-destination maximum with an integer
//                  atomic max on an order-preserving key of the float; pass 2
//                  adds exp(v - max) as 24.40 fixed point with a 64-bit integer
//                  atomic add (at most 2^24 arcs per destination);
//   tropical     : one 64-bit atomic max on (score key, ~flat arc index), which
//                  is exactly "highest score, ties to the lowest flat index".
// Rescaling per frame and the float64 offsets are those of solo_forward_log.
#pragma once
#include "common.hpp"
#include "solo_kernels.hpp"

namespace last {

typedef unsigned long long tk_u64;

// order-preserving signed key of a float (for ds_max_i32); -0 is folded onto +0
__device__ __forceinline__ int tk_skey(float f)
{
    const int b = __float_as_int(f + 0.f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float tk_sval(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }

// order-preserving unsigned key (upper half of the tropical 64-bit key)
__device__ __forceinline__ unsigned tk_ukey(float f)
{
    const unsigned b = __float_as_uint(f + 0.f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float tk_uval(unsigned k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

constexpr float kTkFix = 1099511627776.f;        // 2^40
constexpr double kTkUnfix = 1.0 / 1099511627776.0;

// Every entry of the table must name a state; bad[0] is set otherwise and the
// kernels of the call then report kItemBadTable instead of indexing with it.
__global__ void table_check_kernel(const int* __restrict__ nx, int C, int V, int* __restrict__ bad)
{
    const size_t n = (size_t)C * V;
    int any = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        any |= ((unsigned)nx[i] >= (unsigned)C);
    if (any) atomicOr(bad, 1);
}

__global__ void table_clear_flag_kernel(int* __restrict__ bad) { bad[0] = 0; }

// Shortest distance in the log semiring (Section 2.1; Eq. 2), arcs by source state.
//   alpha_ws [B][T+1][C], offs [B][T+1], Dws [B] as in solo_forward_log (each may be null).
// LDS: sm u64[C] | cur float[C] | mk int[C] | red float[32].
template <int G>
__global__ __launch_bounds__(1024) void table_forward_log(
    const float* __restrict__ w, const int* __restrict__ len, Ctx c, int T,
    float* __restrict__ alpha_ws, double* __restrict__ offs, double* __restrict__ Dws,
    float* __restrict__ dist, int* __restrict__ item_status, const int* __restrict__ bad)
{
    extern __shared__ tk_u64 smem64[];
    tk_u64* sm = smem64;
    float* cur = (float*)(sm + c.C);
    int* mk = (int*)(cur + c.C);
    float* red = (float*)(mk + c.C);
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = len[b];
    const bool badtab = bad[0] != 0;
    if (L < 0 || L > T || badtab) {
        if (tid == 0) {
            if (item_status) item_status[b] = badtab ? kItemBadTable : kItemBadLength;
            dist[b] = __builtin_nanf("");
            if (Dws) Dws[b] = __builtin_nan("");
        }
        return;
    }
    if (tid == 0 && item_status) item_status[b] = kItemOk;
    const size_t fr = (size_t)c.C * c.V1;
    const int NR = blockDim.x / G, r = tid / G, l = tid - r * G;
    const int kneg = tk_skey(LAST_NEG_INF);
    float* al = alpha_ws ? alpha_ws + (size_t)b * (T + 1) * c.C : nullptr;
    for (int d = tid; d < c.C; d += blockDim.x) {
        const float v = d == 0 ? 0.f : LAST_NEG_INF;
        cur[d] = v;
        if (al) al[d] = v;
    }
    if (tid == 0 && offs) offs[(size_t)b * (T + 1)] = 0.0;
    double A = 0.0;
    __syncthreads();
    for (int t = 0; t < L; ++t) {
        const float* wt = w + ((size_t)b * T + t) * fr;
        for (int d = tid; d < c.C; d += blockDim.x) { mk[d] = kneg; sm[d] = 0; }
        __syncthreads();
        for (int q = r; q < c.C; q += NR) {
            const float a = cur[q];
            if (a == LAST_NEG_INF) continue;
            const float* row = wt + (size_t)q * c.V1;
            for (int y = l; y < c.V1; y += G) {
                const float v = a + row[y];
                if (v != LAST_NEG_INF) atomicMax(&mk[ctx_next(c, q, y)], tk_skey(v));
            }
        }
        __syncthreads();
        for (int q = r; q < c.C; q += NR) {
            const float a = cur[q];
            if (a == LAST_NEG_INF) continue;
            const float* row = wt + (size_t)q * c.V1;
            for (int y = l; y < c.V1; y += G) {
                const float v = a + row[y];
                if (v != LAST_NEG_INF) {
                    const int d = ctx_next(c, q, y);
                    atomicAdd(&sm[d], (tk_u64)(expf(v - tk_sval(mk[d])) * kTkFix));
                }
            }
        }
        __syncthreads();
        float mx = LAST_NEG_INF;
        for (int d = tid; d < c.C; d += blockDim.x) {
            const float m = tk_sval(mk[d]);
            const float v = (m == LAST_NEG_INF) ? LAST_NEG_INF
                                                : m + (float)log((double)sm[d] * kTkUnfix);
            mk[d] = __float_as_int(v);      // parked as raw bits until the maximum is known
            mx = fmaxf(mx, v);
        }
        mx = block_max(mx, red);
        if (mx == LAST_NEG_INF) mx = 0.f;
        A += (double)mx;
        for (int d = tid; d < c.C; d += blockDim.x) {
            const float v = __int_as_float(mk[d]) - mx;
            cur[d] = v;
            if (al) al[(size_t)(t + 1) * c.C + d] = v;
        }
        if (tid == 0 && offs) offs[(size_t)b * (T + 1) + t + 1] = A;
        __syncthreads();
    }
    float mx = LAST_NEG_INF;
    for (int d = tid; d < c.C; d += blockDim.x) mx = fmaxf(mx, cur[d]);
    mx = block_max(mx, red);
    float s = 0.f;
    if (mx != LAST_NEG_INF)
        for (int d = tid; d < c.C; d += blockDim.x) s += expf(cur[d] - mx);
    s = block_sum(s, red);
    if (tid == 0) {
        const double D = (mx == LAST_NEG_INF) ? (double)LAST_NEG_INF
                                              : A + (double)mx + (double)logf(s);
        dist[b] = (float)D;
        if (Dws) Dws[b] = D;
    }
}

// Tropical shortest distance with arg-max backpointers (Section 4.2.3), arcs by
// source state.  Same decisions as solo_viterbi: one float32 add per arc, ties to
// the lowest flat arc index q*(V+1)+y, final ties to the lowest state.
// LDS: key u64[C] | cur float[C] | redv float[32] | redi int[32].
template <int G>
__global__ __launch_bounds__(1024) void table_viterbi(
    const float* __restrict__ w, const int* __restrict__ len, Ctx c, int T,
    int* __restrict__ bp, int* __restrict__ final_state, float* __restrict__ score,
    int* __restrict__ item_status, const int* __restrict__ bad)
{
    extern __shared__ tk_u64 smem64[];
    tk_u64* key = smem64;
    float* cur = (float*)(key + c.C);
    float* redv = cur + c.C;
    int* redi = (int*)(redv + 32);
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = len[b];
    const bool badtab = bad[0] != 0;
    if (L < 0 || L > T || badtab) {
        if (tid == 0) {
            if (item_status) item_status[b] = badtab ? kItemBadTable : kItemBadLength;
            score[b] = __builtin_nanf("");
            if (final_state) final_state[b] = -1;
        }
        return;
    }
    if (tid == 0 && item_status) item_status[b] = kItemOk;
    const size_t fr = (size_t)c.C * c.V1;
    const int NR = blockDim.x / G, r = tid / G, l = tid - r * G;
    const tk_u64 knone = (tk_u64)tk_ukey(LAST_NEG_INF) << 32;
    for (int d = tid; d < c.C; d += blockDim.x) cur[d] = d == 0 ? 0.f : LAST_NEG_INF;
    __syncthreads();
    for (int t = 0; t < L; ++t) {
        const float* wt = w + ((size_t)b * T + t) * fr;
        for (int d = tid; d < c.C; d += blockDim.x) key[d] = knone;
        __syncthreads();
        for (int q = r; q < c.C; q += NR) {
            const float a = cur[q];
            if (a == LAST_NEG_INF) continue;
            const float* row = wt + (size_t)q * c.V1;
            for (int y = l; y < c.V1; y += G) {
                const float v = __fadd_rn(a, row[y]);
                if (v != LAST_NEG_INF) {
                    const unsigned flat = (unsigned)(q * c.V1 + y);
                    atomicMax(&key[ctx_next(c, q, y)], ((tk_u64)tk_ukey(v) << 32) | (0xFFFFFFFFu - flat));
                }
            }
        }
        __syncthreads();
        for (int d = tid; d < c.C; d += blockDim.x) {
            const tk_u64 k = key[d];
            const unsigned lo = (unsigned)k;
            cur[d] = lo == 0u ? LAST_NEG_INF : tk_uval((unsigned)(k >> 32));
            if (bp) bp[((size_t)b * T + t) * c.C + d] = lo == 0u ? -1 : (int)(0xFFFFFFFFu - lo);
        }
        __syncthreads();
    }
    float best = LAST_NEG_INF;
    int bidx = 0x7fffffff;
    for (int d = tid; d < c.C; d += blockDim.x)
        if (cur[d] > best || (cur[d] == best && d < bidx)) { best = cur[d]; bidx = d; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, kWave);
        const int oi = __shfl_xor(bidx, o, kWave);
        if (ov > best || (ov == best && oi < bidx)) { best = ov; bidx = oi; }
    }
    const int wid = tid / kWave, nw = blockDim.x / kWave;
    if ((tid & (kWave - 1)) == 0) { redv[wid] = best; redi[wid] = bidx; }
    __syncthreads();
    if (tid == 0) {
        for (int k = 1; k < nw; ++k)
            if (redv[k] > best || (redv[k] == best && redi[k] < bidx)) { best = redv[k]; bidx = redi[k]; }
        score[b] = best;
        if (final_state) final_state[b] = bidx;
    }
}

}  // namespace last
