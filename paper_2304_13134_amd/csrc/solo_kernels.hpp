// One-workgroup-per-item kernels: the general, range-robust path (any context
// order, any vocabulary size).  Everything is kept in the log domain with
// per-destination maxima, and the state vector of the current frame lives in
// LDS for the whole recursion (Eq. 2 of arXiv 2304.13134 visited frame by
// frame, Section 4.1).  States are rescaled per frame, alpha~_t = alpha_t - A_t,
// with the scalar offsets A_t accumulated in float64, so that every float32
// quantity stays O(10) although log-partition values reach several thousand.
#pragma once
#include "common.hpp"

namespace last {

__device__ __forceinline__ void lse_acc(float v, float& m, float& s)
{
    if (v == LAST_NEG_INF) return;
    if (v > m) {
        s = s * expf(m - v) + 1.f;   // m = -inf: s is still 0 and exp(-inf) = 0
        m = v;
    } else {
        s += expf(v - m);
    }
}

// Thread layout of the forward kernels: the workgroup is viewed as R groups of
// CPAD threads; thread (g, dl) accumulates, for destination state d0 + dl, the
// incoming label arcs i = g, g + R, ...; group 0 also takes the empty-label arc.
// Lanes are adjacent destinations, so for a fixed source row the loads are
// contiguous.

// Shortest distance in the log semiring (Section 2.1; Eq. 2).
//   alpha_ws [B][T+1][C] rescaled forward weights (may be null: not stored)
//   offs     [B][T+1]    A_t (may be null)
//   Dws      [B]         D in float64 (may be null);  dist [B] float32
__global__ __launch_bounds__(1024) void solo_forward_log(
    const float* __restrict__ w, const int* __restrict__ len, Ctx c, int T, int CPAD, int R,
    float* __restrict__ alpha_ws, double* __restrict__ offs, double* __restrict__ Dws,
    float* __restrict__ dist, int* __restrict__ item_status)
{
    extern __shared__ float smem[];
    float* cur = smem;
    float* nxt = cur + c.C;
    float* pm = nxt + c.C;
    float* ps = pm + R * CPAD;
    float* red = ps + R * CPAD;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = len[b];
    if (L < 0 || L > T) {
        if (tid == 0) {
            if (item_status) item_status[b] = kItemBadLength;
            dist[b] = __builtin_nanf("");
            if (Dws) Dws[b] = __builtin_nan("");
        }
        return;
    }
    if (tid == 0 && item_status) item_status[b] = kItemOk;
    const int g = tid / CPAD, dl = tid - g * CPAD;
    const size_t fr = (size_t)c.C * c.V1;
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
        for (int d0 = 0; d0 < c.C; d0 += CPAD) {
            const int d = d0 + dl;
            if (g < R && d < c.C) {
                float m = LAST_NEG_INF, s = 0.f;
                const int n = ctx_num_in(c, d);
                const int y = d > 0 ? ctx_in_label(c, d) : 0;
                for (int i = g; i < n; i += R) {
                    const int q = ctx_in_source(c, d, i);
                    lse_acc(cur[q] + wt[(size_t)q * c.V1 + y], m, s);
                }
                if (g == 0) lse_acc(cur[d] + wt[(size_t)d * c.V1], m, s);
                pm[g * CPAD + dl] = m;
                ps[g * CPAD + dl] = s;
            }
            __syncthreads();
            if (g == 0 && d < c.C) {
                float M = LAST_NEG_INF;
                for (int k = 0; k < R; ++k) M = fmaxf(M, pm[k * CPAD + dl]);
                float S = 0.f;
                if (M != LAST_NEG_INF)
                    for (int k = 0; k < R; ++k) {
                        const float mk = pm[k * CPAD + dl];
                        if (mk != LAST_NEG_INF) S += ps[k * CPAD + dl] * expf(mk - M);
                    }
                nxt[d] = (M == LAST_NEG_INF) ? LAST_NEG_INF : M + logf(S);
            }
            __syncthreads();
        }
        float mx = LAST_NEG_INF;
        for (int d = tid; d < c.C; d += blockDim.x) mx = fmaxf(mx, nxt[d]);
        mx = block_max(mx, red);
        if (mx == LAST_NEG_INF) mx = 0.f;   // no state reachable: keep -inf everywhere
        A += (double)mx;
        for (int d = tid; d < c.C; d += blockDim.x) {
            const float v = nxt[d] - mx;
            cur[d] = v;
            if (al) al[(size_t)(t + 1) * c.C + d] = v;
        }
        if (tid == 0 && offs) offs[(size_t)b * (T + 1) + t + 1] = A;
        __syncthreads();
    }
    // all states of the last frame are final with weight 0
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

// Backward weights and arc marginals (Eq. 1; Section 4.2.2).  A group of G
// lanes owns one source state (a row of the frame, contiguous in memory) and
// strides over its V+1 arcs.  gamma = exp(alpha~_t[q] + w + beta~_{t+1}[next]
// + (A_t + B_{t+1} - D)), the bracket formed in float64.
template <int G>
__global__ __launch_bounds__(1024) void solo_backward_log(
    const float* __restrict__ w, const int* __restrict__ len, Ctx c, int T,
    const float* __restrict__ alpha_ws, const double* __restrict__ offs,
    const double* __restrict__ Dws, float* __restrict__ dw, float scale, int accumulate)
{
    extern __shared__ float smem[];
    float* bn = smem;          // beta~_{t+1}
    float* bc = bn + c.C;      // beta_t before rescaling
    float* red = bc + c.C;
    const int b = blockIdx.x, tid = threadIdx.x;
    const size_t fr = (size_t)c.C * c.V1;
    float* gw = dw + (size_t)b * T * fr;
    int L = len[b];
    const bool bad = (L < 0 || L > T);
    if (bad) L = 0;
    if (!accumulate)
        for (size_t i = (size_t)L * fr + tid; i < (size_t)T * fr; i += blockDim.x) gw[i] = 0.f;
    if (bad) return;
    for (int d = tid; d < c.C; d += blockDim.x) bn[d] = 0.f;
    const double D = Dws[b];
    double Boff = 0.0;
    const int NR = blockDim.x / G, r = tid / G, l = tid - r * G;
    __syncthreads();
    for (int t = L - 1; t >= 0; --t) {
        const float* wt = w + ((size_t)b * T + t) * fr;
        float* gt = gw + (size_t)t * fr;
        const float* at = alpha_ws + ((size_t)b * (T + 1) + t) * c.C;
        const float K = (float)(offs[(size_t)b * (T + 1) + t] + Boff - D);
        for (int q0 = 0; q0 < c.C; q0 += NR) {
            const int q = q0 + r;
            const bool valid = q < c.C;
            const float* row = wt + (size_t)q * c.V1;
            float m = LAST_NEG_INF;
            if (valid)
                for (int y = l; y < c.V1; y += G) m = fmaxf(m, row[y] + bn[ctx_next(c, q, y)]);
            m = group_max<G>(m);
            float s = 0.f;
            if (valid && m != LAST_NEG_INF)
                for (int y = l; y < c.V1; y += G) s += expf(row[y] + bn[ctx_next(c, q, y)] - m);
            s = group_sum<G>(s);
            if (valid) {
                if (l == 0) bc[q] = (m == LAST_NEG_INF) ? LAST_NEG_INF : m + logf(s);
                const float a = at[q];
                float* grow = gt + (size_t)q * c.V1;
                for (int y = l; y < c.V1; y += G) {
                    float p = 0.f;
                    if (a != LAST_NEG_INF) p = scale * expf(row[y] + bn[ctx_next(c, q, y)] + a + K);
                    if (accumulate) grow[y] += p; else grow[y] = p;
                }
            }
        }
        __syncthreads();
        float mx = LAST_NEG_INF;
        for (int d = tid; d < c.C; d += blockDim.x) mx = fmaxf(mx, bc[d]);
        mx = block_max(mx, red);
        if (mx == LAST_NEG_INF) mx = 0.f;
        Boff += (double)mx;
        for (int d = tid; d < c.C; d += blockDim.x) bn[d] = bc[d] - mx;
        __syncthreads();
    }
}

// zero the gradient of items whose length is invalid (used by the clustered path too)
// workgroup barrier that orders LDS traffic only: global loads issued before it stay in flight
__device__ __forceinline__ void lds_only_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__global__ void zero_fill_kernel(float* __restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0.f;
}

// Tropical shortest distance with arg-max backpointers (Section 4.2.3): one
// float32 add per arc, exact comparisons, no rescaling.  Ties: lowest flat arc
// index q*(V+1)+y.  bp [B][T][C] (may be null), final_state [B] (may be null).
__device__ __forceinline__ void trop_acc(float v, int flat, float& best, int& bflat)
{
    if (v > best || (v == best && v != LAST_NEG_INF && flat < bflat)) { best = v; bflat = flat; }
}

__global__ __launch_bounds__(1024) void solo_viterbi(
    const float* __restrict__ w, const int* __restrict__ len, Ctx c, int T, int CPAD, int R,
    int* __restrict__ bp, int* __restrict__ final_state, float* __restrict__ score,
    int* __restrict__ item_status)
{
    extern __shared__ float smem[];
    float* cur = smem;
    float* nxt = cur + c.C;
    float* pv = nxt + c.C;
    int* pi = (int*)(pv + R * CPAD);
    float* redv = (float*)(pi + R * CPAD);
    int* redi = (int*)(redv + 32);
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = len[b];
    if (L < 0 || L > T) {
        if (tid == 0) {
            if (item_status) item_status[b] = kItemBadLength;
            score[b] = __builtin_nanf("");
            if (final_state) final_state[b] = -1;
        }
        return;
    }
    if (tid == 0 && item_status) item_status[b] = kItemOk;
    const int g = tid / CPAD, dl = tid - g * CPAD;
    const size_t fr = (size_t)c.C * c.V1;
    for (int d = tid; d < c.C; d += blockDim.x) cur[d] = d == 0 ? 0.f : LAST_NEG_INF;
    __syncthreads();
    for (int t = 0; t < L; ++t) {
        const float* wt = w + ((size_t)b * T + t) * fr;
        for (int d0 = 0; d0 < c.C; d0 += CPAD) {
            const int d = d0 + dl;
            if (g < R && d < c.C) {
                float best = LAST_NEG_INF;
                int bflat = 0x7fffffff;
                const int n = ctx_num_in(c, d);
                const int y = d > 0 ? ctx_in_label(c, d) : 0;
                for (int i = g; i < n; i += R) {
                    const int q = ctx_in_source(c, d, i);
                    trop_acc(__fadd_rn(cur[q], wt[(size_t)q * c.V1 + y]), q * c.V1 + y, best, bflat);
                }
                if (g == 0) trop_acc(__fadd_rn(cur[d], wt[(size_t)d * c.V1]), d * c.V1, best, bflat);
                pv[g * CPAD + dl] = best;
                pi[g * CPAD + dl] = bflat;
            }
            __syncthreads();
            if (g == 0 && d < c.C) {
                float best = LAST_NEG_INF;
                int bflat = 0x7fffffff;
                for (int k = 0; k < R; ++k) trop_acc(pv[k * CPAD + dl], pi[k * CPAD + dl], best, bflat);
                nxt[d] = best;
                if (bp) bp[((size_t)b * T + t) * c.C + d] = (bflat == 0x7fffffff) ? -1 : bflat;
            }
            __syncthreads();
        }
        for (int d = tid; d < c.C; d += blockDim.x) cur[d] = nxt[d];
        __syncthreads();
    }
    // best final state, lowest index among equals
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

// Tropical recursion for the full 1-gram context dependency (state = last label,
// C = V + 1), the bandwidth version of solo_viterbi: one workgroup per item, R row
// groups x CPAD columns.  Thread (g, y) keeps column y of rows g, g + R, ... of
// the NEXT frame in registers while it consumes the current one, so a whole frame
// (C*C*4 bytes) is in flight per compute unit and the weights are streamed at
// what one compute unit can pull from HBM.  Barriers order LDS only, so the loads
// stay in flight across them.  Same decisions as solo_viterbi: one float32 add per
// arc, exact comparisons, ties to the lowest flat arc index q*(V+1)+y.
// Column 0 holds the empty-label arcs q -> q; they are combined per destination.
template <int NR, int R>
__global__ __launch_bounds__(1024) void bigram_viterbi(
    const float* __restrict__ w, const int* __restrict__ len, int C, int T, int CPAD,
    int* __restrict__ bp, int* __restrict__ final_state, float* __restrict__ score,
    int* __restrict__ item_status)
{
    extern __shared__ float smem[];
    float* cur = smem;                      // [C] best score per state
    float* bw = cur + CPAD;                 // [C] empty-label weight of the frame per state
    float* pv = bw + CPAD;                  // [R][CPAD] partial best values
    int* pi = (int*)(pv + R * CPAD);        // [R][CPAD] their row-step index
    float* redv = (float*)(pi + R * CPAD);
    int* redi = (int*)(redv + 32);
    const int b = blockIdx.x, tid = threadIdx.x;
    const int L = len[b];
    if (L < 0 || L > T) {
        if (tid == 0) {
            if (item_status) item_status[b] = kItemBadLength;
            score[b] = __builtin_nanf("");
            if (final_state) final_state[b] = -1;
        }
        return;
    }
    if (tid == 0 && item_status) item_status[b] = kItemOk;
    const int g = tid / CPAD, y = tid - g * CPAD;
    const bool active = g < R && y < C;
    const size_t fr = (size_t)C * C;
    const float* wb = w + (size_t)b * T * fr;
    // element (row g + R i, column y) of a frame through a buffer descriptor over the item's
    // weights: per-thread byte offset + scalar offset (frame, row step); rows past the frame read
    // whatever follows (ignored), reads past the item return 0, so no load needs a guard
    const int yc = y < C ? y : 0, gc = g < R ? g : 0;
    const int voff = (gc * C + yc) * 4;
    const int stride = R * C * 4;
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(wb), 0, (int)((size_t)T * fr * 4), 0x00020000);
    float reg[NR];
    for (int d = tid; d < CPAD; d += blockDim.x) cur[d] = d == 0 ? 0.f : LAST_NEG_INF;
    if (L > 0) {
#pragma unroll
        for (int i = 0; i < NR; ++i)
            reg[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, i * stride, 0));
    }
    lds_only_barrier();
    for (int t = 0; t < L; ++t) {
        const int fo = (int)((size_t)(t + 1 < L ? t + 1 : t) * fr * 4);
        float best = LAST_NEG_INF;
        int bi = -1;
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const float wv = reg[i];
            reg[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, fo + i * stride, 0));
            const int q = g + R * i;
            if (q < C) {
                if (y == 0) {
                    if (active) bw[q] = wv;
                } else {
                    const float v = __fadd_rn(cur[q], wv);
                    if (v > best) { best = v; bi = i; }          // ascending q: the first maximum stays
                }
            }
        }
        if (active) { pv[g * CPAD + y] = best; pi[g * CPAD + y] = bi; }
        lds_only_barrier();
        if (g == 0 && y < C) {
            // destination y: label arcs from every q (partial maxima of the row groups), empty label from y itself
            float bv = LAST_NEG_INF;
            int bflat = 0x7fffffff;
            if (y > 0) {
#pragma unroll
                for (int k = 0; k < R; ++k) {
                    const int i = pi[k * CPAD + y];
                    if (i >= 0) trop_acc(pv[k * CPAD + y], (k + R * i) * C + y, bv, bflat);
                }
            }
            trop_acc(__fadd_rn(cur[y], bw[y]), y * C, bv, bflat);
            cur[y] = bv;
            if (bp) bp[((size_t)b * T + t) * C + y] = (bflat == 0x7fffffff) ? -1 : bflat;
        }
        lds_only_barrier();
    }
    // best final state, lowest index among equals
    float best = LAST_NEG_INF;
    int bidx = 0x7fffffff;
    for (int d = tid; d < C; d += blockDim.x)
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

// Follow the backpointers from the best final state (the 0/1 arc mask of the tropical gradient,
// Section 2.3, returned as indices).  A walk of len dependent loads would take len memory latencies,
// so the frames are cut into segments of S:
//   1. compose: for every segment and every state at its upper end, the state at its lower end
//      (S dependent loads, all segments and states in parallel);
//   2. boundaries: one thread per item hops from segment to segment (len/S dependent loads);
//   3. emit: every segment is walked once more from its now known upper state, writing labels
//      and states; frames past the length get -1.
// map [B][nseg][C], bnd [B][nseg+1].  An item without a path (invalid length, final state -1) gets
// -1 everywhere.  States read from bp are clamped into range: whatever the array holds, no access
// leaves it.
__device__ __forceinline__ int bt_prev_state(int arc, int V1, int C)
{
    const int q = arc / V1;
    return q < 0 ? 0 : (q >= C ? C - 1 : q);
}

__global__ void backtrace_compose_kernel(const int* __restrict__ bp, const int* __restrict__ len, int C, int V1,
                                         int T, int S, int nseg, int* __restrict__ map)
{
    const int s = blockIdx.x, b = blockIdx.y;
    const int L = len[b];
    if (L < 0 || L > T) return;
    const int t0 = s * S;
    const int t1 = t0 + S < L ? t0 + S : L;          // states at frame t1 -> states at frame t0
    if (t0 >= L) return;
    for (int q0 = threadIdx.x; q0 < C; q0 += blockDim.x) {
        int q = q0;
        for (int t = t1 - 1; t >= t0; --t) q = bt_prev_state(bp[((size_t)b * T + t) * C + q], V1, C);
        map[((size_t)b * nseg + s) * C + q0] = q;
    }
}

__global__ void backtrace_boundaries_kernel(const int* __restrict__ map, const int* __restrict__ len,
                                            const int* __restrict__ final_state, int B, int C, int T, int S,
                                            int nseg, int* __restrict__ bnd)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int L = len[b];
    int q = final_state[b];
    if (L < 0 || L > T || q < 0) return;
    q = q >= C ? C - 1 : q;
    const int last = L > 0 ? (L - 1) / S : -1;
    for (int s = last; s >= 0; --s) {
        bnd[(size_t)b * (nseg + 1) + s + 1] = q;          // state at the upper end of segment s
        q = map[((size_t)b * nseg + s) * C + q];
    }
    bnd[(size_t)b * (nseg + 1)] = q;
}

__global__ void backtrace_emit_kernel(const int* __restrict__ bp, const int* __restrict__ len,
                                      const int* __restrict__ final_state, const int* __restrict__ bnd,
                                      int C, int V1, int T, int S, int nseg,
                                      int* __restrict__ labels, int* __restrict__ states)
{
    const int s = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    int L = len[b];
    if (L < 0 || L > T || final_state[b] < 0) L = -1;   // no path was found for this item: all -1
    const int t0 = s * S;
    // padding of this segment's frames (and, by the last segment, of the last state)
    for (int t = t0 + tid; t < t0 + S && t < T; t += blockDim.x) {
        if (t >= L) labels[(size_t)b * T + t] = -1;
        if (t > L) states[(size_t)b * (T + 1) + t] = -1;
    }
    if (s == nseg - 1 && tid == 0 && T > L) states[(size_t)b * (T + 1) + T] = -1;
    if (tid != 0 || L < 0) return;
    if (L == 0) {
        if (s == 0) states[(size_t)b * (T + 1)] = bnd[(size_t)b * (nseg + 1)];
        return;
    }
    if (t0 >= L) return;
    const int t1 = t0 + S < L ? t0 + S : L;
    int q = bnd[(size_t)b * (nseg + 1) + s + 1];
    if (t1 == L) states[(size_t)b * (T + 1) + L] = q;
    for (int t = t1 - 1; t >= t0; --t) {
        const int arc = bp[((size_t)b * T + t) * C + q];
        q = bt_prev_state(arc, V1, C);
        labels[(size_t)b * T + t] = arc - q * V1;
        states[(size_t)b * (T + 1) + t] = q;
    }
}

}  // namespace last
