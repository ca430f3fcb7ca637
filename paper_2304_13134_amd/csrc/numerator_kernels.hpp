// Numerator of the globally normalised loss: the complete lattice intersected
// with the reference label string, and the log-semiring shortest distance on
// the resulting (t, u) grid (arXiv 2304.13134, Section 2.1; Table 1 "GNAT,
// intersected": O(TU) states and arcs, small enough to store).
//
// Three stages, all on the caller's stream:
//   1. gather   : the 2 arc weights leaving every (t, u) are pulled out of the
//                 dense tensor into a compact [B][T][U1][2] array (fully
//                 parallel, it is the only stage that touches the big tensor);
//   2. recursion: per item one workgroup runs the forward weights and a second
//                 one the backward weights, frame-serial, state-parallel;
//   3. scatter  : arc marginals exp(a + w + b' - N) are added onto the arcs of
//                 the complete lattice they ride on.
// Grid values are kept in float64 (they reach several thousand and feed an
// exponent that must be good to 1e-6); the transcendental part of each
// log-add-exp has an O(1) argument and is evaluated in float32.
#pragma once
#include "common.hpp"

namespace last {

// context state after the first u reference labels
__device__ __forceinline__ int ref_context(const Ctx& c, const int* __restrict__ r, int u)
{
    if (u == 0) return 0;
    if (c.order == 1 || u == 1) return r[u - 1];
    return 1 + c.V + (r[u - 2] - 1) * c.V + (r[u - 1] - 1);
}

__device__ __forceinline__ int clamp_label(int y, int V) { return y < 1 ? 1 : (y > V ? V : y); }

// status [B]: 0 ok, or the item_status code of the first problem found
__global__ void num_check_kernel(const int* __restrict__ len, const int* __restrict__ refs,
                                 const int* __restrict__ ulen, int T, int V, int Umax,
                                 int* __restrict__ status)
{
    __shared__ int bad;
    const int b = blockIdx.x;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    const int L = len[b], U = ulen[b];
    int code = kItemOk;
    if (L < 0 || L > T) code = kItemBadLength;
    else if (U < 0 || U > Umax) code = kItemBadRefLength;
    else {
        for (int u = threadIdx.x; u < U; u += blockDim.x) {
            const int y = refs[(size_t)b * Umax + u];
            if (y < 1 || y > V) atomicOr(&bad, 1);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (code == kItemOk && bad) code = kItemBadLabel;
        if (code == kItemOk && U > L) code = kItemInfeasible;
        status[b] = code;
    }
}

// wi[b][t][u][0] = w[b][t][ctx(u)][0]; wi[b][t][u][1] = w[b][t][ctx(u)][ref[u]] (u < U)
__global__ void num_gather_kernel(const float* __restrict__ w, const int* __restrict__ len,
                                  const int* __restrict__ refs, const int* __restrict__ ulen,
                                  const int* __restrict__ status, Ctx c, int T, int Umax,
                                  float2* __restrict__ wi)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.z, t = blockIdx.y;
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    if (t >= L || u > U) return;
    const int* r = refs + (size_t)b * Umax;
    const int q = ref_context(c, r, u);
    const float* row = w + (((size_t)b * T + t) * c.C + q) * c.V1;
    float2 o;
    o.x = row[0];
    o.y = (u < U) ? row[r[u]] : LAST_NEG_INF;
    wi[((size_t)b * T + t) * U1 + u] = o;
}

__device__ __forceinline__ double log_add(double x, double y)
{
    const double m = x > y ? x : y;
    if (m == (double)LAST_NEG_INF) return m;
    const double lo = x > y ? y : x;
    const float d = (float)(lo - m);           // <= 0, -inf allowed
    return m + (double)log1pf(__expf(d));
}

// grid (B, 2): blockIdx.y = 0 forward weights a[b][t][u], = 1 backward weights bk.
// Both arrays are [B][T+1][U1] float64; cells outside the reachable cone hold -inf.
__global__ __launch_bounds__(256) void num_recursion_kernel(
    const float2* __restrict__ wi, const int* __restrict__ len, const int* __restrict__ ulen,
    const int* __restrict__ status, int T, int Umax,
    double* __restrict__ a, double* __restrict__ bk, double* __restrict__ Nws,
    float* __restrict__ numerator, int* __restrict__ item_status)
{
    extern __shared__ double sm[];
    const int U1 = Umax + 1;
    const int b = blockIdx.x, tid = threadIdx.x;
    const bool fwd = blockIdx.y == 0;
    const int st = status[b];
    if (st != kItemOk) {
        if (fwd && tid == 0) {
            if (item_status) item_status[b] = st;
            numerator[b] = (st == kItemInfeasible) ? LAST_NEG_INF : __builtin_nanf("");
            Nws[b] = (double)LAST_NEG_INF;
        }
        return;
    }
    if (fwd && tid == 0 && item_status) item_status[b] = kItemOk;
    const int L = len[b], U = ulen[b];
    double* buf0 = sm;
    double* buf1 = sm + U1 + 1;               // one pad cell on the right for bk[u+1]
    const double NI = (double)LAST_NEG_INF;
    const float2* wb = wi + (size_t)b * T * U1;
    if (fwd) {
        double* A = a + (size_t)b * (T + 1) * U1;
        for (int u = tid; u <= U; u += blockDim.x) {
            const double v = u == 0 ? 0.0 : NI;
            buf0[u] = v;
            A[u] = v;
        }
        __syncthreads();
        double* cur = buf0;
        double* nxt = buf1;
        for (int t = 0; t < L; ++t) {
            const float2* wt = wb + (size_t)t * U1;
            for (int u = tid; u <= U; u += blockDim.x) {
                double v = cur[u] + (double)wt[u].x;
                if (u >= 1) v = log_add(v, cur[u - 1] + (double)wt[u - 1].y);
                nxt[u] = v;
                A[(size_t)(t + 1) * U1 + u] = v;
            }
            __syncthreads();
            double* s = cur; cur = nxt; nxt = s;
        }
        if (tid == 0) {
            Nws[b] = cur[U];
            numerator[b] = (float)cur[U];
        }
    } else {
        double* Bk = bk + (size_t)b * (T + 1) * U1;
        for (int u = tid; u <= U + 1; u += blockDim.x) {
            const double v = u == U ? 0.0 : NI;
            buf0[u] = v;
            buf1[u] = NI;
            if (u <= U) Bk[(size_t)L * U1 + u] = v;
        }
        __syncthreads();
        double* cur = buf0;
        double* nxt = buf1;
        for (int t = L - 1; t >= 0; --t) {
            const float2* wt = wb + (size_t)t * U1;
            for (int u = tid; u <= U; u += blockDim.x) {
                const float2 ww = wt[u];
                double v = (double)ww.x + cur[u];
                if (u < U) v = log_add(v, (double)ww.y + cur[u + 1]);
                nxt[u] = v;
                Bk[(size_t)t * U1 + u] = v;
            }
            __syncthreads();
            double* s = cur; cur = nxt; nxt = s;
        }
    }
}

// Marginals of the intersected lattice (Eq. 1 on the (t,u) grid), added with
// the caller's scale onto dw[b][t][ctx(u)][label].  Several u may share one
// arc of the complete lattice, hence atomic adds.
__global__ void num_scatter_kernel(const float2* __restrict__ wi, const int* __restrict__ len,
                                   const int* __restrict__ refs, const int* __restrict__ ulen,
                                   const int* __restrict__ status, Ctx c, int T, int Umax,
                                   const double* __restrict__ a, const double* __restrict__ bk,
                                   const double* __restrict__ Nws, float* __restrict__ dw,
                                   float scale)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.z, t = blockIdx.y;
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    if (t >= L || u > U) return;
    const double N = Nws[b];
    const double av = a[((size_t)b * (T + 1) + t) * U1 + u];
    if (av == (double)LAST_NEG_INF || N == (double)LAST_NEG_INF) return;
    const int* r = refs + (size_t)b * Umax;
    const int q = ref_context(c, r, u);
    const float2 ww = wi[((size_t)b * T + t) * U1 + u];
    float* row = dw + (((size_t)b * T + t) * c.C + q) * c.V1;
    const double* bn = bk + ((size_t)b * (T + 1) + t + 1) * U1;
    const double e0 = av + (double)ww.x + bn[u] - N;
    if (e0 > -100.0) atomicAdd(row, scale * __expf((float)e0));
    if (u < U) {
        const double e1 = av + (double)ww.y + bn[u + 1] - N;
        if (e1 > -100.0) atomicAdd(row + r[u], scale * __expf((float)e1));
    }
}

}  // namespace last
