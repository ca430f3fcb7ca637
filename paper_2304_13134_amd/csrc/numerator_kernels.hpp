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
// The locally normalised variant (Section 2.1: a model like RNN-T is the same
// intersection followed by a shortest distance, with the arcs leaving each state
// normalised; Table 1, first row) adds to the gather the log-sum-exp lz of the
// V+1 arcs leaving (t, ctx(u)), subtracts it in the recursion, and its scatter
// writes d/dw = marginals - (occupancy of the state) * softmax(row), row by row.
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

// status [B]: 0 ok, or the item_status code of the first problem found.
// ctxs [B][U1]: context state after the first u reference labels (-1 past U).
// link [B][U1][2]: [0] = the next u' > u with the same context (-1: none), [1] = 1 when no
// u' < u has the same context (u heads its chain).  Cells of one chain ride on the same rows
// of the complete lattice.
__global__ void num_check_kernel(const int* __restrict__ len, const int* __restrict__ refs,
                                 const int* __restrict__ ulen, Ctx c, int T, int Umax,
                                 int* __restrict__ status, int* __restrict__ ctxs,
                                 int* __restrict__ link, const int* __restrict__ badtab)
{
    __shared__ int bad;
    const int b = blockIdx.x;
    const int U1 = Umax + 1;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    const int L = len[b], U = ulen[b];
    int code = kItemOk;
    if (badtab && badtab[0]) code = kItemBadTable;
    else if (L < 0 || L > T) code = kItemBadLength;
    else if (U < 0 || U > Umax) code = kItemBadRefLength;
    else {
        for (int u = threadIdx.x; u < U; u += blockDim.x) {
            const int y = refs[(size_t)b * Umax + u];
            if (y < 1 || y > c.V) atomicOr(&bad, 1);
        }
    }
    __syncthreads();
    if (code == kItemOk && bad) code = kItemBadLabel;
    if (code == kItemOk && U > L) code = kItemInfeasible;
    if (threadIdx.x == 0) status[b] = code;
    int* cx = ctxs + (size_t)b * U1;
    if (code != kItemOk && code != kItemInfeasible) {
        for (int u = threadIdx.x; u < U1; u += blockDim.x) cx[u] = -1;
        return;
    }
    const int* r = refs + (size_t)b * Umax;
    if (c.order == 0) {
        // a general automaton has to be walked label by label
        if (threadIdx.x == 0) {
            int q = 0;
            cx[0] = 0;
            for (int u = 1; u <= U; ++u) { q = ctx_next(c, q, r[u - 1]); cx[u] = q; }
        }
        for (int u = U + 1 + threadIdx.x; u < U1; u += blockDim.x) cx[u] = -1;
    } else {
        for (int u = threadIdx.x; u < U1; u += blockDim.x) cx[u] = u <= U ? ref_context(c, r, u) : -1;
    }
    __syncthreads();
    int* lk = link + (size_t)b * U1 * 2;
    for (int u = threadIdx.x; u < U1; u += blockDim.x) {
        int nxt = -1, head = 1;
        if (u <= U) {
            const int q = cx[u];
            for (int v = u + 1; v <= U; ++v)
                if (cx[v] == q) { nxt = v; break; }
            for (int v = u - 1; v >= 0; --v)
                if (cx[v] == q) { head = 0; break; }
        } else {
            head = 0;
        }
        lk[2 * u] = nxt;
        lk[2 * u + 1] = head;
    }
}

// wi[b][t][u][0] = w[b][t][ctx(u)][0]; wi[b][t][u][1] = w[b][t][ctx(u)][ref[u]] (u < U)
__global__ void num_gather_kernel(const float* __restrict__ w, const int* __restrict__ len,
                                  const int* __restrict__ refs, const int* __restrict__ ulen,
                                  const int* __restrict__ status, const int* __restrict__ ctxs,
                                  Ctx c, int T, int Umax, float2* __restrict__ wi)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.z, t = blockIdx.y;
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    if (t >= L || u > U) return;
    const int* r = refs + (size_t)b * Umax;
    const int q = ctxs[(size_t)b * U1 + u];
    const float* row = w + (((size_t)b * T + t) * c.C + q) * c.V1;
    float2 o;
    o.x = row[0];
    o.y = (u < U) ? row[r[u]] : LAST_NEG_INF;
    wi[((size_t)b * T + t) * U1 + u] = o;
}

// Locally normalised variant of the gather: one wavefront per cell (t, u) also takes
// lz[b][t][u] = log sum_y exp w[b][t][ctx(u)][y].  Cells outside the cone that paths from (0,0)
// to (len, U) can visit get zeros without touching the weights (their forward or backward weight
// is -inf, whatever the arc weights).
__global__ __launch_bounds__(256) void num_gather_local_kernel(
    const float* __restrict__ w, const int* __restrict__ len, const int* __restrict__ refs,
    const int* __restrict__ ulen, const int* __restrict__ status, const int* __restrict__ ctxs,
    Ctx c, int T, int Umax, float2* __restrict__ wi, double* __restrict__ lz)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.z, t = blockIdx.y;
    const int u = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    if (t >= L || u > U) return;
    const size_t cell = ((size_t)b * T + t) * U1 + u;
    if (u > t || U - u > L - t) {
        if (lane == 0) { wi[cell] = make_float2(0.f, 0.f); lz[cell] = 0.0; }
        return;
    }
    const int* r = refs + (size_t)b * Umax;
    const int q = ctxs[(size_t)b * U1 + u];
    const float* row = w + (((size_t)b * T + t) * c.C + q) * c.V1;
    float m = LAST_NEG_INF;
    for (int y = lane; y < c.V1; y += kWave) m = fmaxf(m, row[y]);
    m = wave_max(m);
    float s = 0.f;
    if (m != LAST_NEG_INF)
        for (int y = lane; y < c.V1; y += kWave) s += expf(row[y] - m);
    s = wave_sum(s);
    if (lane == 0) {
        float2 o;
        o.x = row[0];
        o.y = (u < U) ? row[r[u]] : LAST_NEG_INF;
        wi[cell] = o;
        lz[cell] = (m == LAST_NEG_INF) ? (double)LAST_NEG_INF : (double)m + log((double)s);
    }
}

// log(exp x + exp y): the large part m in float64, the correction log(1 + exp(lo - m)) in (0, log 2]
// with the hardware exp2 / log2 (absolute error of a few 1e-8, far below what feeds an exponent
// that must be good to 1e-6 after a few hundred frames)
__device__ __forceinline__ double log_add(double x, double y)
{
    const double m = x > y ? x : y;
    if (m == (double)LAST_NEG_INF) return m;
    const double lo = x > y ? y : x;
    const float d = (float)(lo - m);           // <= 0, -inf allowed
    return m + (double)__logf(1.f + __expf(d));
}

// grid (B, 2): blockIdx.y = 0 forward weights a[b][t][u], = 1 backward weights bk.
// Both arrays are [B][T+1][U1] float64; cells outside the reachable cone hold -inf.
__global__ __launch_bounds__(256) void num_recursion_kernel(
    const float2* __restrict__ wi, const double* __restrict__ lz, const int* __restrict__ len,
    const int* __restrict__ ulen, const int* __restrict__ status, int T, int Umax,
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
    const double* zb = lz ? lz + (size_t)b * T * U1 : nullptr;   // locally normalised: w - lz
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
            const double* zt = zb ? zb + (size_t)t * U1 : nullptr;
            for (int u = tid; u <= U; u += blockDim.x) {
                double v = cur[u] + ((double)wt[u].x - (zt ? zt[u] : 0.0));
                if (u >= 1) v = log_add(v, cur[u - 1] + ((double)wt[u - 1].y - (zt ? zt[u - 1] : 0.0)));
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
            const double* zt = zb ? zb + (size_t)t * U1 : nullptr;
            for (int u = tid; u <= U; u += blockDim.x) {
                const float2 ww = wt[u];
                const double z = zt ? zt[u] : 0.0;
                double v = ((double)ww.x - z) + cur[u];
                if (u < U) v = log_add(v, ((double)ww.y - z) + cur[u + 1]);
                nxt[u] = v;
                Bk[(size_t)t * U1 + u] = v;
            }
            __syncthreads();
            double* s = cur; cur = nxt; nxt = s;
        }
    }
}

// The same recursion with one wavefront per item and direction, for references of up to
// 64 * CPL - 1 labels: lane l keeps the states u = l*CPL .. l*CPL + CPL-1 of the current frame in
// registers (one lane shuffle per frame hands a value across the lane boundary; no LDS, no
// workgroup barrier), and it reads the gathered arc weights of its states a chunk of CH frames ahead
// of the recursion.  (Pulling them straight out of the dense tensor instead was measured slower:
// every lane then touches two cache lines of its own per frame, and one wavefront cannot keep
// enough of those in flight.)  Arithmetic as in num_recursion_kernel.

template <int CPL, int CH>
struct NwBuf {
    float w0[CH][CPL], w1[CH][CPL];
};

typedef __amdgpu_buffer_rsrc_t nw_buf_t;
constexpr unsigned kNwOut = 0xfffffff0u;        // a byte offset no buffer of an item reaches: loads give 0, stores are dropped

__device__ __forceinline__ nw_buf_t nw_rsrc(const void* p, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)(unsigned)bytes, 0x00020000);
}
__device__ __forceinline__ void nw_store64(double v, nw_buf_t r, unsigned voff, unsigned soff)
{
    typedef decltype(__builtin_amdgcn_raw_buffer_load_b64(r, 0, 0, 0)) b64_t;
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(b64_t, v), r, (int)voff, (int)soff, 0);
}
// log_add without a branch: -inf + -inf stays -inf
__device__ __forceinline__ double nw_log_add(double x, double y)
{
    const double m = x > y ? x : y;
    const double lo = x > y ? y : x;
    const float d = m == (double)LAST_NEG_INF ? 0.f : (float)(lo - m);
    return m + (double)__logf(1.f + __expf(d));
}

// the arc weights of CH frames, t = t0 + k*dir clamped into the item (values of frames outside it are unused)
template <int CPL, int CH>
__device__ __forceinline__ void nw_load(NwBuf<CPL, CH>& d, nw_buf_t irs, unsigned rowb, int t0, int dir, int L,
                                        const unsigned (&ou)[CPL])
{
#pragma unroll
    for (int k = 0; k < CH; ++k) {
        int t = t0 + k * dir;
        t = t < L ? t : L - 1;
        t = t < 0 ? 0 : t;
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const float2 v = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(irs, (int)ou[i], (int)((unsigned)t * rowb), 0));
            d.w0[k][i] = v.x;
            d.w1[k][i] = v.y;
        }
    }
}

// Requires (T+1)*(Umax+1)*8 below 2^32 - 16 (byte offsets inside one item's arrays).
template <int CPL, int CH>
__global__ __launch_bounds__(kWave) void num_wave_kernel(
    const float2* __restrict__ wi, const int* __restrict__ len, const int* __restrict__ ulen,
    const int* __restrict__ status, int T, int Umax, double* __restrict__ a, double* __restrict__ bk,
    double* __restrict__ Nws, float* __restrict__ numerator, int* __restrict__ item_status)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.x, lane = threadIdx.x;
    const bool fwd = blockIdx.y == 0;
    const int st = status[b];
    if (st != kItemOk) {
        if (fwd && lane == 0) {
            if (item_status) item_status[b] = st;
            numerator[b] = (st == kItemInfeasible) ? LAST_NEG_INF : __builtin_nanf("");
            Nws[b] = (double)LAST_NEG_INF;
        }
        return;
    }
    if (fwd && lane == 0 && item_status) item_status[b] = kItemOk;
    const int L = len[b], U = ulen[b];
    const double NI = (double)LAST_NEG_INF;
    const unsigned rowb = (unsigned)U1 * 8u;
    const nw_buf_t irs = nw_rsrc(wi + (size_t)b * T * U1, (size_t)T * U1 * 8);
    // byte offset of each of this lane's states inside a row of the (t,u) arrays; kNwOut past the reference
    unsigned ou[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
        const int u = lane * CPL + i;
        ou[i] = u <= U ? (unsigned)u * 8u : kNwOut;
    }
    double cur[CPL];
    NwBuf<CPL, CH> nxt;
    if (fwd) {
        const nw_buf_t ars = nw_rsrc(a + (size_t)b * (T + 1) * U1, (size_t)(T + 1) * U1 * 8);
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            cur[i] = lane * CPL + i == 0 ? 0.0 : NI;
            nw_store64(cur[i], ars, ou[i], 0);
        }
        if (L > 0) nw_load<CPL, CH>(nxt, irs, rowb, 0, 1, L, ou);
        for (int t0 = 0; t0 < L; t0 += CH) {
            const NwBuf<CPL, CH> now = nxt;                       // (waits for the chunk, then frees its registers)
            nw_load<CPL, CH>(nxt, irs, rowb, t0 + CH, 1, L, ou);
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                const int t = t0 + k;
                if (t < L) {
                    double up[CPL];
#pragma unroll
                    for (int i = 0; i < CPL; ++i) up[i] = cur[i] + (double)now.w1[k][i];     // label arc u -> u+1
                    double left = __shfl_up(up[CPL - 1], 1, kWave);
                    left = lane == 0 ? NI : left;
#pragma unroll
                    for (int i = 0; i < CPL; ++i) {
                        const double v = nw_log_add(cur[i] + (double)now.w0[k][i], i == 0 ? left : up[i - 1]);
                        cur[i] = v;
                        nw_store64(v, ars, ou[i], (unsigned)(t + 1) * rowb);
                    }
                }
            }
        }
        // N = the forward weight of (L, U)
        double nv = NI;
#pragma unroll
        for (int i = 0; i < CPL; ++i) nv = lane * CPL + i == U ? cur[i] : nv;
        if (lane == U / CPL) {
            Nws[b] = nv;
            numerator[b] = (float)nv;
        }
    } else {
        const nw_buf_t brs = nw_rsrc(bk + (size_t)b * (T + 1) * U1, (size_t)(T + 1) * U1 * 8);
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            cur[i] = lane * CPL + i == U ? 0.0 : NI;
            nw_store64(cur[i], brs, ou[i], (unsigned)L * rowb);
        }
        // frames walked downwards: the chunk that ends below frame tend holds frames tend-1, tend-2, ...
        if (L > 0) nw_load<CPL, CH>(nxt, irs, rowb, L - 1, -1, L, ou);
        for (int tend = L; tend > 0; tend -= CH) {
            const NwBuf<CPL, CH> now = nxt;
            nw_load<CPL, CH>(nxt, irs, rowb, tend - CH - 1, -1, L, ou);
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                const int t = tend - 1 - k;
                if (t >= 0) {
                    double right = __shfl_down(cur[0], 1, kWave);
                    right = lane == kWave - 1 ? NI : right;
#pragma unroll
                    for (int i = 0; i < CPL; ++i) {
                        const double nb = i + 1 < CPL ? cur[i + 1] : right;     // still the weight of frame t+1
                        const double v = nw_log_add((double)now.w0[k][i] + cur[i], (double)now.w1[k][i] + nb);
                        cur[i] = v;
                        nw_store64(v, brs, ou[i], (unsigned)t * rowb);
                    }
                }
            }
        }
    }
}

// Marginals of the intersected lattice (Eq. 1 on the (t,u) grid), added with
// the caller's scale onto dw[b][t][ctx(u)][label].  Several u may share one
// arc of the complete lattice, hence atomic adds.
__global__ void num_scatter_kernel(const float2* __restrict__ wi, const int* __restrict__ len,
                                   const int* __restrict__ refs, const int* __restrict__ ulen,
                                   const int* __restrict__ status, const int* __restrict__ ctxs,
                                   Ctx c, int T, int Umax,
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
    const int q = ctxs[(size_t)b * U1 + u];
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

// Gradient of the locally normalised log-likelihood (Section 2.1) with respect to the weights,
// dw[b][t][q][y] (+)= scale * ( [marginals of the intersected lattice riding on arc (t,q,y)]
//                              - [their sum over the arcs leaving (t,q)] * softmax(w[b][t][q])[y] ).
// One wavefront per frame and chain of cells with the same context q (see num_check_kernel):
// it alone writes row (t,q), so no atomics are needed and the result does not depend on timing.
// LDS: blockDim.x/64 arrays of V1 floats (the label marginals of the chain).
__global__ __launch_bounds__(256) void num_scatter_local_kernel(
    const float* __restrict__ w, const float2* __restrict__ wi, const double* __restrict__ lz,
    const int* __restrict__ len, const int* __restrict__ refs, const int* __restrict__ ulen,
    const int* __restrict__ status, const int* __restrict__ ctxs, const int* __restrict__ link,
    Ctx c, int T, int Umax, const double* __restrict__ a, const double* __restrict__ bk,
    const double* __restrict__ Nws, float* __restrict__ dw, float scale, int accumulate)
{
    extern __shared__ float nsl_lab[];
    const int U1 = Umax + 1;
    const int b = blockIdx.z, t = blockIdx.y;
    const int wv = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    const int u = blockIdx.x * (blockDim.x / kWave) + wv;
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    if (t >= L || u > U) return;
    const int* lk = link + (size_t)b * U1 * 2;
    if (!lk[2 * u + 1]) return;
    const double N = Nws[b];
    if (N == (double)LAST_NEG_INF) return;
    float* lab = nsl_lab + (size_t)wv * c.V1;
    const int* r = refs + (size_t)b * Umax;
    const double* at = a + ((size_t)b * (T + 1) + t) * U1;
    const double* bn = bk + ((size_t)b * (T + 1) + t + 1) * U1;
    const size_t cell0 = ((size_t)b * T + t) * U1;
    // first walk: is any cell of the chain on a path at all?  (cells outside the cone of paths
    // carry no log-sum-exp; every cell inside it carries the same one, that of row (t,q))
    int vin = -1;
    for (int v = u; v >= 0; v = lk[2 * v])
        if (vin < 0 && at[v] != (double)LAST_NEG_INF && v <= t && U - v <= L - t) vin = v;
    if (vin < 0) return;
    const double z = lz[cell0 + vin];
    for (int y = lane; y < c.V1; y += kWave) lab[y] = 0.f;
    float occ = 0.f, pbs = 0.f;
    for (int v = u; v >= 0; v = lk[2 * v]) {
        const double av = at[v];
        if (av == (double)LAST_NEG_INF) continue;
        const float2 ww = wi[cell0 + v];
        const double e0 = av + ((double)ww.x - z) + bn[v] - N;
        const float p0 = e0 > -100.0 ? __expf((float)e0) : 0.f;
        float p1 = 0.f;
        if (v < U) {
            const double e1 = av + ((double)ww.y - z) + bn[v + 1] - N;
            if (e1 > -100.0) p1 = __expf((float)e1);
            if (lane == 0) lab[r[v]] += p1;    // one lane, chain order: deterministic
        }
        occ += p0 + p1;
        pbs += p0;
    }
    const int q = ctxs[(size_t)b * U1 + u];
    const size_t ro = (((size_t)b * T + t) * c.C + q) * c.V1;
    const float* row = w + ro;
    float* grow = dw + ro;
    __builtin_amdgcn_wave_barrier();
    for (int y = lane; y < c.V1; y += kWave) {
        float g = lab[y] - occ * __expf((float)((double)row[y] - z));
        if (y == 0) g += pbs;
        if (accumulate) grow[y] += scale * g; else grow[y] = scale * g;
    }
}

}  // namespace last
