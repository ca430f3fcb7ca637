// Numerator of the globally normalised loss when the weights come from the
// shared-embedding weight function and are never materialised (arXiv
// 2304.13134, Sections 2.1 and 4.1): only the two arcs that leave each state
// (t, u) of the intersected lattice are evaluated,
//   w0 = bf16(tanh(f_t + e_ctx(u))) . W[:, 0],   w1 = ... . W[:, ref[u]],
// with float32 accumulation, then the (t, u) recursion of
// numerator_kernels.hpp runs on them.  Two dot products per state are no
// matrix-core work: a wavefront takes one state, every lane H/64 hidden units.
//
// The gradient chains the marginals pb, pl of the intersected lattice through
// the weight function in two passes, each recomputing the hidden vectors
// instead of storing T*U*H of them:
//   by frame : df[b][t]   = sum_u dpre(t,u)          one wavefront per (b, t), plain stores
//   by label : de[ctx(u)] += sum_t dpre(t,u)         one wavefront per (b, u, chunk of frames),
//              dW[:, 0] += sum_t h pb, dW[:, ref[u]] += sum_t h pl     float atomics at the end
// with dpre = (pb W[:,0] + pl W[:,ref[u]]) (1 - h^2).
#pragma once
#include "common.hpp"
#include "fused_kernels.hpp"
#include "numerator_kernels.hpp"

namespace last {

constexpr int kFnMaxPairs = 4;      // hidden units per lane / 2: H = 128 * pairs... H <= 512
constexpr int kFnWaves = 4;         // wavefronts per workgroup
constexpr int kFnStrip = 16;        // frames per wavefront in the gather
constexpr int kFnChunk = 128;       // frames per wavefront in the by-label pass

// Wt [V1][H] float32 = W transposed: a label's column becomes a contiguous row
__global__ void fnum_transpose_w_kernel(const __bf16* __restrict__ W, int H, int V1, float* __restrict__ Wt)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= H * V1) return;
    const int y = i / H, k = i - y * H;
    Wt[i] = (float)W[(size_t)k * V1 + y];
}

__device__ __forceinline__ bool fn_in_cone(int t, int u, int L, int U) { return u <= t && U - u <= L - t; }

// hidden units of one lane: pairs j = 0..np-1 cover units 2*(lane*np + j), +1
struct FnLane {
    unsigned e[kFnMaxPairs];
    float w0[2 * kFnMaxPairs], w1[2 * kFnMaxPairs];
};

__device__ __forceinline__ void fn_load_lane(FnLane& r, const __bf16* __restrict__ erow,
                                             const float* __restrict__ Wt, int H, int y1, int np, int lane)
{
#pragma unroll
    for (int j = 0; j < kFnMaxPairs; ++j) {
        const bool on = j < np;
        const int k = 2 * (lane * np + j);
        r.e[j] = on ? *(const unsigned*)(erow + k) : 0u;
        r.w0[2 * j] = on ? Wt[k] : 0.f;
        r.w0[2 * j + 1] = on ? Wt[k + 1] : 0.f;
        r.w1[2 * j] = (on && y1 > 0) ? Wt[(size_t)y1 * H + k] : 0.f;
        r.w1[2 * j + 1] = (on && y1 > 0) ? Wt[(size_t)y1 * H + k + 1] : 0.f;
    }
}

__device__ __forceinline__ float fn_lo(unsigned pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float fn_hi(unsigned pair) { return __uint_as_float(pair & 0xffff0000u); }

// wi[b][t][u] = (w0, w1) for every state of the intersected lattice; grid (ceil(U1/4), ceil(T/16), B)
__global__ __launch_bounds__(kFnWaves * kWave) void fnum_gather_kernel(
    const __bf16* __restrict__ f, const __bf16* __restrict__ e, const float* __restrict__ Wt,
    const int* __restrict__ len, const int* __restrict__ refs, const int* __restrict__ ulen,
    const int* __restrict__ status, const int* __restrict__ ctxs, int T, int Umax, int H,
    float2* __restrict__ wi)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.z;
    const int u = blockIdx.x * kFnWaves + threadIdx.x / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    if (u > U) return;
    const int np = H / 128;
    const int y1 = u < U ? refs[(size_t)b * Umax + u] : 0;
    FnLane r;
    fn_load_lane(r, e + (size_t)ctxs[(size_t)b * U1 + u] * H, Wt, H, y1, np, lane);
    const int t0 = blockIdx.y * kFnStrip;
    for (int t = t0; t < t0 + kFnStrip && t < L; ++t) {
        const size_t cell = ((size_t)b * T + t) * U1 + u;
        if (!fn_in_cone(t, u, L, U)) {          // no path through this state: the weights are never used
            if (lane == 0) wi[cell] = make_float2(0.f, 0.f);
            continue;
        }
        const __bf16* ft = f + ((size_t)b * T + t) * H;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int j = 0; j < kFnMaxPairs; ++j) {
            if (j < np) {
                const unsigned h = tanh_pair(*(const unsigned*)(ft + 2 * (lane * np + j)), r.e[j]);
                s0 = fmaf(fn_lo(h), r.w0[2 * j], s0);
                s0 = fmaf(fn_hi(h), r.w0[2 * j + 1], s0);
                s1 = fmaf(fn_lo(h), r.w1[2 * j], s1);
                s1 = fmaf(fn_hi(h), r.w1[2 * j + 1], s1);
            }
        }
        s0 = wave_sum(s0);
        s1 = wave_sum(s1);
        if (lane == 0) wi[cell] = make_float2(s0, u < U ? s1 : LAST_NEG_INF);
    }
}

// marginals of the two arcs leaving (t, u); false when the state is on no path
__device__ __forceinline__ bool fn_marginals(const float2* __restrict__ wi, const double* __restrict__ a,
                                             const double* __restrict__ bk, double N, int T, int U1,
                                             int b, int t, int u, int U, float& p0, float& p1)
{
    const double av = a[((size_t)b * (T + 1) + t) * U1 + u];
    p0 = 0.f;
    p1 = 0.f;
    if (av == (double)LAST_NEG_INF) return false;
    const float2 ww = wi[((size_t)b * T + t) * U1 + u];
    const double* bn = bk + ((size_t)b * (T + 1) + t + 1) * U1;
    const double e0 = av + (double)ww.x + bn[u] - N;
    if (e0 > -100.0) p0 = __expf((float)e0);
    if (u < U) {
        const double e1 = av + (double)ww.y + bn[u + 1] - N;
        if (e1 > -100.0) p1 = __expf((float)e1);
    }
    return p0 != 0.f || p1 != 0.f;
}

// df[b][t][:] (+)= scale * sum_u dpre(t, u); one wavefront per (b, t), grid (ceil(T/4), B).
// Frames past the length and items without a path get zeros (or stay as they are when accumulating).
__global__ __launch_bounds__(kFnWaves * kWave) void fnum_df_kernel(
    const __bf16* __restrict__ f, const __bf16* __restrict__ e, const float* __restrict__ Wt,
    const float2* __restrict__ wi, const int* __restrict__ len, const int* __restrict__ refs,
    const int* __restrict__ ulen, const int* __restrict__ status, const int* __restrict__ ctxs,
    const double* __restrict__ a, const double* __restrict__ bk, const double* __restrict__ Nws,
    int T, int Umax, int H, float* __restrict__ df, float scale, int accumulate)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.y;
    const int t = blockIdx.x * kFnWaves + threadIdx.x / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    if (t >= T) return;
    const int np = H / 128;
    float acc[2 * kFnMaxPairs];
#pragma unroll
    for (int i = 0; i < 2 * kFnMaxPairs; ++i) acc[i] = 0.f;
    const int L = len[b], U = ulen[b];
    const double N = Nws[b];
    if (status[b] == kItemOk && t < L && N != (double)LAST_NEG_INF) {
        const __bf16* ft = f + ((size_t)b * T + t) * H;
        unsigned fp[kFnMaxPairs];
#pragma unroll
        for (int j = 0; j < kFnMaxPairs; ++j) fp[j] = j < np ? *(const unsigned*)(ft + 2 * (lane * np + j)) : 0u;
        const int ulo = U - (L - t) > 0 ? U - (L - t) : 0, uhi = t < U ? t : U;
        for (int u = ulo; u <= uhi; ++u) {
            float p0, p1;
            if (!fn_marginals(wi, a, bk, N, T, U1, b, t, u, U, p0, p1)) continue;
            const int y1 = u < U ? refs[(size_t)b * Umax + u] : 0;
            FnLane r;
            fn_load_lane(r, e + (size_t)ctxs[(size_t)b * U1 + u] * H, Wt, H, y1, np, lane);
#pragma unroll
            for (int j = 0; j < kFnMaxPairs; ++j) {
                if (j < np) {
                    const unsigned h = tanh_pair(fp[j], r.e[j]);
                    const float h0 = fn_lo(h), h1 = fn_hi(h);
                    acc[2 * j] += (p0 * r.w0[2 * j] + p1 * r.w1[2 * j]) * (1.f - h0 * h0);
                    acc[2 * j + 1] += (p0 * r.w0[2 * j + 1] + p1 * r.w1[2 * j + 1]) * (1.f - h1 * h1);
                }
            }
        }
    }
    float* o = df + ((size_t)b * T + t) * H;
#pragma unroll
    for (int j = 0; j < kFnMaxPairs; ++j) {
        if (j < np) {
            const int k = 2 * (lane * np + j);
            if (accumulate) { o[k] += scale * acc[2 * j]; o[k + 1] += scale * acc[2 * j + 1]; }
            else { o[k] = scale * acc[2 * j]; o[k + 1] = scale * acc[2 * j + 1]; }
        }
    }
}

// de[ctx(u)][:] += scale * sum_t dpre(t, u), dW[:, 0] += scale * sum_t h pb, dW[:, ref[u]] += scale * sum_t h pl
// over one chunk of frames; one wavefront per (b, u, chunk), grid (ceil(U1/4), ceil(T/128), B).
__global__ __launch_bounds__(kFnWaves * kWave) void fnum_de_dw_kernel(
    const __bf16* __restrict__ f, const __bf16* __restrict__ e, const float* __restrict__ Wt,
    const float2* __restrict__ wi, const int* __restrict__ len, const int* __restrict__ refs,
    const int* __restrict__ ulen, const int* __restrict__ status, const int* __restrict__ ctxs,
    const double* __restrict__ a, const double* __restrict__ bk, const double* __restrict__ Nws,
    int T, int Umax, int H, int V1, float* __restrict__ de, float* __restrict__ dW, float scale)
{
    const int U1 = Umax + 1;
    const int b = blockIdx.z;
    const int u = blockIdx.x * kFnWaves + threadIdx.x / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    if (u >= U1 || status[b] != kItemOk) return;
    const int L = len[b], U = ulen[b];
    const double N = Nws[b];
    if (u > U || N == (double)LAST_NEG_INF) return;
    // frames at which (t, u) is on a path and has arcs leaving it
    int tlo = u, thi = L - (U - u);
    if (thi > L - 1) thi = L - 1;
    const int c0 = blockIdx.y * kFnChunk;
    if (tlo < c0) tlo = c0;
    if (thi > c0 + kFnChunk - 1) thi = c0 + kFnChunk - 1;
    if (tlo > thi) return;
    const int np = H / 128;
    const int y1 = u < U ? refs[(size_t)b * Umax + u] : 0;
    const int q = ctxs[(size_t)b * U1 + u];
    FnLane r;
    fn_load_lane(r, e + (size_t)q * H, Wt, H, y1, np, lane);
    float ae[2 * kFnMaxPairs], a0[2 * kFnMaxPairs], a1[2 * kFnMaxPairs];
#pragma unroll
    for (int i = 0; i < 2 * kFnMaxPairs; ++i) { ae[i] = 0.f; a0[i] = 0.f; a1[i] = 0.f; }
    for (int t = tlo; t <= thi; ++t) {
        float p0, p1;
        if (!fn_marginals(wi, a, bk, N, T, U1, b, t, u, U, p0, p1)) continue;
        const __bf16* ft = f + ((size_t)b * T + t) * H;
#pragma unroll
        for (int j = 0; j < kFnMaxPairs; ++j) {
            if (j < np) {
                const unsigned h = tanh_pair(*(const unsigned*)(ft + 2 * (lane * np + j)), r.e[j]);
                const float h0 = fn_lo(h), h1 = fn_hi(h);
                ae[2 * j] += (p0 * r.w0[2 * j] + p1 * r.w1[2 * j]) * (1.f - h0 * h0);
                ae[2 * j + 1] += (p0 * r.w0[2 * j + 1] + p1 * r.w1[2 * j + 1]) * (1.f - h1 * h1);
                a0[2 * j] += h0 * p0;
                a0[2 * j + 1] += h1 * p0;
                a1[2 * j] += h0 * p1;
                a1[2 * j + 1] += h1 * p1;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kFnMaxPairs; ++j) {
        if (j < np) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int k = 2 * (lane * np + j) + i;
                atomicAdd(de + (size_t)q * H + k, scale * ae[2 * j + i]);
                atomicAdd(dW + (size_t)k * V1, scale * a0[2 * j + i]);
                if (y1 > 0) atomicAdd(dW + (size_t)k * V1 + y1, scale * a1[2 * j + i]);
            }
        }
    }
}

}  // namespace last
