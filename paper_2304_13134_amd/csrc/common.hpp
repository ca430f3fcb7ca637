// Shared device helpers for the gfx950 lattice kernels: context-dependency
// index arithmetic (the ForwardReduce / BackwardBroadcast primitives of
// Section 3 of arXiv 2304.13134 expressed as closed-form index maps),
// wavefront (64 lanes) and workgroup reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace last {

constexpr int kWave = 64;
#define LAST_NEG_INF (-__builtin_huge_valf())

// Context dependency (Section 3): the full n-gram one of size 1 or 2 in closed form
// (Figure 1a is size 1), or any deterministic automaton given as a next-state table.
struct Ctx {
    int V;      // vocabulary size, labels 1..V, 0 = empty label
    int order;  // context size n (1 or 2); 0 = next-state table
    int C;      // number of context states
    int V1;     // V + 1 labels per state
    const int* nx;  // order 0: device table [C][V], nx[q*V + y-1] = state after label y
};

// destination context state of arc (q, y); the empty label keeps the state
__device__ __forceinline__ int ctx_next(const Ctx& c, int q, int y)
{
    if (y == 0) return q;
    if (c.order == 0) {
        // clamped: a table with an entry that names no state is reported by the check kernel of the
        // call (kItemBadTable); meanwhile nothing may index outside the state vectors
        const unsigned n = (unsigned)c.nx[(size_t)q * c.V + (y - 1)];
        return (int)(n < (unsigned)c.C ? n : (unsigned)(c.C - 1));
    }
    if (c.order == 1) return y;
    if (q == 0) return y;
    if (q <= c.V) return 1 + c.V + (q - 1) * c.V + (y - 1);
    const int b = (q - 1 - c.V) % c.V + 1;
    return 1 + c.V + (b - 1) * c.V + (y - 1);
}

// number of label arcs (y > 0) entering state d
__device__ __forceinline__ int ctx_num_in(const Ctx& c, int d)
{
    if (d == 0) return 0;
    if (c.order == 1) return c.C;
    return d <= c.V ? 1 : c.V + 1;
}

// label carried by every label arc entering state d (d > 0)
__device__ __forceinline__ int ctx_in_label(const Ctx& c, int d)
{
    if (c.order == 1) return d;
    return d <= c.V ? d : (d - 1 - c.V) % c.V + 1;
}

// source state of the i-th label arc entering state d, in increasing state order
__device__ __forceinline__ int ctx_in_source(const Ctx& c, int d, int i)
{
    if (c.order == 1) return i;
    if (d <= c.V) return 0;
    const int b = (d - 1 - c.V) / c.V + 1;
    return i == 0 ? b : 1 + c.V + (i - 1) * c.V + (b - 1);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// reductions inside aligned groups of G lanes (G a power of two <= 64)
template <int G>
__device__ __forceinline__ float group_max(float v)
{
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

template <int G>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Workgroup-wide max / sum; `red` is an LDS array of at least 32 floats.
// Every thread of the workgroup must call; the result is returned to all.
__device__ __forceinline__ float block_max(float v, float* red)
{
    v = wave_max(v);
    const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[wid] = v;
    __syncthreads();
    float r = LAST_NEG_INF;
    for (int i = 0; i < nw; ++i) r = fmaxf(r, red[i]);
    return r;
}

__device__ __forceinline__ float block_sum(float v, float* red)
{
    v = wave_sum(v);
    const int wid = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[wid] = v;
    __syncthreads();
    float r = 0.f;
    for (int i = 0; i < nw; ++i) r += red[i];
    return r;
}

// per-item status codes written to item_status (see last.h)
enum : int { kItemOk = 0, kItemBadLength = 1, kItemBadLabel = 2, kItemBadRefLength = 3,
             kItemInfeasible = 4, kItemTimeout = 5, kItemRange = 6, kItemBadTable = 7 };

}  // namespace last
