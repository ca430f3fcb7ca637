// Plain streaming kernels of known traffic: a read-only sweep and a copy of a
// buffer.  They are the yardstick the lattice kernels are held against (what
// this GPU streams when nothing else happens) and the calibration of the HBM
// byte counters.  Shapes chosen by measurement on MI355X: 16 bytes per lane,
// every workgroup takes contiguous tiles, non-temporal accesses; the sweep runs
// 8192 workgroups over tiles of 16 KiB (7.1 TB/s), the copy gives every tile of
// 4 KiB a workgroup of its own (6.4 TB/s read + written; grid-stride loops over
// scattered pieces reach 4.3 to 5.4 TB/s).
#pragma once
#include <hip/hip_runtime.h>

namespace last {

typedef float probe_f4 __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 256;
constexpr int kProbeReadUnroll = 4;
constexpr int kProbeReadGrid = 8192;

__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const probe_f4* __restrict__ p, size_t n4,
                                                                    float* __restrict__ sink)
{
    constexpr size_t tile = (size_t)kProbeThreads * kProbeReadUnroll;
    const size_t ntiles = (n4 + tile - 1) / tile;
    probe_f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t base = t * tile + threadIdx.x;
        probe_f4 v[kProbeReadUnroll];
#pragma unroll
        for (int k = 0; k < kProbeReadUnroll; ++k)
            if (base + (size_t)k * kProbeThreads < n4) v[k] = __builtin_nontemporal_load(&p[base + (size_t)k * kProbeThreads]);
#pragma unroll
        for (int k = 0; k < kProbeReadUnroll; ++k)
            if (base + (size_t)k * kProbeThreads < n4) acc += v[k];
    }
    // every load feeds the sum; the sum is stored only for a value no data produces in practice
    const float s = acc.x + acc.y + acc.z + acc.w;
    if (s == -1.2345678e-30f) sink[0] = s;
}

// one workgroup per tile of kProbeThreads * 16 bytes
__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(const probe_f4* __restrict__ src,
                                                                    probe_f4* __restrict__ dst, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * kProbeThreads + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

// The two read patterns of the bigram forward-backward kernel at 256 labels, without its arithmetic: the
// tensor is taken as frames of [257][257] floats; 32 groups of 8 workgroups of 8 waves walk the frames;
// each lane has four 16-byte loads in flight and every element is read once.
//   COLUMNS: workgroup k of a group reads columns 32k .. 32k+31 of every row: pieces of 128 bytes at a
//            stride of 1028 bytes (wave w: rows 32w .. 32w+31, eight rows per instruction);
//   ROWS   : wave w of workgroup k reads rows 1+4u .. 4+4u, u = 8k + w: 4112 contiguous bytes.
// (Row 0 / the last row and column are left out: a yardstick, not a checksum.)
template <bool COLUMNS>
__global__ __launch_bounds__(512) void probe_pattern_kernel(const float* __restrict__ w, int nframes,
                                                            float* __restrict__ sink)
{
    constexpr int C = 257;
    const int k = blockIdx.x & 7, group = blockIdx.x >> 3, ngroups = gridDim.x >> 3;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    probe_f4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int f = group; f < nframes; f += ngroups) {
        const float* fr = w + (size_t)f * C * C;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float* p = COLUMNS ? fr + (size_t)(32 * wave + 8 * j + (lane >> 3)) * C + 32 * k + 4 * (lane & 7)
                                     : fr + (size_t)(1 + 4 * (8 * k + wave) + j) * C + 4 * lane;
            probe_f4 v;
            __builtin_memcpy(&v, p, 16);         // (rows are only 4-byte aligned)
            acc += v;
        }
    }
    const float s = acc.x + acc.y + acc.z + acc.w;
    if (s == -1.2345678e-30f) sink[0] = s;
}

// Where the workgroups of a launch of the cooperating-workgroup shape (one workgroup per compute unit)
// actually run.  Every workgroup writes the XCD it is on (bits 0..3 of its word) and whether it saw all
// workgroups of the launch arrive while it was resident (bit 8): out[blockIdx.x].  The wait is bounded,
// so the kernel ends whatever the placement is.  counter: one word, zero at the start.
__global__ __launch_bounds__(512) void probe_placement_kernel(unsigned* __restrict__ out, unsigned* counter,
                                                              int spin_limit)
{
    if (threadIdx.x != 0) return;
    // hardware register 20 (XCC_ID), bits 0..3: the XCD of this compute unit
    const unsigned xcc = (unsigned)__builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    bool all = false;
    for (int n = 0; n < spin_limit && !all; ++n) {
        all = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= gridDim.x;
        if (!all) __builtin_amdgcn_s_sleep(8);
    }
    out[blockIdx.x] = xcc | (all ? 0x100u : 0u);
}

}  // namespace last
