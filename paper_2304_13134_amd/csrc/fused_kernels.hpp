// Trigram (context size 2) lattice with arc weights computed on the fly
// (arXiv 2304.13134, Section 4.1: weights are produced frame by frame during
// the topological visit and never stored), for the shared-embedding weight
// function  w[t][q][:] = bf16(tanh(f[t] + e[q])) @ W  with float32 accumulation.
//
// Ownership follows the structure of the full 2-gram context dependency: the
// label arcs into state (b,y) all leave states whose LAST label is b, i.e.
// (b) and (a,b) for every a.  One workgroup per item and last label b owns
// exactly those V+1 source states (plus a private copy of the start state):
//   * their rows of e stay in LDS for the whole pass,
//   * per frame it forms the hidden tile tanh(f_t + e_q) (bf16, in LDS), runs
//     the [rows x hidden] x [hidden x (V+1)] contraction on the matrix cores
//     (v_mfma_f32_16x16x32_bf16; the W fragments live in registers), and feeds
//     the resulting weights straight into the log-sum-exp of the recursion,
//   * the fully reduced forward weight of (b,y) is sent to workgroup y, which
//     owns (b,y) as a source state and adds the empty-label arc itself.
// The per-frame exchange is therefore a V x V transpose between the V
// workgroups of an item (64-bit words [value|tag], agent-scope atomics, bounded
// polls; the workgroups of one item span more than one XCD).
// Values are log-domain float32 relative to a running offset that advances by a
// predicted amount per frame (same predictor as the bigram cluster kernel), so
// magnitudes stay O(10) while log-partition values reach several thousand.
#pragma once
#include <type_traits>

#include "common.hpp"
#include "cluster_kernels.hpp"

namespace last {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

constexpr int kFuThreads = 512;
constexpr int kFuMaxRows = 80;      // V + 2 rows padded to a multiple of 16
constexpr int kFuMaxNT = 5;         // (V + 1) labels in tiles of 16
constexpr int kFuWS = 81;           // row stride of the weight tile in LDS (floats)
constexpr int kFuMaxKS = 16;        // hidden / 32
constexpr int kFuKC = 128;          // hidden units per chunk of the hidden tile (forward kernel)
constexpr int kFuNC = 4;            // chunks (hidden <= 512, a multiple of kFuKC)
constexpr int kFuHS = kFuKC + 8;    // row stride (bf16) of a hidden-tile chunk in LDS
constexpr int kFuHB = kFuMaxRows * kFuHS;   // elements per chunk buffer at most (a kernel with MT row tiles: 16 MT rows)
constexpr int kFuHF = 512 + 8;      // row stride (bf16) of the whole hidden tile (backward kernels)
constexpr int kFuGS = 104;          // row stride (bf16) of the marginal tiles in LDS; 96 used
constexpr int kFuKT = 4;            // 16-wide tiles of the hidden dimension per wave (8 waves x 4 x 16 = 512)
constexpr int kFuER = 9;            // rows of e per thread and frame in the backward kernels

struct FusedArgs {
    const __bf16* f;     // [B][T][H]
    const __bf16* e;     // [C][H]
    const bf16x8* Wf;    // W as operand fragments, see fused_pack_w_kernel
    const int* len;
    float* dist;
    int* item_status;
    float* alpha_ws;     // [B][T+1][C] forward weights relative to offs (null: not stored)
    double* offs;        // [B][T+1] running offset
    float* part;         // [B][V] per-workgroup log-sum-exp of the last frame
    double* Aend;        // [B] running offset of the last frame (NaN for an invalid length)
    u64* xb;             // [ncl][2][V+1][XW] exchange words; row V = headers
    int B, T, V, H, C;
    int ncl, XW;
    int spin_limit;
};


__device__ __forceinline__ float word_value(u64 x) { return __uint_as_float((unsigned)x); }

__device__ __forceinline__ float fast_tanh(float x)
{
    // 1 - 2 / (1 + 2^(2 x log2 e)); saturates correctly at both ends
    const float ex = __builtin_amdgcn_exp2f(x * (2.f * kLog2e));
    return fmaf(-2.f, __builtin_amdgcn_rcpf(1.f + ex), 1.f);
}

__device__ __forceinline__ float log_add_f(float x, float y)
{
    const float m = fmaxf(x, y);
    if (m == LAST_NEG_INF) return m;
    return m + __logf(1.f + __expf(fminf(x, y) - m));
}

// wait (bounded) until the exchange word carries `tag`; x is a first look taken earlier
__device__ __forceinline__ u64 poll_from(const u64* p, u64 x, unsigned tag, int limit, int& dead)
{
    int n = 0;
    while (!dead && (unsigned)(x >> 32) != tag) {
        if (++n > limit) { dead = 1; break; }
        __builtin_amdgcn_s_sleep(1);
        x = xload(p);
    }
    return x;
}

// local row r of workgroup b (1..V): 0 -> start state, 1 -> (b), 1 + a -> (a,b)
__device__ __forceinline__ int fused_state(int V, int b, int r)
{
    if (r == 0) return 0;
    if (r == 1) return b;
    return 1 + V + (r - 2) * V + (b - 1);
}

// two adjacent hidden units at once: bf16 pairs in, tanh in float32, bf16 pair out
__device__ __forceinline__ unsigned tanh_pair(unsigned fbits, unsigned ebits)
{
    const float x0 = __uint_as_float(fbits << 16) + __uint_as_float(ebits << 16);
    const float x1 = __uint_as_float(fbits & 0xffff0000u) + __uint_as_float(ebits & 0xffff0000u);
    const floatx2 h = {fast_tanh(x0), fast_tanh(x1)};
    const bf16x2 r = __builtin_convertvector(h, bf16x2);
    return __builtin_bit_cast(unsigned, r);
}

// workgroup barrier that orders LDS traffic only: global loads issued before it stay in flight
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Contraction of hidden-tile chunk C (static, so that the fragment registers are addressed
// directly).  Label waves (BLANK = false) run the four 32-wide steps of the chunk against their
// 16 labels; the four blank waves share the single empty-label column: wave 4 + i takes step i
// of every chunk (fragment wfrag[C]) and the partial sums are added up later.
template <int MT, int C, bool BLANK>
__device__ __forceinline__ void fused_mfma_chunk(const __bf16* hb, floatx4 (&acc)[MT],
                                                 const bf16x8 (&wfrag)[kFuMaxKS], int kstep)
{
    const int lane = threadIdx.x & 63;
    const __bf16* hp = hb + (lane & 15) * kFuHS + 8 * (lane >> 4);
    if (BLANK) {
        bf16x8 av[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) av[mt] = *(const bf16x8*)&hp[16 * mt * kFuHS + 32 * kstep];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mt], wfrag[C], acc[mt], 0, 0, 0);
    } else {
        // two steps per batch: ten LDS reads in flight, then ten matrix instructions
#pragma unroll
        for (int k2 = 0; k2 < kFuKC / 64; ++k2) {
            bf16x8 av[2][MT];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) av[h][mt] = *(const bf16x8*)&hp[16 * mt * kFuHS + 32 * (2 * k2 + h)];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[h][mt], wfrag[(kFuKC / 32) * C + 2 * k2 + h], acc[mt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Hidden tile + contraction of NF consecutive frames in NC + 1 phases (NC = H / kFuKC).  Phase
// p runs the matrix-core contraction of chunk p-1 and forms the hidden tile
// tanh(f + e) of chunk p, so the transcendental work of one chunk overlaps the
// contraction of the previous one; chunks alternate between two LDS buffers.  With NF = 2
// ("two frames per tile") a row of e is read once for both frames and the phase barriers are
// shared; the frames have their own hidden tiles and accumulators.
// Columns of the weight tile: waves 0..NTL-1 hold labels 16 n + 1 .. 16 n + 16
// (lane l, tile mt, element i -> row 16 mt + 4 (l / 16) + i, label 16 n + l % 16 + 1);
// waves 4..7 hold partial sums of the empty-label column (lanes with l % 16 == 0).
// One contraction wave of each kind per SIMD keeps the matrix cores evenly loaded.
// f_s [NF][H] bf16 (features of the frames), e_s [R][H] bf16, hid_s [2][NF][16 MT][kFuHS]
// bf16 (constant strides keep the LDS addresses of the contraction immediate).
// `early` (may be null): an exchange word this thread will need afterwards; a first
// look at it is issued after phase 1 and returned in `early_word`.
template <int MT, int NF>
__device__ __forceinline__ void fused_weights_phases(const __bf16* f_s, const __bf16* e_s,
                                                     __bf16* hid_s, floatx4 (&acc)[NF][MT],
                                                     const bf16x8 (&wfrag)[kFuMaxKS], int R, int H, int NTL,
                                                     const u64* early, u64& early_word, int p_begin, int p_end)
{
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NC = H / kFuKC;
    const int kp = tid % (kFuKC / 2);                 // 64 pairs of hidden units x 8 waves
    // rows of the tanh pass: the label waves, which carry most of the contraction, take the
    // first RL rows (wave, wave + 4, ...), the other four waves the rest
    const int RL = (3 * R) / 8 & ~3;
    const int r_first = wave < 4 ? wave : RL + (wave - 4);
    const int r_end = wave < 4 ? RL : R;
    // phases p_begin .. p_end of 0 .. NC: phase 0 alone (the hidden tile of the first chunk) leaves the
    // accumulators alone, so it can run while those of the frames before are still in use
    if (p_end >= 1) {
#pragma unroll
        for (int fr = 0; fr < NF; ++fr)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[fr][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll 1
    for (int p = p_begin; p <= p_end; ++p) {
        if (p == 2 && early) early_word = xload(early);
        if (p >= 1) {
#pragma unroll
            for (int fr = 0; fr < NF; ++fr) {
                const __bf16* hb = hid_s + (((p - 1) & 1) * NF + fr) * (16 * MT * kFuHS);
                if (wave >= 4) {
                    switch (p) {
                    case 1: fused_mfma_chunk<MT, 0, true>(hb, acc[fr], wfrag, wave - 4); break;
                    case 2: fused_mfma_chunk<MT, 1, true>(hb, acc[fr], wfrag, wave - 4); break;
                    case 3: fused_mfma_chunk<MT, 2, true>(hb, acc[fr], wfrag, wave - 4); break;
                    default: fused_mfma_chunk<MT, 3, true>(hb, acc[fr], wfrag, wave - 4); break;
                    }
                } else if (wave < NTL) {
                    switch (p) {
                    case 1: fused_mfma_chunk<MT, 0, false>(hb, acc[fr], wfrag, 0); break;
                    case 2: fused_mfma_chunk<MT, 1, false>(hb, acc[fr], wfrag, 0); break;
                    case 3: fused_mfma_chunk<MT, 2, false>(hb, acc[fr], wfrag, 0); break;
                    default: fused_mfma_chunk<MT, 3, false>(hb, acc[fr], wfrag, 0); break;
                    }
                }
            }
        }
        if (p < NC) {
            __bf16* hb = hid_s + (p & 1) * NF * (16 * MT * kFuHS) + 2 * kp;
            unsigned f2[NF];
#pragma unroll
            for (int fr = 0; fr < NF; ++fr) f2[fr] = *(const unsigned*)(f_s + (size_t)fr * H + kFuKC * p + 2 * kp);
            const __bf16* ep = e_s + kFuKC * p + 2 * kp;
            for (int r = r_first; r < r_end; r += 12) {
                // three rows per trip: the LDS reads go out together
                const int r1 = r + 4, r2 = r + 8;
                const unsigned e0 = *(const unsigned*)(ep + (size_t)r * H);
                const unsigned e1 = *(const unsigned*)(ep + (size_t)(r1 < r_end ? r1 : r) * H);
                const unsigned e2 = *(const unsigned*)(ep + (size_t)(r2 < r_end ? r2 : r) * H);
#pragma unroll
                for (int fr = 0; fr < NF; ++fr) {
                    __bf16* hf = hb + fr * (16 * MT * kFuHS);
                    *(unsigned*)(hf + r * kFuHS) = tanh_pair(f2[fr], e0);
                    if (r1 < r_end) *(unsigned*)(hf + r1 * kFuHS) = tanh_pair(f2[fr], e1);
                    if (r2 < r_end) *(unsigned*)(hf + r2 * kFuHS) = tanh_pair(f2[fr], e2);
                }
            }
            lds_barrier();
        }
    }
}

// W repacked as matrix-core operand fragments (one 16-byte load per lane and fragment):
//   Wf [kFuMaxNT][kFuMaxKS][64]: lane l of (n, ks) holds W[32 ks + 8 (l / 16) + j][label], where
//      label = 16 n + l % 16 + 1 for the label tiles n = 0..3 and, for tile 4, the empty label 0
//      in column l % 16 == 0 only (B operand of  w[r][y] = sum_k h[r][k] W[k][y])
//   Wt [H / 16][3][64]:          lane l of (kt, ys) holds W[16 kt + l % 16][32 ys + 8 (l / 16) + j]
//      (B operand of  d[r][k] = sum_y gamma[r][y] W[k][y]),           j = 0..7, zero outside W
__global__ void fused_pack_w_kernel(const __bf16* __restrict__ W, int H, int V1, bf16x8* __restrict__ Wf,
                                    bf16x8* __restrict__ Wt)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int nf = kFuMaxNT * kFuMaxKS * 64;
    if (i < nf) {
        const int lane = i & 63, ks = (i >> 6) % kFuMaxKS, n = (i >> 6) / kFuMaxKS;
        const int y = n < kFuMaxNT - 1 ? 16 * n + (lane & 15) + 1 : ((lane & 15) == 0 ? 0 : V1);
        bf16x8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = 32 * ks + 8 * (lane >> 4) + j;
            v[j] = (k < H && y < V1) ? W[(size_t)k * V1 + y] : (__bf16)0.f;
        }
        Wf[i] = v;
    }
    const int nt = (H / 16) * 3 * 64;
    if (Wt && i < nt) {
        const int lane = i & 63, ys = (i >> 6) % 3, kt = (i >> 6) / 3;
        const int k = 16 * kt + (lane & 15);
        bf16x8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int y = 32 * ys + 8 * (lane >> 4) + j;
            v[j] = (y < V1) ? W[(size_t)k * V1 + y] : (__bf16)0.f;
        }
        Wt[i] = v;
    }
}

// Fragments of W for the forward kernel: waves 0..3 hold all steps of their label tile; wave
// 4 + i holds, for chunk c, the fragment of the empty-label tile for step 4 c + i in wfrag[c].
__device__ __forceinline__ void fused_load_wfrag(const bf16x8* __restrict__ Wf, bf16x8 (&wfrag)[kFuMaxKS])
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int ks = 0; ks < kFuMaxKS; ++ks) {
        const int n = wave < 4 ? wave : kFuMaxNT - 1;
        const int k = wave < 4 ? ks : (kFuKC / 32) * (ks & 3) + (wave - 4);
        wfrag[ks] = Wf[((size_t)n * kFuMaxKS + k) * 64 + lane];
    }
}

// largest forward weight among the own states -> header word of this workgroup (wave 0 only)
__device__ __forceinline__ void fused_publish_header(const float* al, int R, u64* slot, unsigned tag)
{
    const int lane = threadIdx.x;            // caller guarantees threadIdx.x < 64
    float mx = (lane < R) ? al[lane] : LAST_NEG_INF;
    if (lane + 64 < R) mx = fmaxf(mx, al[lane + 64]);
    mx = wave_max_dpp(mx);                   // result broadcast to every lane
    if (lane == 0) xstore(slot, pack_word(mx, tag));
}

// Shortest distance in the log semiring with on-the-fly weights (Eq. 2 visited
// frame by frame, Section 4.1).  Grid: ncl * V workgroups of 512 threads; MT =
// number of 16-row tiles that cover the V + 2 rows of a workgroup; NF = frames whose
// weights are computed at a time (1 or 2).
// Per frame: the waves that hold the weight tile reduce the label arcs of the
// own rows column by column in registers and publish the V partial values; the
// weights of the NEXT NF frames (independent of the recursion) are then computed
// while those words travel (NF = 2: after the second frame of a group; the exchange of
// the first one is waited for); finally the own states are assembled from what the
// other workgroups sent.
template <int MT, int NF>
__global__ __launch_bounds__(kFuThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_forward_kernel(FusedArgs a)
{
    extern __shared__ unsigned char smem_raw[];
    const int V = a.V, H = a.H, R = V + 2;
    const int NTL = (V + 15) / 16;                                   // label tiles (waves 0..NTL-1)
    __bf16* e_s = (__bf16*)smem_raw;                                  // [R][H]
    __bf16* hid_s = e_s + (size_t)R * H;                              // [2][NF][16 MT][kFuHS]
    static_assert(NF == 1 || NF == 2, "the forward weights of a group's frames sit in two LDS rows");
    float* al_s = (float*)(hid_s + 2 * NF * (16 * MT * kFuHS));       // [2][kFuMaxRows] forward weights
    float* pb_s = al_s + 2 * kFuMaxRows;                              // [4][kFuMaxRows] partial empty-label weights
    float* sa_s = pb_s + 4 * kFuMaxRows;                              // [8] label arc start -> (b)
    float* red = sa_s + 8;                                            // [32]
    int* ctl_s = (int*)(red + 32);                                    // [8]
    __bf16* f_s = (__bf16*)(ctl_s + 8);                               // [NF][H] features of the frames being prepared

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cl = blockIdx.x / V, b = blockIdx.x % V + 1;
    // zero the pad rows of the hidden tile once; they stay zero
    for (int i = tid; i < 2 * NF * (16 * MT * kFuHS); i += kFuThreads) hid_s[i] = (__bf16)0.f;
    // rows of e owned by this workgroup
    for (int i = tid; i < R * H; i += kFuThreads) {
        const int r = i / H, k = i - r * H;
        e_s[i] = a.e[(size_t)fused_state(V, b, r) * H + k];
    }
    bf16x8 wfrag[kFuMaxKS];
    fused_load_wfrag(a.Wf, wfrag);
    floatx4 acc[NF][MT];
    unsigned gstep = 0;
    __syncthreads();

    for (int item = cl; item < a.B; item += a.ncl) {
        int L = a.len[item];
        const bool bad = L < 0 || L > a.T;
        if (bad) L = 0;
        u64* xbase = a.xb + (size_t)cl * 2 * (V + 1) * a.XW;
        float* aws = a.alpha_ws ? a.alpha_ws + (size_t)item * (a.T + 1) * a.C : nullptr;
        const __bf16* fi = a.f + (size_t)item * a.T * H;
        if (tid < 2 * kFuMaxRows) al_s[tid] = (tid == 0) ? 0.f : LAST_NEG_INF;
        if (tid == 0) ctl_s[0] = 0;
        __syncthreads();
        if (aws && tid < R && (tid > 0 || b == 1)) aws[fused_state(V, b, tid)] = al_s[tid];
        if (a.offs && b == 1 && tid == 0) a.offs[(size_t)item * (a.T + 1)] = 0.0;
        double A = 0.0;                       // running offset, identical in every workgroup
        double A_at[2] = {0.0, 0.0};          // ... after frame s - 1, at [s & 1], for the two newest s
        float P_cur = 0.f, P_prev = 0.f, mu_prev = 0.f;
        int dead = 0;
        int kept = 0;                         // forward weights of frames 0 .. kept are in the workspace
        // The forward weights kept for the backward pass leave LDS once per group, right before the weights
        // of the next group are computed: a look at the exchange waits for every store the wave issued
        // before it, and there the next look is furthest away.
        auto keep = [&](int upto) __attribute__((always_inline)) {
            for (int sfr = kept + 1; sfr <= upto; ++sfr) {
                if (aws && tid < R && (tid > 0 || b == 1))
                    aws[(size_t)sfr * a.C + fused_state(V, b, tid)] = al_s[(sfr & 1) * kFuMaxRows + tid];
                if (a.offs && b == 1 && tid == 0) a.offs[(size_t)item * (a.T + 1) + sfr] = A_at[sfr & 1];
            }
            kept = max(kept, upto);
        };
        if (L > 0 && wave == 0)
            fused_publish_header(al_s, R, xbase + (size_t)(gstep & 1) * (V + 1) * a.XW + (size_t)V * a.XW + (b - 1),
                                 gstep + 1);
        // frame features travel two groups ahead: register (group g + 2) -> LDS (group g + 1)
        unsigned fnext[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j)
            fnext[j] = (2 * tid < H && L > 0) ? *(const unsigned*)(fi + (size_t)(j < L ? j : L - 1) * H + 2 * tid) : 0u;
        // frames are taken in groups of NF; group -1 only computes the weights of the first NF frames
        for (int t0 = (L > 0 ? -NF : 0); t0 < L; t0 += NF) {
            if (2 * tid < H) {
#pragma unroll
                for (int j = 0; j < NF; ++j) {
                    const int tn = t0 + 2 * NF + j;
                    *(unsigned*)(f_s + (size_t)j * H + 2 * tid) = fnext[j];
                    fnext[j] = *(const unsigned*)(fi + (size_t)(tn < L ? tn : L - 1) * H + 2 * tid);
                }
            }
            bool pre = false;                                // phase 0 of the next group's weights is done
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const int t = t0 + j;
                const bool live = t >= 0 && t < L;           // (the same in every thread of the item's workgroups)
                const int par = t & 1;
                const float* al = al_s + par * kFuMaxRows;
                float* an = al_s + (par ^ 1) * kFuMaxRows;
                const unsigned tag = gstep + 1;
                u64* xs = xbase + (size_t)(gstep & 1) * (V + 1) * a.XW;
                // label arcs (b), (a,b) --y--> (b,y): reduced over the own rows, sent to workgroup y
                if (live && wave < NTL) {
                    const int g = lane >> 4, y = 16 * wave + (lane & 15) + 1;
                    float v[MT][4];
                    float m = LAST_NEG_INF;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const floatx4 a4 = *(const floatx4*)&al[16 * mt + 4 * g];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int row = 16 * mt + 4 * g + i;
                            v[mt][i] = (row >= 1 && row < R) ? a4[i] + acc[j][mt][i] : LAST_NEG_INF;
                            m = fmaxf(m, v[mt][i]);
                        }
                    }
                    const float v00 = al[0] + acc[j][0][0];       // row 0 (lanes with g == 0): start --y--> (y)
                    m = fmaxf(m, __shfl_xor(m, 16));
                    m = fmaxf(m, __shfl_xor(m, 32));
                    const float ms = (m == LAST_NEG_INF) ? 0.f : m;
                    float sum = 0.f;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int i = 0; i < 4; ++i) sum += __expf(v[mt][i] - ms);
                    sum += __shfl_xor(sum, 16);
                    sum += __shfl_xor(sum, 32);
                    const float p = (m != LAST_NEG_INF) ? m + __logf(sum) - P_cur : LAST_NEG_INF;
                    if (g == 0 && y <= V) xstore(xs + (size_t)(y - 1) * a.XW + (b - 1), pack_word(p, tag));
                    if (g == 0 && y == b) sa_s[0] = v00 - P_cur;
                } else if (live && wave >= 4) {
                    // partial empty-label weights of the own rows
                    if ((lane & 15) == 0) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                pb_s[(wave - 4) * kFuMaxRows + 16 * mt + 4 * (lane >> 4) + i] = acc[j][mt][i];
                    }
                }
                lds_barrier();
                // after the last frame of the group: the weights of the next group while the partial values
                // travel; the first look at the incoming words is issued half way and consumed afterwards
                const u64* pw = nullptr;
                if (live) {
                    if (tid >= 1 && tid <= V) pw = xs + (size_t)(b - 1) * a.XW + (tid - 1);
                    else if (tid >= 128 && tid < 128 + V) pw = xs + (size_t)V * a.XW + (tid - 128);
                }
                u64 x = 0;
                if (j == NF - 1) keep(min(t0 + NF - 1, L));
                if (j == NF - 1 && t0 + NF < L) {
                    fused_weights_phases<MT, NF>(f_s, e_s, hid_s, acc, wfrag, R, H, NTL, pw, x, pre ? 1 : 0, H / kFuKC);
                } else {
                    // not the last frame of the group: its exchange is waited for in the open; the first
                    // phase of the next group's weights (tanh only, no accumulator) fills part of the wait
                    if (NF > 1 && live && j == 0 && t0 + NF < L) {
                        u64 unused = 0;
                        fused_weights_phases<MT, NF>(f_s, e_s, hid_s, acc, wfrag, R, H, NTL, nullptr, unused, 0, 0);
                        pre = true;
                    }
                    if (pw) x = xload(pw);
                }
                if (!live) continue;
                // gather: (a,b) receives its label-arc part from workgroup a; headers from everybody
                float hv = LAST_NEG_INF;
                if (pw) x = poll_from(pw, x, tag, a.spin_limit, dead);
                // empty-label arc of own row r: alpha[r] + w[r][0]
                auto blank = [&](int r) {
                    return al[r] + ((pb_s[r] + pb_s[kFuMaxRows + r]) + (pb_s[2 * kFuMaxRows + r] + pb_s[3 * kFuMaxRows + r])) - P_cur;
                };
                if (tid >= 1 && tid <= V) {
                    an[1 + tid] = log_add_f(word_value(x), blank(1 + tid));
                } else if (tid == 0) {
                    an[0] = blank(0);
                    an[1] = log_add_f(sa_s[0], blank(1));
                } else if (pw) {
                    hv = word_value(x);
                }
                // the header words all sit in wave 2: their maximum goes through LDS; one barrier
                // publishes it together with the new forward weights
                if (wave == 2) {
                    const float hm = wave_max_dpp(hv);
                    if (lane == 0) red[0] = hm;
                }
                if (dead) ctl_s[0] = 1;
                lds_barrier();
                const float mu = red[0];
                // offset bookkeeping, identical everywhere
                const float G = mu - mu_prev + P_prev;
                const float P_next = mu + 2.f * G - P_cur;
                A += (double)P_cur;
                A_at[(t + 1) & 1] = A;
                mu_prev = mu; P_prev = P_cur; P_cur = P_next;
                gstep += 1;
                if (wave == 0 && t + 1 < L)
                    fused_publish_header(an, R, xbase + (size_t)(gstep & 1) * (V + 1) * a.XW + (size_t)V * a.XW + (b - 1),
                                         gstep + 1);
            }
        }
        keep(L);
        // all states of the last frame are final: per-workgroup log-sum-exp, combined by fused_finalize
        {
            const float* al = al_s + (L & 1) * kFuMaxRows;
            const bool mine = tid < R && (tid > 0 || b == 1);
            float v = mine ? al[tid] : LAST_NEG_INF;
            const float mx = block_max(v, red);
            float s = (mine && mx != LAST_NEG_INF) ? __expf(v - mx) : 0.f;
            s = block_sum(s, red);
            if (tid == 0) {
                // a workgroup that gave up waiting marks its part: the item's distance becomes NaN
                a.part[(size_t)item * V + (b - 1)] = ctl_s[0] ? __builtin_nanf("")
                                                     : (mx == LAST_NEG_INF) ? LAST_NEG_INF : mx + __logf(s);
                if (b == 1) {
                    a.Aend[item] = bad ? __builtin_nan("") : A;
                    if (a.item_status) a.item_status[item] = bad ? kItemBadLength : (ctl_s[0] ? kItemTimeout : kItemOk);
                }
            }
        }
        __syncthreads();
    }
}

// D[item] = offset + log-sum-exp over the workgroups' partial values; NaN and status 5 when a
// workgroup of the item timed out (its part is NaN)
__global__ void fused_finalize_kernel(const float* __restrict__ part, const double* __restrict__ Aend,
                                      int B, int V, float* __restrict__ dist, double* __restrict__ Dws,
                                      int* __restrict__ item_status)
{
    const int item = blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= B) return;
    const double A = Aend[item];
    float mx = LAST_NEG_INF;
    bool tmo = false;
    for (int j = 0; j < V; ++j) {
        const float p = part[(size_t)item * V + j];
        tmo = tmo || p != p;
        mx = fmaxf(mx, p);
    }
    float s = 0.f;
    for (int j = 0; j < V; ++j) s += expf(part[(size_t)item * V + j] - mx);
    const double D = (A != A || tmo) ? __builtin_nan("") : A + (double)mx + (double)logf(s);
    dist[item] = (float)D;
    if (Dws) Dws[item] = D;
    if (tmo && A == A && item_status) item_status[item] = kItemTimeout;
}

// ---------------------------------------------------------------------------
// Backward side: beta recursion, arc marginals (Eq. 1) and their chain through
// the weight function.  With h = bf16(tanh(f_t + e_q)) and gamma the marginals,
//   dW[k][y] += h[k] gamma[q][y],   dpre[q][k] = (sum_y gamma[q][y] W[k][y]) (1 - h[k]^2),
//   de[q][k] += dpre[q][k],         df[t][k]   += sum_q dpre[q][k]
// (the rounding of h is treated as the identity when differentiating).
// gamma is split into two bf16 halves (hi + lo) so that the matrix-core
// contractions keep 16 significant bits of it.
// ---------------------------------------------------------------------------

struct FusedBwdArgs {
    const __bf16* f;
    const __bf16* e;
    const bf16x8* Wf;        // W as operand fragments, see fused_pack_w_kernel
    const bf16x8* Wt;
    const int* len;
    const float* alpha_ws;   // [B][T+1][C] forward weights relative to offs
    const double* offs;      // [B][T+1]
    const double* Dws;       // [B] shortest distance
    float* beta_ws;          // [B][T+1][C] backward weights relative to (D - offs)
    __bf16* gamma_ws;        // null, or [B][T][V][2][V+2][P] the marginals of every frame as two bf16 halves
                             // (hi plane, lo plane; P = V + 1 rounded up to a multiple of 8), written by the
                             // backward kernel for the dW kernel
    float* df;               // [B][T][H]
    float* de;               // [C][H]
    float* dW;               // [H][V+1]
    float scale;
    int* item_status;
    float* dist;             // [B]: set to NaN for an item on which a workgroup gave up waiting
    u64* xb;
    int B, T, V, H, C;
    int ncl, XW;
    int spin_limit;
    int nch, TC;             // frame chunks of the dW kernel
};

// Rows of e for one frame of a backward kernel, fetched from global memory (e
// stays in L2): thread -> 8 adjacent hidden units (one 16-byte load) of rows
// rg, rg + nrg, ...; all loads of a frame are issued together.
struct FusedERows {
    uintx4 v[kFuER];
};

__device__ __forceinline__ void fused_load_e(const __bf16* __restrict__ e, int V, int b, int R, int H,
                                             FusedERows& er)
{
    // lane -> hidden units 8 lane .. 8 lane + 7 (idle when beyond H), wave -> rows wave, wave + 8, ...
    const int kg = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int kc = 8 * kg < H ? 8 * kg : 0;
#pragma unroll
    for (int i = 0; i < kFuER; ++i) {
        const int r = rg + 8 * i;
        er.v[i] = *(const uintx4*)(e + (size_t)fused_state(V, b, r < R ? r : 0) * H + kc);
    }
}

// Hidden tile over the whole hidden dimension (kept for the gradient
// contractions) + weights of one frame into w_s.  hid_s [.][kFuHF] bf16, rows
// >= R stay zero.
// hidden tile tanh(f_t + e) of one frame over the whole hidden dimension (no barrier)
__device__ __forceinline__ void fused_hidden_full(const __bf16* __restrict__ ft, const FusedERows& er,
                                                  __bf16* hid_s, int R, int H)
{
    const int kg = threadIdx.x & 63;
    const int rg = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));     // same mapping as fused_load_e
    if (8 * kg < H) {
        const uintx4 f4 = *(const uintx4*)(ft + 8 * kg);
        __bf16* hw = hid_s + rg * kFuHF + 8 * kg;
#pragma unroll
        for (int i = 0; i < kFuER; ++i) {
            const int r = rg + 8 * i;
            if (r < R) {
                uintx4 h;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // opaque copy: keeps the unpacking of the (frame-invariant) rows of e inside the frame
                    // loop; hoisted, the unpacked values would double the registers they take
                    unsigned eb = er.v[i][j];
                    asm volatile("" : "+v"(eb));
                    h[j] = tanh_pair(f4[j], eb);
                }
                *(uintx4*)(hw + 8 * i * kFuHF) = h;
            }
        }
    }
}

template <int MT>
__device__ __forceinline__ void fused_weights_full(const __bf16* __restrict__ ft, const FusedERows& er,
                                                   __bf16* hid_s, float* w_s, const bf16x8* __restrict__ Wf,
                                                   int R, int H, int NTL, const u64* early, u64& early_word)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // contraction waves: 0..NTL-1 -> label tiles, 4 -> the empty-label column.  Their fragments
    // of W are fetched per frame and chunk (L2), one chunk ahead, so that few of them are live.
    const bool mm = wave < NTL || wave == 4;
    const bf16x8* wp = Wf + (size_t)wave * kFuMaxKS * 64 + lane;
    bf16x8 wcur[kFuKC / 32];
    if (mm) {
#pragma unroll
        for (int ks = 0; ks < kFuKC / 32; ++ks) wcur[ks] = wp[ks * 64];
    }
    fused_hidden_full(ft, er, hid_s, R, H);
    lds_barrier();
    if (early) early_word = xload(early);        // first look at the exchange word, consumed by the caller
    if (mm) {
        floatx4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
        const __bf16* hp = hid_s + (lane & 15) * kFuHF + 8 * (lane >> 4);
#pragma unroll
        for (int c = 0; c < kFuNC; ++c)
            if (kFuKC * c < H) {
                bf16x8 wnext[kFuKC / 32];
                if (kFuKC * (c + 1) < H) {
#pragma unroll
                    for (int ks = 0; ks < kFuKC / 32; ++ks) wnext[ks] = wp[((kFuKC / 32) * (c + 1) + ks) * 64];
                }
#pragma unroll
                for (int ks = 0; ks < kFuKC / 32; ++ks) {
                    bf16x8 av[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) av[mt] = *(const bf16x8*)&hp[16 * mt * kFuHF + kFuKC * c + 32 * ks];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mt], wcur[ks], acc[mt], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int ks = 0; ks < kFuKC / 32; ++ks) wcur[ks] = wnext[ks];
            }
        const int y = wave < 4 ? 16 * wave + (lane & 15) + 1 : 0;
        if (wave < 4 || (lane & 15) == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) w_s[(16 * mt + 4 * (lane >> 4) + r) * kFuWS + y] = acc[mt][r];
        }
    }
    lds_barrier();
}

__device__ __forceinline__ void split_bf16(float g, __bf16& hi, __bf16& lo)
{
    hi = (__bf16)g;
    lo = (__bf16)(g - (float)hi);
}

// Marginals of one frame for the rows of this workgroup and the backward
// weights of the frame before: v[r][y] = w[r][y] + beta'[next(r,y)] - P,
// beta_t[r] = logsumexp_y v[r][y], gamma[r][y] = exp(alpha'_t[r] + v[r][y]).
// TRANSPOSED selects the LDS layout of gamma: [r][y] (false) or [y][r] (true).
template <bool TRANSPOSED>
__device__ __forceinline__ void fused_rows(const float* w_s, const float* bl, const float* bn_s,
                                           const float* bs_s, const float* aw_s, float P, int V, int R,
                                           bool own_start, float* bl_new, __bf16* gh_s, __bf16* gl_s)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (int r = wave; r < R; r += kFuThreads / 64) {
        const bool valid = r > 0 || own_start;
        const float* nb = (r == 0) ? bs_s : bn_s;
        const int y0 = lane, y1 = lane + 64;
        float v0 = LAST_NEG_INF, v1 = LAST_NEG_INF;
        if (y0 <= V) v0 = w_s[r * kFuWS + y0] + (y0 == 0 ? bl[r] : nb[y0]) - P;
        if (y1 <= V) v1 = w_s[r * kFuWS + y1] + nb[y1] - P;
        const float m = wave_max_dpp(fmaxf(v0, v1));        // result broadcast to every lane
        float sum = (y0 <= V ? __expf(v0 - m) : 0.f) + (y1 <= V ? __expf(v1 - m) : 0.f);
        sum = wave_sum_dpp(sum);
        if (bl_new && lane == 0) bl_new[r] = valid ? m + __logf(sum) : LAST_NEG_INF;
        const float ar = aw_s[r];
        const float g0 = (valid && y0 <= V) ? __expf(ar + v0) : 0.f;
        const float g1 = (valid && y1 <= V) ? __expf(ar + v1) : 0.f;
        __bf16 hi, lo;
        if (y0 <= V) {
            split_bf16(g0, hi, lo);
            const int idx = TRANSPOSED ? y0 * kFuGS + r : r * kFuGS + y0;
            gh_s[idx] = hi; gl_s[idx] = lo;
        }
        if (y1 <= V) {
            split_bf16(g1, hi, lo);
            const int idx = TRANSPOSED ? y1 * kFuGS + r : r * kFuGS + y1;
            gh_s[idx] = hi; gl_s[idx] = lo;
        }
    }
}

// Backward recursion over the same ownership as the forward kernel.  What a
// workgroup needs from the others per frame is beta_{t+1}[(b,y)] for every y
// (state (b,y) is a row of workgroup y), again a V x V transpose; workgroup 1,
// which also differentiates the start state, additionally needs beta_{t+1}[(y)].
// Backward weights are kept relative to D - offs[t], which bounds
// alpha' + beta' <= 0, so no offset has to be negotiated.  Also forms
// dpre = (gamma W^T)(1 - h^2) on the matrix cores, accumulates de in registers
// and adds the column sums into df.
template <int MT>
__global__ __launch_bounds__(kFuThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_backward_kernel(FusedBwdArgs a)
{
    extern __shared__ unsigned char smem_raw[];
    const int V = a.V, V1 = V + 1, H = a.H, R = V + 2;
    const int NTL = (V + 15) / 16;
    __bf16* hid_s = (__bf16*)smem_raw;                                // [kFuMaxRows][kFuHF]
    float* w_s = (float*)(hid_s + (size_t)kFuMaxRows * kFuHF);        // [kFuMaxRows][kFuWS]
    __bf16* gh_s = (__bf16*)(w_s + (size_t)kFuMaxRows * kFuWS);       // [kFuMaxRows][kFuGS]
    __bf16* gl_s = gh_s + (size_t)kFuMaxRows * kFuGS;
    float* bl_s = (float*)(gl_s + (size_t)kFuMaxRows * kFuGS);        // [2][kFuMaxRows]
    float* bn_s = bl_s + 2 * kFuMaxRows;                              // [kFuMaxRows]
    float* bs_s = bn_s + kFuMaxRows;                                  // [kFuMaxRows]
    float* aw_s = bs_s + kFuMaxRows;                                  // [kFuMaxRows]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cl = blockIdx.x / V, b = blockIdx.x % V + 1;
    for (int i = tid; i < kFuMaxRows * kFuHF; i += kFuThreads) hid_s[i] = (__bf16)0.f;
    for (int i = tid; i < 2 * kFuMaxRows * kFuGS; i += kFuThreads) gh_s[i] = (__bf16)0.f;
    if (tid < kFuMaxRows) { bn_s[tid] = 0.f; bs_s[tid] = 0.f; aw_s[tid] = LAST_NEG_INF; }
    floatx4 de_acc[kFuKT][MT];
#pragma unroll
    for (int kt = 0; kt < kFuKT; ++kt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) de_acc[kt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    // the rows of e of this workgroup do not change from frame to frame: they stay in registers
    FusedERows er;
    fused_load_e(a.e, V, b, R, H, er);
    unsigned gstep = 0;
    __syncthreads();

    for (int item = cl; item < a.B; item += a.ncl) {
        int L = a.len[item];
        if (L < 0 || L > a.T) L = 0;
        if (L == 0) continue;
        u64* xbase = a.xb + (size_t)cl * 2 * (V + 1) * a.XW;
        const float* aws = a.alpha_ws + (size_t)item * (a.T + 1) * a.C;
        float* bws = a.beta_ws + (size_t)item * (a.T + 1) * a.C;
        const double* offs = a.offs + (size_t)item * (a.T + 1);
        const float init = (float)(offs[L] - a.Dws[item]);       // beta_L = 0 for every state
        if (tid < kFuMaxRows) bl_s[tid] = (tid < R) ? init : LAST_NEG_INF;
        if (tid < R && (tid > 0 || b == 1)) bws[(size_t)L * a.C + fused_state(V, b, tid)] = init;
        int dead = 0, any_dead = 0;
        __syncthreads();
        for (int t = L - 1; t >= 0; --t) {
            const int par = (L - 1 - t) & 1;
            const float* bl = bl_s + par * kFuMaxRows;
            float* bl_new = bl_s + (par ^ 1) * kFuMaxRows;
            const unsigned tag = gstep + 1;
            u64* xs = xbase + (size_t)(gstep & 1) * (V + 1) * a.XW;
            // publish beta_{t+1}: state (a,b) goes to workgroup a, state (b) to workgroup 1
            if (tid >= 1 && tid <= V) xstore(xs + (size_t)(tid - 1) * a.XW + (b - 1), pack_word(bl[1 + tid], tag));
            else if (tid == V + 1) xstore(xs + (size_t)V * a.XW + (b - 1), pack_word(bl[1], tag));
            if (tid < R) aw_s[tid] = aws[(size_t)t * a.C + fused_state(V, b, tid)];
            const u64* pw = nullptr;
            if (tid >= 1 && tid <= V) pw = xs + (size_t)(b - 1) * a.XW + (tid - 1);
            else if (b == 1 && tid >= 128 && tid < 128 + V) pw = xs + (size_t)V * a.XW + (tid - 128);
            u64 x = 0;
            fused_weights_full<MT>(a.f + ((size_t)item * a.T + t) * H, er, hid_s, w_s, a.Wf, R, H, NTL, pw, x);
            if (pw) x = poll_from(pw, x, tag, a.spin_limit, dead);
            if (tid >= 1 && tid <= V) bn_s[tid] = word_value(x);
            else if (pw) bs_s[tid - 127] = word_value(x);
            const float P = (float)(offs[t + 1] - offs[t]);
            if (__syncthreads_or(dead)) any_dead = 1;
            // fragments of W for the dpre contraction: the first column tile is requested now and used after
            // the row pass, every further one while its predecessor is being used (all of them at once cost
            // 48 registers, which this kernel then spills)
            bf16x8 wt[2][3];
#pragma unroll
            for (int ys = 0; ys < 3; ++ys)
                wt[0][ys] = a.Wt[((size_t)min(kFuKT * wave, H / 16 - 1) * 3 + ys) * 64 + lane];
            fused_rows<false>(w_s, bl, bn_s, bs_s, aw_s, P, V, R, b == 1, bl_new, gh_s, gl_s);
            lds_barrier();
            if (tid < R && (tid > 0 || b == 1)) bws[(size_t)t * a.C + fused_state(V, b, tid)] = bl_new[tid];
            if (a.gamma_ws) {
                // the marginals of the frame for the dW kernel, so that it need not evaluate the weights again:
                // both bf16 planes, rows of P values, 16 bytes at a time
                const int P8 = (V1 + 7) / 8, per_plane = R * P8;
                uintx4* gout = (uintx4*)(a.gamma_ws + (((size_t)item * a.T + t) * V + (b - 1)) * 2 * R * 8 * P8);
                for (int i = tid; i < 2 * per_plane; i += kFuThreads) {
                    const int plane = i >= per_plane ? 1 : 0, k = i - plane * per_plane;
                    const int r = k / P8, c8 = k - r * P8;
                    gout[i] = *(const uintx4*)((plane ? gl_s : gh_s) + r * kFuGS + 8 * c8);
                }
            }
            // dpre = (gamma W^T) (1 - h^2): this wave owns hidden units [64 wave, 64 wave + 64)
            float* dft = a.df + ((size_t)item * a.T + t) * H;
#pragma unroll
            for (int kt = 0; kt < kFuKT; ++kt) {
                const int k0 = 16 * (kFuKT * wave + kt);
                if (kt + 1 < kFuKT) {
#pragma unroll
                    for (int ys = 0; ys < 3; ++ys)
                        wt[(kt + 1) & 1][ys] = a.Wt[((size_t)min(kFuKT * wave + kt + 1, H / 16 - 1) * 3 + ys) * 64 + lane];
                }
                if (k0 < H) {
                    float colsum = 0.f;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ys = 0; ys < 3; ++ys)
                            if (32 * ys < V1) {
                                const int off = (16 * mt + (lane & 15)) * kFuGS + 32 * ys + 8 * (lane >> 4);
                                const bf16x8 ah = *(const bf16x8*)&gh_s[off];
                                const bf16x8 al = *(const bf16x8*)&gl_s[off];
                                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, wt[kt & 1][ys], acc, 0, 0, 0);
                                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, wt[kt & 1][ys], acc, 0, 0, 0);
                            }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float h = (float)hid_s[(16 * mt + 4 * (lane >> 4) + i) * kFuHF + k0 + (lane & 15)];
                            const float d = acc[i] * (1.f - h * h);
                            de_acc[kt][mt][i] += d;
                            colsum += d;
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    colsum += __shfl_xor(colsum, 16);
                    colsum += __shfl_xor(colsum, 32);
                    if (lane < 16) unsafeAtomicAdd(dft + k0 + lane, a.scale * colsum);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            gstep += 1;
            lds_barrier();
        }
        // any workgroup that gave up waiting voids the item (its gradients are wrong): status 5, dist NaN
        if (any_dead && tid == 0 && a.len[item] >= 0 && a.len[item] <= a.T) {
            if (a.item_status)
                __hip_atomic_store(a.item_status + item, (int)kItemTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.dist + item, __builtin_nanf(""), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // de: rows of different clusters (items) add up
#pragma unroll
    for (int kt = 0; kt < kFuKT; ++kt) {
        const int k0 = 16 * (kFuKT * wave + kt);
        if (k0 < H) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 16 * mt + 4 * (lane >> 4) + i;
                    if (r < R && (r > 0 || b == 1))
                        unsafeAtomicAdd(a.de + (size_t)fused_state(V, b, r) * H + k0 + (lane & 15),
                                        a.scale * de_acc[kt][mt][i]);
                }
        }
    }
}

// h^T gamma of one frame added to the accumulators of this wave (hidden units [64 wave, 64 wave + 64), all
// labels): row step by row step, the h^T fragments of the wave's four column tiles are formed once, every
// gamma fragment ([y][r] layout, two bf16 halves) is read once and meets all four.
template <int MT>
__device__ __forceinline__ void fused_dw_accumulate(const __bf16* hid_s, const __bf16* gh_s, const __bf16* gl_s,
                                                    floatx4 (&acc)[kFuKT][kFuMaxNT], int NT, int H)
{
    constexpr int RS = (16 * MT + 31) / 32;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (16 * kFuKT * wave < H) {
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            bf16x8 hv[kFuKT];
#pragma unroll
            for (int kt = 0; kt < kFuKT; ++kt)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    hv[kt][j] = hid_s[(32 * rs + 8 * (lane >> 4) + j) * kFuHF + 16 * (kFuKT * wave + kt) + (lane & 15)];
#pragma unroll
            for (int yt = 0; yt < kFuMaxNT; ++yt)
                if (yt < NT) {
                    const int off = (16 * yt + (lane & 15)) * kFuGS + 32 * rs + 8 * (lane >> 4);
                    const bf16x8 gh = *(const bf16x8*)&gh_s[off];
                    const bf16x8 gl = *(const bf16x8*)&gl_s[off];
#pragma unroll
                    for (int kt = 0; kt < kFuKT; ++kt) {
                        acc[kt][yt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hv[kt], gh, acc[kt][yt], 0, 0, 0);
                        acc[kt][yt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hv[kt], gl, acc[kt][yt], 0, 0, 0);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}
// the accumulators of a workgroup added to dW (workgroups of other items, labels and frame chunks add theirs)
__device__ __forceinline__ void fused_dw_flush(const floatx4 (&acc)[kFuKT][kFuMaxNT], float* dW, float scale,
                                               int NT, int H, int V1)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
#pragma unroll
    for (int kt = 0; kt < kFuKT; ++kt) {
        const int k0 = 16 * (kFuKT * wave + kt);
        if (k0 < H) {
#pragma unroll
            for (int yt = 0; yt < kFuMaxNT; ++yt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = k0 + 4 * (lane >> 4) + i, y = 16 * yt + (lane & 15);
                    if (yt < NT && y < V1) unsafeAtomicAdd(dW + (size_t)k * V1 + y, scale * acc[kt][yt][i]);
                }
        }
    }
}

// dW = sum over items, frames and states of h^T gamma.  No recursion: grid =
// B * V * nch workgroups, each owning the rows of one last label b of one item
// over one chunk of frames; the marginals are rebuilt from the stored forward
// and backward weights and the recomputed weights of the frame.
template <int MT>
__global__ __launch_bounds__(kFuThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_dw_kernel(FusedBwdArgs a)
{
    extern __shared__ unsigned char smem_raw[];
    const int V = a.V, V1 = V + 1, H = a.H, R = V + 2;
    const int NT = (V1 + 15) / 16;
    constexpr int RS = (16 * MT + 31) / 32;                           // 32-row steps of the contraction
    constexpr int kRows = 32 * RS;
    __bf16* hid_s = (__bf16*)smem_raw;                                // [kRows][kFuHF]
    float* w_s = (float*)(hid_s + (size_t)kRows * kFuHF);             // [kFuMaxRows][kFuWS]
    __bf16* gh_s = (__bf16*)(w_s + (size_t)kFuMaxRows * kFuWS);       // [kFuMaxRows (y)][kFuGS (r)]
    __bf16* gl_s = gh_s + (size_t)kFuMaxRows * kFuGS;
    float* bl_s = (float*)(gl_s + (size_t)kFuMaxRows * kFuGS);        // [kFuMaxRows]
    float* bn_s = bl_s + kFuMaxRows;
    float* bs_s = bn_s + kFuMaxRows;
    float* aw_s = bs_s + kFuMaxRows;

    const int tid = threadIdx.x;
    const int ch = blockIdx.x % a.nch;
    const int b = (blockIdx.x / a.nch) % V + 1;
    const int item = blockIdx.x / (a.nch * V);
    int L = a.len[item];
    if (L < 0 || L > a.T) L = 0;
    const int t0 = ch * a.TC, t1 = min(L, t0 + a.TC);
    if (t0 >= t1) return;
    for (int i = tid; i < kRows * kFuHF; i += kFuThreads) hid_s[i] = (__bf16)0.f;
    for (int i = tid; i < 2 * kFuMaxRows * kFuGS; i += kFuThreads) gh_s[i] = (__bf16)0.f;
    if (tid < kFuMaxRows) { bl_s[tid] = 0.f; bn_s[tid] = 0.f; bs_s[tid] = 0.f; aw_s[tid] = LAST_NEG_INF; }
    floatx4 acc[kFuKT][kFuMaxNT];
#pragma unroll
    for (int kt = 0; kt < kFuKT; ++kt)
#pragma unroll
        for (int yt = 0; yt < kFuMaxNT; ++yt) acc[kt][yt] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float* aws = a.alpha_ws + (size_t)item * (a.T + 1) * a.C;
    const float* bws = a.beta_ws + (size_t)item * (a.T + 1) * a.C;
    const double* offs = a.offs + (size_t)item * (a.T + 1);
    __syncthreads();
    FusedERows er;
    fused_load_e(a.e, V, b, R, H, er);
    for (int t = t0; t < t1; ++t) {
        if (tid < R) {
            const int q = fused_state(V, b, tid);
            aw_s[tid] = aws[(size_t)t * a.C + q];
            bl_s[tid] = bws[(size_t)(t + 1) * a.C + q];
        } else if (tid >= 128 && tid < 128 + V) {
            const int y = tid - 127;
            bn_s[y] = bws[(size_t)(t + 1) * a.C + 1 + V + (b - 1) * V + (y - 1)];
            if (b == 1) bs_s[y] = bws[(size_t)(t + 1) * a.C + y];
        }
        u64 unused_word = 0;
        fused_weights_full<MT>(a.f + ((size_t)item * a.T + t) * H, er, hid_s, w_s, a.Wf, R, H, (V + 15) / 16, nullptr,
                               unused_word);
        const float P = (float)(offs[t + 1] - offs[t]);
        fused_rows<true>(w_s, bl_s, bn_s, bs_s, aw_s, P, V, R, b == 1, nullptr, gh_s, gl_s);
        lds_barrier();
        fused_dw_accumulate<MT>(hid_s, gh_s, gl_s, acc, NT, H);
        lds_barrier();
    }
    fused_dw_flush(acc, a.dW, a.scale, NT, H, V1);
}

// The same sum from the marginals the backward kernel has kept (FusedBwdArgs::gamma_ws): per frame the
// hidden tile (tanh only, no contraction with W) and the frame's two bf16 planes, fetched with 16-byte
// loads that are requested before the tanh pass and transposed into LDS after it.
template <int MT>
__global__ __launch_bounds__(kFuThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_dw_kept_kernel(FusedBwdArgs a)
{
    extern __shared__ unsigned char smem_raw[];
    const int V = a.V, V1 = V + 1, H = a.H, R = V + 2;
    const int NT = (V1 + 15) / 16;
    constexpr int RS = (16 * MT + 31) / 32;
    constexpr int kRows = 32 * RS;
    constexpr int kGV = (2 * (64 + 2) * ((64 + 1 + 7) / 8) + kFuThreads - 1) / kFuThreads;   // 16-byte pieces per thread at most (V <= 64)
    __bf16* hid_s = (__bf16*)smem_raw;                                // [kRows][kFuHF]
    __bf16* gh_s = hid_s + (size_t)kRows * kFuHF;                     // [kFuMaxRows (y)][kFuGS (r)]
    __bf16* gl_s = gh_s + (size_t)kFuMaxRows * kFuGS;

    const int tid = threadIdx.x;
    const int ch = blockIdx.x % a.nch;
    const int b = (blockIdx.x / a.nch) % V + 1;
    const int item = blockIdx.x / (a.nch * V);
    int L = a.len[item];
    if (L < 0 || L > a.T) L = 0;
    const int t0 = ch * a.TC, t1 = min(L, t0 + a.TC);
    if (t0 >= t1) return;
    for (int i = tid; i < kRows * kFuHF; i += kFuThreads) hid_s[i] = (__bf16)0.f;
    for (int i = tid; i < 2 * kFuMaxRows * kFuGS; i += kFuThreads) gh_s[i] = (__bf16)0.f;
    floatx4 acc[kFuKT][kFuMaxNT];
#pragma unroll
    for (int kt = 0; kt < kFuKT; ++kt)
#pragma unroll
        for (int yt = 0; yt < kFuMaxNT; ++yt) acc[kt][yt] = floatx4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    FusedERows er;
    fused_load_e(a.e, V, b, R, H, er);
    const int P8 = (V1 + 7) / 8, per_plane = R * P8;
    for (int t = t0; t < t1; ++t) {
        const uintx4* gin = (const uintx4*)(a.gamma_ws + (((size_t)item * a.T + t) * V + (b - 1)) * 2 * R * 8 * P8);
        uintx4 gv[kGV];
#pragma unroll
        for (int j = 0; j < kGV; ++j) {
            const int i = tid + j * kFuThreads;
            gv[j] = i < 2 * per_plane ? gin[i] : uintx4{0u, 0u, 0u, 0u};
        }
        fused_hidden_full(a.f + ((size_t)item * a.T + t) * H, er, hid_s, R, H);
#pragma unroll
        for (int j = 0; j < kGV; ++j) {
            const int i = tid + j * kFuThreads;
            if (i < 2 * per_plane) {
                const int plane = i >= per_plane ? 1 : 0, k = i - plane * per_plane;
                const int r = k / P8, c8 = k - r * P8;
                unsigned short* dst = (unsigned short*)(plane ? gl_s : gh_s) + r;
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int y = 8 * c8 + 2 * e2;
                    if (y <= V) dst[(size_t)y * kFuGS] = (unsigned short)(gv[j][e2] & 0xffffu);
                    if (y + 1 <= V) dst[(size_t)(y + 1) * kFuGS] = (unsigned short)(gv[j][e2] >> 16);
                }
            }
        }
        lds_barrier();
        fused_dw_accumulate<MT>(hid_s, gh_s, gl_s, acc, NT, H);
        lds_barrier();
    }
    fused_dw_flush(acc, a.dW, a.scale, NT, H, V1);
}

}  // namespace last
