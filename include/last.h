/*
 * last.h -- C ABI of the MI355X (gfx950) lattice library.
 *
 * The library computes, on one GPU, the semiring shortest distance over the
 * complete recognition lattice of a globally normalised transducer
 * (arXiv 2304.13134, Sections 2.1 and 3), its gradient (the arc marginals of
 * Eq. 1, obtained by forward-backward as in Section 4.2.2), the shortest
 * distance on the lattice intersected with a reference label string
 * (Section 2.1, the numerator of the globally normalised loss), and the
 * tropical shortest path with integer backpointers (Sections 2.3, 4.2.3).
 *
 * Lattice (Section 3): context dependency = full n-gram of context size
 * `order` (1 or 2) over `vocab` labels, or any deterministic automaton that
 * accepts every label string, given as a next-state table (order = 0; this is
 * also how context sizes of 3 and more are expressed); alignment lattice = frame dependent (exactly
 * one arc, a label or the empty label, per frame; Figure 1b); weight function
 * = a dense tensor, or the shared-embedding function evaluated on the fly
 * (Section 4.1) as tanh(f[b][t] + e[q]) @ W.
 *
 * Index conventions (part of this ABI):
 *   labels y in 0..V, y = 0 is the empty label; it keeps the context state.
 *   context states q in 0..C-1; 0 = empty history;
 *     order 1: state a (1..V) = "last label a";               C = 1 + V
 *     order 2: (a) -> a, (a,b) -> 1 + V + (a-1)V + (b-1);     C = 1 + V + V^2
 *   next(q, y>0): order 1 -> y; order 2: () -> (y), (a) -> (a,y), (a,b) -> (b,y);
 *     order 0: next_table[q*V + (y-1)], the start state is 0.
 *   every state (len[b], q) is final with weight 0.
 *   dense weights: w[b][t][q][y], float32, C-contiguous [B][T][C][V+1].
 *   semirings: higher is better; (+) = log-add-exp (LAST_LOG) or max
 *   (LAST_TROPICAL), (x) = +, zero = -inf, one = 0.
 *
 * Memory and execution:
 *   Pointers marked "dev" are device (HBM) pointers owned by the caller; the
 *   library never allocates, frees or keeps them.  Structs are host memory.
 *   All work is enqueued on `hip_stream` (a hipStream_t passed as void*;
 *   NULL = the default stream) and the calls return without synchronising.
 *   `ws` is a dev scratch buffer of at least last_workspace_bytes() bytes,
 *   256-byte aligned, contents undefined before and after a call.  Outputs
 *   must not alias inputs.
 *
 * Errors: the return value reports what the host can check (null pointers,
 * bad shapes, num_states inconsistent with (vocab, order), workspace too
 * small, unsupported combination, HIP launch failure); on error nothing is
 * enqueued.  Data-dependent conditions are reported per item in the optional
 * dev array item_status[B]:
 *   0 ok; 1 length outside [0,T]; 2 reference label outside [1,V];
 *   3 reference length outside [0,Umax]; 4 infeasible (reference longer than
 *   the number of frames: numerator = -inf, its marginals are 0);
 *   5 the cooperating workgroups of an item timed out waiting for each other
 *   (results of that item are undefined; never expected in normal operation);
 *   6 the weights of the item span more dynamic range than the bandwidth path
 *   for dense bigram lattices guarantees for marginals (it keeps state vectors
 *   in scaled float32: entries more than 2^126 below the largest of a frame
 *   are zero there).  dist is still exact; marginals of arcs that leave such
 *   states may be lost.  Not raised for weights within about +-50; setting the
 *   environment variable LAST_FORCE_SOLO=1 selects the log-domain kernels,
 *   which have no such limit.
 * Items with status 1..3 get dist = NaN and zero gradients.
 * Frames t >= len[b] do not exist for item b: their weights are never read
 * into a result, their marginals are 0 and their path entries are -1.
 */
#ifndef LAST_H_
#define LAST_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LAST_OK = 0,
    LAST_ERR_NULL = 1,        /* a required pointer is NULL                    */
    LAST_ERR_SHAPE = 2,       /* a size is non-positive or too large           */
    LAST_ERR_CONTEXT = 3,     /* order not in {0,1,2} or num_states inconsistent */
    LAST_ERR_SEMIRING = 4,    /* unknown semiring                              */
    LAST_ERR_WORKSPACE = 5,   /* ws NULL, misaligned or too small              */
    LAST_ERR_UNSUPPORTED = 6, /* combination not implemented                   */
    LAST_ERR_HIP = 7          /* a HIP call failed                             */
} last_status_t;

typedef enum { LAST_LOG = 0, LAST_TROPICAL = 1 } last_semiring_t;

typedef enum {
    LAST_OP_SHORTEST_DISTANCE = 0,
    LAST_OP_ARC_POSTERIORS = 1,
    LAST_OP_INTERSECT_REFERENCE = 2,
    LAST_OP_SHORTEST_PATH = 3,
    LAST_OP_LOCAL_LOG_LIKELIHOOD = 4,
    LAST_OP_LOSS = 5
} last_op_t;

/* Context dependency (Section 3): the full n-gram one in closed form (Figure 1a
 * is order 1), or a next-state table.  next_table: dev int32 [C][V], read by
 * every call that uses the struct, never written; it must stay valid until the
 * work enqueued by the call has finished.  With a table, the weights must be
 * dense, every call runs one workgroup per item, C is limited by the 160 KiB of
 * LDS of a compute unit (about 10000 states for the log semiring, 13000 for the
 * tropical one) and C*V by 2^24 (LAST_ERR_UNSUPPORTED beyond), and each call validates the table
 * on the device (item_status 7). */
typedef struct {
    int32_t vocab;             /* V >= 1                                              */
    int32_t order;             /* context size n: 1 or 2; 0 = next_table              */
    int32_t num_states;        /* C; order 1, 2: must equal sum_{k<=n} V^k            */
    const int32_t* next_table; /* order 0 only (NULL otherwise)                       */
} last_context_t;

enum { LAST_WEIGHTS_DENSE = 0, LAST_WEIGHTS_SHARED_EMB = 1 };

/* Weight function (Section 3).  kind = dense: `w` dev float32 [B][T][C][V+1].
 * kind = shared_emb: f dev bf16 [B][T][hidden], e dev bf16 [C][hidden],
 * W dev bf16 [hidden][V+1] (bf16 = upper 16 bits of a float32); the hidden
 * vector tanh(f + e) is rounded to bf16 before the float32-accumulated
 * contraction with W; the weights are never stored (Section 4.1).  Supported
 * for context size 2, V <= 64, hidden a multiple of 128 up to 512, in
 * last_shortest_distance (LAST_LOG) and last_arc_posteriors; f, e, W must be
 * 16-byte aligned.  Other combinations return LAST_ERR_UNSUPPORTED. */
typedef struct {
    int32_t kind;
    int32_t B, T;
    const float* w;
    const uint16_t* f;
    const uint16_t* e;
    const uint16_t* W;
    int32_t hidden;
} last_weights_t;

/* Where gradients go.  dense: dw dev float32 [B][T][C][V+1].  shared_emb:
 * df dev float32 [B][T][hidden], de dev float32 [C][hidden], dW dev float32
 * [hidden][V+1].  accumulate = 0: out = scale * marginal (every element of the
 * tensor is written); accumulate = 1: out += scale * marginal. */
typedef struct {
    float* dw;
    float* df;
    float* de;
    float* dW;
    int32_t accumulate;
    float scale;
} last_grads_t;

/* Scratch bytes `op` needs for these shapes (Umax only matters for
 * LAST_OP_INTERSECT_REFERENCE and LAST_OP_LOCAL_LOG_LIKELIHOOD).  Returns 0 on
 * invalid arguments. */
size_t last_workspace_bytes(const last_weights_t* weights, const last_context_t* context,
                            int32_t op, int32_t Umax);

/* Shortest distance over the complete lattice (Section 2.1; Eq. 2 visited in
 * increasing t as in Section 4.1).  lengths: dev int32 [B].  dist: dev
 * float32 [B] = (+)-sum over all accepting paths (LAST_LOG) or the best path
 * score (LAST_TROPICAL). */
last_status_t last_shortest_distance(const last_weights_t* weights, const int32_t* lengths,
                                     const last_context_t* context, last_semiring_t semiring,
                                     float* dist, int32_t* item_status,
                                     void* ws, size_t ws_bytes, void* hip_stream);

/* Log-semiring shortest distance and its gradient, the arc marginals of
 * Eq. 1, by forward-backward (Section 4.2.2: only alpha and beta are kept,
 * O(|Q|) extra space).  dist: dev float32 [B].  out: see last_grads_t. */
last_status_t last_arc_posteriors(const last_weights_t* weights, const int32_t* lengths,
                                  const last_context_t* context, float* dist,
                                  const last_grads_t* out, int32_t* item_status,
                                  void* ws, size_t ws_bytes, void* hip_stream);

/* Intersection with the reference string and log-semiring shortest distance
 * on it (Section 2.1; Table 1 "GNAT, intersected": O(TU) states and arcs).
 * State (t,u): u reference labels read, context ctx(u) = next(ctx(u-1), ref[u]);
 * arcs: empty label to (t+1,u) with weight w[t][ctx(u)][0], label ref[u+1] to
 * (t+1,u+1) with weight w[t][ctx(u)][ref[u+1]]; only (len, U) is final.
 * refs: dev int32 [B][Umax] labels in 1..V; ref_lengths: dev int32 [B].
 * numerator: dev float32 [B].  out (or NULL): marginals of the intersected
 * lattice scattered onto the arcs of the complete lattice they ride on
 * (dense weights only), normally with accumulate = 1, scale = -1 after
 * last_arc_posteriors so that dw = d(dist - numerator)/dw. */
last_status_t last_intersect_reference(const last_weights_t* weights, const int32_t* lengths,
                                       const last_context_t* context,
                                       const int32_t* refs, const int32_t* ref_lengths,
                                       int32_t Umax, float* numerator,
                                       const last_grads_t* out, int32_t* item_status,
                                       void* ws, size_t ws_bytes, void* hip_stream);

/* The globally normalised loss in one call (Section 2.1): dist = denominator
 * (last_arc_posteriors), numerator (last_intersect_reference), and
 * out (+)= scale * d(dist - numerator)/d(weights), i.e. the arc marginals of the
 * complete lattice minus those of the intersected lattice (dense: dw; shared_emb:
 * df, de, dW).  Results as from the two calls in sequence, but the numerator's
 * recursion runs beside the denominator on a stream of the library's own (one
 * per device, default priority, created at the first call and kept until the
 * process ends; forked from and joined to hip_stream with events, so the call
 * is still asynchronous and ordered like any other work on hip_stream).
 * Workspace: last_workspace_bytes(..., LAST_OP_LOSS, Umax).  item_status reports
 * the first problem of either part. */
last_status_t last_globally_normalized_loss(const last_weights_t* weights, const int32_t* lengths,
                                           const last_context_t* context,
                                           const int32_t* refs, const int32_t* ref_lengths, int32_t Umax,
                                           float* dist, float* numerator, const last_grads_t* out,
                                           int32_t* item_status, void* ws, size_t ws_bytes, void* hip_stream);

/* Log-likelihood of the reference string under the locally normalised model on
 * the same lattice (Section 2.1: intersection and shortest distance, with the
 * weights of the V+1 arcs leaving each state (t,q) normalised,
 * w'[t][q][y] = w[t][q][y] - log sum_y' exp w[t][q][y']; Table 1, first row).
 * No denominator lattice is needed.  Arguments as last_intersect_reference;
 * loglik: dev float32 [B].  out (or NULL): d loglik / d w on the dense tensor,
 * i.e. the marginals of the intersected lattice on the arcs they ride on minus
 * (their sum over the arcs leaving the state) * softmax(w[t][q])[y]; rows of
 * states the reference never visits are 0.  Unlike last_intersect_reference
 * the result is independent of timing (no floating-point atomics).
 * Requires 4*(V+1)*4 bytes <= 64 KiB of LDS (V < 4096). */
last_status_t last_local_log_likelihood(const last_weights_t* weights, const int32_t* lengths,
                                        const last_context_t* context,
                                        const int32_t* refs, const int32_t* ref_lengths,
                                        int32_t Umax, float* loglik,
                                        const last_grads_t* out, int32_t* item_status,
                                        void* ws, size_t ws_bytes, void* hip_stream);

/* Tropical shortest path (Sections 2.1, 2.3, 4.2.3): one float32 add per arc,
 * arg max kept per state as the flat arc index q*(V+1)+y, ties to the lowest
 * flat index, final ties to the lowest state; then a backtrace.
 * labels: dev int32 [B][T]; states: dev int32 [B][T+1]; entries past len are
 * -1.  score: dev float32 [B]. */
last_status_t last_shortest_path(const last_weights_t* weights, const int32_t* lengths,
                                 const last_context_t* context,
                                 int32_t* labels, int32_t* states, float* score,
                                 int32_t* item_status,
                                 void* ws, size_t ws_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): last_shortest_distance
 * without the workspace arguments.  The scratch memory is a static device array
 * of LAST_STATIC_SCRATCH_BYTES inside the library; each GPU the library runs on
 * holds its own copy until the process ends.  The call allocates and frees
 * nothing.  Shapes whose last_workspace_bytes(..., LAST_OP_SHORTEST_DISTANCE, 0)
 * exceeds LAST_STATIC_SCRATCH_BYTES are rejected with LAST_ERR_WORKSPACE (nothing
 * is enqueued).  All calls on one GPU share that GPU's array: calls that overlap
 * in time on one GPU (two streams, two threads) race on it and must be serialised
 * by the caller; calls in sequence on one stream are fine (whatever must start
 * from zero is cleared by the call itself).  Everything else as
 * last_shortest_distance. */
#define LAST_STATIC_SCRATCH_BYTES (32u << 20)
last_status_t last_shortest_distance_static(const last_weights_t* weights, const int32_t* lengths,
                                            const last_context_t* context, last_semiring_t semiring,
                                            float* dist, int32_t* item_status, void* hip_stream);

/* Process-wide settings, for cross-checks and tests; they take effect on the next call.
 *   LAST_OPT_FORCE_SOLO (0/1, default 0): 1 = always the one-workgroup-per-item kernels (log domain,
 *     no limit on the dynamic range of the weights).
 *   LAST_OPT_CLUSTER_GENERATION (0..3, default 0): which cooperating-workgroup forward-backward kernel
 *     dense bigram lattices take; 0 = the newest that supports the shape, 3 = sixteen workgroups per
 *     direction and item (256 labels only), 2 = eight (5..264 states), 1 = the oldest (one exchange per
 *     frame).  A generation that does not support the shape falls back to the next older one.
 *   LAST_OPT_CLUSTER_VITERBI (0..2, default 1): shortest path of dense bigram lattices: 0 = one workgroup
 *     per item; 1 = cooperating workgroups, the newest kernel that takes the shape; 2 = cooperating
 *     workgroups, the older kernel also where the newer one (256 labels only) would run.
 *   LAST_OPT_SPIN_LIMIT (>= 1, default 2^20): polls a cooperating workgroup makes before it gives up
 *     waiting for the others (the item then gets status 5 and dist = NaN; every kernel still ends).
 *   LAST_OPT_FUSED_FRAMES_PER_TILE (1 or 2, default 2): frames whose on-the-fly weights the forward
 *     kernel of the shared_emb path computes at a time (Section 5 discusses evaluating the weight
 *     function for several frames at once).  2 shares the rows of e and the phase barriers between
 *     two frames and doubles the hidden tile in LDS; a shape whose tiles then no longer fit uses 1.
 *     The shortest distance does not depend on it bit for bit.
 *   LAST_OPT_FUSED_KEEP_MARGINALS (0/1, default 1): 1 = the backward pass of the shared_emb path keeps
 *     the arc marginals of every frame (two bfloat16 halves each) in the workspace for the kernel that
 *     forms dW, which then does not evaluate the weight function a third time; as long as they take
 *     at most 8 GiB (B T V (V+2) (V+1 rounded up to 8) 4 bytes), else and with 0 they are recomputed.
 *     last_workspace_bytes follows the setting: ask again after changing it.
 * last_set_option returns LAST_ERR_UNSUPPORTED for an unknown option or value; last_get_option
 * returns -1 for an unknown option. */
typedef enum {
    LAST_OPT_FORCE_SOLO = 0,
    LAST_OPT_CLUSTER_GENERATION = 1,
    LAST_OPT_CLUSTER_VITERBI = 2,
    LAST_OPT_SPIN_LIMIT = 3,
    LAST_OPT_FUSED_FRAMES_PER_TILE = 4,
    LAST_OPT_FUSED_KEEP_MARGINALS = 5,
    LAST_OPT_COUNT_ = 6
} last_option_t;
last_status_t last_set_option(int32_t option, int32_t value);
int32_t last_get_option(int32_t option);

/* Measurement aid, not part of the method: plain streaming kernels of known
 * traffic, the yardstick the lattice kernels are held against and the
 * calibration of HBM byte counters.  LAST_PROBE_READ reads `bytes` bytes at
 * src (dev) once and writes nothing (dst: dev, at least 16 bytes, left
 * untouched); LAST_PROBE_COPY copies them to dst (dev, `bytes` bytes, must not
 * overlap src).  bytes a positive multiple of 16, both pointers 16-byte
 * aligned (LAST_ERR_SHAPE otherwise).  LAST_PROBE_READ_ROWS and
 * LAST_PROBE_READ_COLUMNS read src, taken as frames of [257][257] float32
 * (bytes a multiple of 257*257*4), once in the two access patterns of the
 * bigram forward-backward kernel at 256 labels, with its launch shape and none
 * of its arithmetic: whole rows per wavefront, or blocks of 32 columns per
 * workgroup (128-byte pieces at a stride of 1028 bytes); dst as for
 * LAST_PROBE_READ. */
enum { LAST_PROBE_READ = 0, LAST_PROBE_COPY = 1, LAST_PROBE_READ_ROWS = 2, LAST_PROBE_READ_COLUMNS = 3 };
last_status_t last_probe_bandwidth(int32_t kind, const void* src, void* dst, size_t bytes, void* hip_stream);

/* Check, on the current device, what the cooperating-workgroup kernels rely on (Section 4 of the
 * paper leaves the mapping to hardware open; this is this library's): a launch of 256 workgroups is
 * resident all at once, and workgroups i and j run on the same XCD exactly when i = j (mod 8), so
 * that the workgroups of an item exchange their partial results through one XCD's L2.  Runs a small
 * probe on `hip_stream` and WAITS for it (the one call here besides last_globally_normalized_loss'
 * set-up that synchronises; not for use under stream capture).  workspace: device memory, at least
 * 2048 bytes, 4-byte aligned, contents overwritten.  LAST_OK: the layout holds.
 * LAST_ERR_UNSUPPORTED: it does not (or the chip has fewer than 256 compute units); from then on
 * every call on this device takes the one-workgroup-per-item kernels.  Without this call the layout
 * is assumed on chips of 256 compute units; if it did not hold there, the bounded waits would end
 * the kernels and the items would carry status 5.  The binding calls it once per device. */
last_status_t last_verify_placement(void* workspace, size_t workspace_bytes, void* hip_stream);

const char* last_status_string(last_status_t status);

/* Text of the HIP error behind the most recent LAST_ERR_HIP (diagnostics). */
const char* last_hip_error_string(void);

/* Library version and the kernel variant a call would use, for diagnostics:
 * 0 = one workgroup per item, 1 = cooperating workgroups per item (dense
 * weights, context size 1), 2 = on-the-fly weights (shared_emb), -1 = the
 * combination is not supported (the call would return LAST_ERR_UNSUPPORTED or
 * an argument error). */
int32_t last_version(void);
int32_t last_kernel_variant(const last_weights_t* weights, const last_context_t* context,
                            int32_t op);

#ifdef __cplusplus
}
#endif
#endif /* LAST_H_ */
