/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Plain, slow, float64 CPU implementation of the lattice computations of
 * "LAST: Scalable Lattice-Based Speech Modelling in JAX" (arXiv 2304.13134).
 * It exists only so that tests, the smoke check and the benchmark's CPU
 * baseline leg have something independent to compare the GPU library with.
 * It shares no code, header, table or helper with the HIP library and is
 * never loaded by it.
 *
 * Conventions (the paper fixes none of these; they are this build's readings):
 *   labels y in {0..V}; y = 0 is the empty label (epsilon, "blank");
 *   context states q in {0..C-1}; q = 0 is the empty history (start state);
 *   dense arc weights w[b][t][q][y], fp32, C-contiguous [B][T][C][V+1];
 *   semiring convention: higher is better, (+) = log-add-exp or max,
 *   (x) = +, zero = -inf, one = 0 (Section 2.1 with the log-semiring formula
 *   of Section 4.2.2 and the max of Section 4.2.3);
 *   every state (len, q) is final with weight 0 (Figure 1c: all last-frame
 *   states are accepting);
 *   the empty label keeps the context state (the context dependency of
 *   Figure 1a has no epsilon arcs, so intersection leaves its state alone).
 *
 * Every routine follows the passage it cites in the paper's own order:
 * no blocking, no fusion, no rescaling tricks; log-sum-exp is always the
 * two-pass form max, then log(sum(exp(x - max))).
 *
 * Pins (tests/test_oracle_*.py, all run without a GPU): brute-force
 * enumeration of every accepting path (the definitions in Section 2.3),
 * closed forms, finite differences, the Figure 1 topology counts, and
 * special cases that reduce to a library log-sum-exp.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define NEG_INF (-INFINITY)

/* ---------------------------------------------------------------------- */
/* Context dependency: full n-gram, context size n = order (Section 3,      */
/* Figure 1a shows order 1).  Deterministic, accepts Sigma^*.               */
/* order 1: state 0 = empty history, state a = "last label a".             */
/* order 2: state 0, states (a) -> a, states (a,b) -> 1+V+(a-1)V+(b-1).    */
/* ---------------------------------------------------------------------- */

/* A context dependency may also be any deterministic automaton that accepts  */
/* Sigma^*, given by a look-up table ("NextStateTable", Section 3):          */
/* table[q][y-1] = destination of label y out of state q.  It is registered  */
/* with lo_set_next_table and selected with order == 0.                      */
static const int32_t* g_table = NULL;
static int g_table_C = 0, g_table_V = 0;

void lo_set_next_table(const int32_t* table, int C, int V)
{
    g_table = table;
    g_table_C = C;
    g_table_V = V;
}

int lo_num_states(int V, int order)
{
    if (V < 1) return -1;
    if (order == 0) return (g_table != NULL && V == g_table_V) ? g_table_C : -1;
    if (order == 1) return 1 + V;
    if (order == 2) return 1 + V + V * V;
    return -1;
}

/* destination context state of the arc (q, y); the empty label stays. */
int lo_next_state(int V, int order, int q, int y)
{
    if (y == 0) return q;
    if (order == 0) return g_table[q * V + (y - 1)];
    if (order == 1) return y;
    /* order 2 */
    if (q == 0) return y;                       /* ()    --y--> (y)    */
    if (q <= V) return 1 + V + (q - 1) * V + (y - 1); /* (a) --y--> (a,y) */
    {
        int b = (q - 1 - V) % V + 1;            /* (a,b) --y--> (b,y)  */
        return 1 + V + (b - 1) * V + (y - 1);
    }
}

int lo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void lo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static int clamp_len(int len, int T)
{
    if (len < 0) return 0;
    if (len > T) return T;
    return len;
}

/* two-pass log-sum-exp of n values */
static double lse(const double* x, int n)
{
    double m = NEG_INF;
    for (int i = 0; i < n; ++i)
        if (x[i] > m) m = x[i];
    if (m == NEG_INF) return NEG_INF;
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += exp(x[i] - m);
    return m + log(s);
}

/* ---------------------------------------------------------------------- */
/* One step of the forward recurrence, Eq. 2, for all states of frame t+1: */
/* alpha'[q'] = (+)_{arcs e into q'} alpha[prev e] (x) w[e].               */
/* Written as two sweeps over the arcs (max, then sum of exp).             */
/* ---------------------------------------------------------------------- */
static void forward_step(const double* alpha, const double* wt /*[C][V1]*/,
                         int C, int V, int order, double* out, double* mx)
{
    const int V1 = V + 1;
    for (int d = 0; d < C; ++d) { mx[d] = NEG_INF; out[d] = 0.0; }
    for (int q = 0; q < C; ++q)
        for (int y = 0; y < V1; ++y) {
            double v = alpha[q] + wt[q * V1 + y];
            int d = lo_next_state(V, order, q, y);
            if (v > mx[d]) mx[d] = v;
        }
    for (int q = 0; q < C; ++q)
        for (int y = 0; y < V1; ++y) {
            int d = lo_next_state(V, order, q, y);
            if (mx[d] == NEG_INF) continue;
            double v = alpha[q] + wt[q * V1 + y];
            out[d] += exp(v - mx[d]);
        }
    for (int d = 0; d < C; ++d)
        out[d] = (mx[d] == NEG_INF) ? NEG_INF : mx[d] + log(out[d]);
}

/* reverse step: beta[q] = (+)_y w[q][y] (x) beta'[next(q,y)] */
static void backward_step(const double* beta_next, const double* wt, int C, int V,
                          int order, double* out, double* tmp /*[V1]*/)
{
    const int V1 = V + 1;
    for (int q = 0; q < C; ++q) {
        for (int y = 0; y < V1; ++y)
            tmp[y] = wt[q * V1 + y] + beta_next[lo_next_state(V, order, q, y)];
        out[q] = lse(tmp, V1);
    }
}

static void load_frame(const float* w, double* wt, size_t n)
{
    for (size_t i = 0; i < n; ++i) wt[i] = (double)w[i];
}

/*
 * Shortest distance in the log semiring over the complete recognition
 * lattice (Section 2.1 "Shortest distance", Eq. 2; Section 4.1: states are
 * (t, q) visited in increasing t).
 *   alpha : out [B][T+1][C] float64, alpha[b][0] = (0, -inf, ...);
 *           rows t > len[b] repeat row len[b].
 *   D     : out [B]  = log-sum-exp over q of alpha[b][len[b]][q].
 */
int lo_forward(const float* w, const int32_t* len, int B, int T, int V, int order,
               double* alpha, double* D)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const size_t fr = (size_t)C * V1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double* wt = (double*)malloc(fr * sizeof(double));
        double* mx = (double*)malloc((size_t)C * sizeof(double));
        double* al = alpha + (size_t)b * (T + 1) * C;
        const int L = clamp_len(len[b], T);
        al[0] = 0.0;
        for (int q = 1; q < C; ++q) al[q] = NEG_INF;
        for (int t = 0; t < T; ++t) {
            if (t < L) {
                load_frame(w + ((size_t)b * T + t) * fr, wt, fr);
                forward_step(al + (size_t)t * C, wt, C, V, order, al + (size_t)(t + 1) * C, mx);
            } else {
                memcpy(al + (size_t)(t + 1) * C, al + (size_t)t * C, (size_t)C * sizeof(double));
            }
        }
        D[b] = lse(al + (size_t)L * C, C);
        free(wt);
        free(mx);
    }
    return 0;
}

/*
 * Backward weights (Section 4.2.2: beta[q] = sum of path weights from q to
 * the final states).  beta : out [B][T+1][C]; rows t >= len[b] are 0.
 */
int lo_backward(const float* w, const int32_t* len, int B, int T, int V, int order,
                double* beta)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const size_t fr = (size_t)C * V1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double* wt = (double*)malloc(fr * sizeof(double));
        double* tmp = (double*)malloc((size_t)V1 * sizeof(double));
        double* be = beta + (size_t)b * (T + 1) * C;
        const int L = clamp_len(len[b], T);
        for (int t = T; t >= L; --t)
            for (int q = 0; q < C; ++q) be[(size_t)t * C + q] = 0.0;
        for (int t = L - 1; t >= 0; --t) {
            load_frame(w + ((size_t)b * T + t) * fr, wt, fr);
            backward_step(be + (size_t)(t + 1) * C, wt, C, V, order, be + (size_t)t * C, tmp);
        }
        free(wt);
        free(tmp);
    }
    return 0;
}

/*
 * Arc marginals, Eq. 1, from the forward and backward weights:
 * gamma[b][t][q][y] = exp(alpha_t[q] + w + beta_{t+1}[next(q,y)] - D);
 * exactly 0 where alpha_t[q] = -inf and for frames t >= len[b].
 * gamma : out [B][T][C][V+1] float64.
 */
int lo_posteriors(const float* w, const int32_t* len, int B, int T, int V, int order,
                  const double* alpha, const double* beta, const double* D, double* gamma)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const size_t fr = (size_t)C * V1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int L = clamp_len(len[b], T);
        const double* al = alpha + (size_t)b * (T + 1) * C;
        const double* be = beta + (size_t)b * (T + 1) * C;
        for (int t = 0; t < T; ++t) {
            const float* wt = w + ((size_t)b * T + t) * fr;
            double* g = gamma + ((size_t)b * T + t) * fr;
            for (int q = 0; q < C; ++q)
                for (int y = 0; y < V1; ++y) {
                    double a = al[(size_t)t * C + q];
                    if (t >= L || a == NEG_INF) { g[q * V1 + y] = 0.0; continue; }
                    int d = lo_next_state(V, order, q, y);
                    g[q * V1 + y] = exp(a + (double)wt[q * V1 + y] + be[(size_t)(t + 1) * C + d] - D[b]);
                }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Numerator: intersection of the complete lattice with a reference label  */
/* string, then shortest distance on it (Section 2.1, the two-step recipe   */
/* for the globally normalised loss; Table 1 "GNAT, intersected").          */
/* States of the intersection are (t, u): u labels of the reference read.   */
/* From (t,u): the empty label goes to (t+1,u) with weight                  */
/* w[t][ctx(u)][0]; label ref[u] (0-based storage) goes to (t+1,u+1) with   */
/* weight w[t][ctx(u)][ref[u]].  Only (len, U) is final.                    */
/*   refs  [B][Umax] int32 labels in 1..V;  ulen [B]                        */
/*   ctx   out [B][Umax+1] context state after u labels                     */
/*   a, bb out [B][T+1][Umax+1] forward / backward weights (-inf outside)   */
/*   N     out [B] numerator (-inf when U > len)                            */
/*   pb    out [B][T][Umax+1] marginal of the empty-label arc out of (t,u)  */
/*   pl    out [B][T][Umax+1] marginal of the label arc out of (t,u), u<U   */
/* ---------------------------------------------------------------------- */
int lo_numerator(const float* w, const int32_t* len, const int32_t* refs, const int32_t* ulen,
                 int B, int T, int V, int order, int Umax,
                 int32_t* ctx, double* a, double* bb, double* N, double* pb, double* pl)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const int U1 = Umax + 1;
    const size_t fr = (size_t)C * V1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int L = clamp_len(len[b], T);
        const int U = ulen[b];
        const int32_t* r = refs + (size_t)b * Umax;
        int32_t* cx = ctx + (size_t)b * U1;
        double* A = a + (size_t)b * (T + 1) * U1;
        double* Bk = bb + (size_t)b * (T + 1) * U1;
        double* PB = pb + (size_t)b * T * U1;
        double* PL = pl + (size_t)b * T * U1;
        for (size_t i = 0; i < (size_t)(T + 1) * U1; ++i) { A[i] = NEG_INF; Bk[i] = NEG_INF; }
        for (size_t i = 0; i < (size_t)T * U1; ++i) { PB[i] = 0.0; PL[i] = 0.0; }
        cx[0] = 0;
        for (int u = 1; u <= Umax; ++u)
            cx[u] = (u <= U) ? lo_next_state(V, order, cx[u - 1], r[u - 1]) : -1;
        /* forward */
        A[0] = 0.0;
        for (int t = 0; t < L; ++t) {
            const float* wt = w + ((size_t)b * T + t) * fr;
            for (int u = 0; u <= U; ++u) {
                double c[2];
                c[0] = A[(size_t)t * U1 + u] + (double)wt[cx[u] * V1 + 0];
                c[1] = NEG_INF;
                if (u >= 1)
                    c[1] = A[(size_t)t * U1 + u - 1] + (double)wt[cx[u - 1] * V1 + r[u - 1]];
                A[(size_t)(t + 1) * U1 + u] = lse(c, 2);
            }
        }
        N[b] = A[(size_t)L * U1 + U];
        /* backward */
        Bk[(size_t)L * U1 + U] = 0.0;
        for (int t = L - 1; t >= 0; --t) {
            const float* wt = w + ((size_t)b * T + t) * fr;
            for (int u = 0; u <= U; ++u) {
                double c[2];
                c[0] = (double)wt[cx[u] * V1 + 0] + Bk[(size_t)(t + 1) * U1 + u];
                c[1] = NEG_INF;
                if (u < U)
                    c[1] = (double)wt[cx[u] * V1 + r[u]] + Bk[(size_t)(t + 1) * U1 + u + 1];
                Bk[(size_t)t * U1 + u] = lse(c, 2);
            }
        }
        /* arc marginals (Eq. 1 on the intersected lattice) */
        if (N[b] != NEG_INF) {
            for (int t = 0; t < L; ++t) {
                const float* wt = w + ((size_t)b * T + t) * fr;
                for (int u = 0; u <= U; ++u) {
                    double av = A[(size_t)t * U1 + u];
                    if (av == NEG_INF) continue;
                    double nb = Bk[(size_t)(t + 1) * U1 + u];
                    if (nb != NEG_INF)
                        PB[(size_t)t * U1 + u] = exp(av + (double)wt[cx[u] * V1 + 0] + nb - N[b]);
                    if (u < U) {
                        double nl = Bk[(size_t)(t + 1) * U1 + u + 1];
                        if (nl != NEG_INF)
                            PL[(size_t)t * U1 + u] = exp(av + (double)wt[cx[u] * V1 + r[u]] + nl - N[b]);
                    }
                }
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Locally normalised model on the intersected lattice (Section 2.1: a     */
/* model like RNN-T is the intersection followed by a shortest distance;    */
/* Table 1, first row).  The weights of the V+1 arcs leaving a state (t,q)  */
/* are normalised, w'[t][q][y] = w[t][q][y] - log sum_y' exp w[t][q][y'],   */
/* and the shortest distance of the intersected lattice under w' is the     */
/* log-likelihood of the reference string; there is no denominator.         */
/* Same outputs as lo_numerator, plus                                       */
/*   grad out [B][T][C][V+1] (or NULL): d N / d w, i.e. for every state     */
/*        (t,u) with context q: its arc marginals on (q,0) and (q,ref[u])   */
/*        minus (their sum) * softmax(w[t][q])[y] on every y.               */
/* ---------------------------------------------------------------------- */
static double row_lse(const float* wt, int V1, int q)
{
    double tmp[V1];
    for (int k = 0; k < V1; ++k) tmp[k] = (double)wt[q * V1 + k];
    return lse(tmp, V1);
}

/* normalised weight of arc (q, y) of the frame whose weights start at wt */
static double local_logw(const float* wt, int V1, int q, int y)
{
    return (double)wt[q * V1 + y] - row_lse(wt, V1, q);
}

int lo_numerator_local(const float* w, const int32_t* len, const int32_t* refs, const int32_t* ulen,
                       int B, int T, int V, int order, int Umax,
                       int32_t* ctx, double* a, double* bb, double* N, double* pb, double* pl,
                       double* grad)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const int U1 = Umax + 1;
    const size_t fr = (size_t)C * V1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int L = clamp_len(len[b], T);
        const int U = ulen[b];
        const int32_t* r = refs + (size_t)b * Umax;
        int32_t* cx = ctx + (size_t)b * U1;
        double* A = a + (size_t)b * (T + 1) * U1;
        double* Bk = bb + (size_t)b * (T + 1) * U1;
        double* PB = pb + (size_t)b * T * U1;
        double* PL = pl + (size_t)b * T * U1;
        for (size_t i = 0; i < (size_t)(T + 1) * U1; ++i) { A[i] = NEG_INF; Bk[i] = NEG_INF; }
        for (size_t i = 0; i < (size_t)T * U1; ++i) { PB[i] = 0.0; PL[i] = 0.0; }
        if (grad) for (size_t i = 0; i < (size_t)T * fr; ++i) grad[(size_t)b * T * fr + i] = 0.0;
        cx[0] = 0;
        for (int u = 1; u <= Umax; ++u)
            cx[u] = (u <= U) ? lo_next_state(V, order, cx[u - 1], r[u - 1]) : -1;
        A[0] = 0.0;
        for (int t = 0; t < L; ++t) {
            const float* wt = w + ((size_t)b * T + t) * fr;
            for (int u = 0; u <= U; ++u) {
                double c[2];
                c[0] = A[(size_t)t * U1 + u] + local_logw(wt, V1, cx[u], 0);
                c[1] = NEG_INF;
                if (u >= 1)
                    c[1] = A[(size_t)t * U1 + u - 1] + local_logw(wt, V1, cx[u - 1], r[u - 1]);
                A[(size_t)(t + 1) * U1 + u] = lse(c, 2);
            }
        }
        N[b] = A[(size_t)L * U1 + U];
        Bk[(size_t)L * U1 + U] = 0.0;
        for (int t = L - 1; t >= 0; --t) {
            const float* wt = w + ((size_t)b * T + t) * fr;
            for (int u = 0; u <= U; ++u) {
                double c[2];
                c[0] = local_logw(wt, V1, cx[u], 0) + Bk[(size_t)(t + 1) * U1 + u];
                c[1] = NEG_INF;
                if (u < U)
                    c[1] = local_logw(wt, V1, cx[u], r[u]) + Bk[(size_t)(t + 1) * U1 + u + 1];
                Bk[(size_t)t * U1 + u] = lse(c, 2);
            }
        }
        if (N[b] != NEG_INF) {
            for (int t = 0; t < L; ++t) {
                const float* wt = w + ((size_t)b * T + t) * fr;
                for (int u = 0; u <= U; ++u) {
                    double av = A[(size_t)t * U1 + u];
                    if (av == NEG_INF) continue;
                    double nb = Bk[(size_t)(t + 1) * U1 + u];
                    if (nb != NEG_INF)
                        PB[(size_t)t * U1 + u] = exp(av + local_logw(wt, V1, cx[u], 0) + nb - N[b]);
                    if (u < U) {
                        double nl = Bk[(size_t)(t + 1) * U1 + u + 1];
                        if (nl != NEG_INF)
                            PL[(size_t)t * U1 + u] = exp(av + local_logw(wt, V1, cx[u], r[u]) + nl - N[b]);
                    }
                    if (grad) {
                        double* g = grad + ((size_t)b * T + t) * fr + (size_t)cx[u] * V1;
                        const double occ = PB[(size_t)t * U1 + u] + PL[(size_t)t * U1 + u];
                        g[0] += PB[(size_t)t * U1 + u];
                        if (u < U) g[r[u]] += PL[(size_t)t * U1 + u];
                        const double z = row_lse(wt, V1, cx[u]);
                        for (int y = 0; y < V1; ++y) g[y] -= occ * exp((double)wt[cx[u] * V1 + y] - z);
                    }
                }
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Shortest path = tropical shortest distance with the arg max kept per    */
/* state (Sections 2.1 "Shortest path", 2.3 and 4.2.3).                    */
/* Tie rule: among equal maxima into a state the arc with the lowest flat  */
/* index q*(V+1)+y wins; among equal final scores the lowest state wins.   */
/* Two arithmetic variants: float32 adds (one rounding per arc, which is   */
/* the precision the indices are defined in) and float64.                   */
/*   labels out [B][T]   (-1 for t >= len)                                  */
/*   states out [B][T+1] (-1 for t >  len)                                  */
/* ---------------------------------------------------------------------- */
#define VITERBI_BODY(REAL)                                                              \
    const int C = lo_num_states(V, order);                                              \
    if (C < 0) return 1;                                                                \
    const int V1 = V + 1;                                                               \
    const size_t fr = (size_t)C * V1;                                                   \
    _Pragma("omp parallel for schedule(dynamic, 1)")                                    \
    for (int b = 0; b < B; ++b) {                                                       \
        const int L = clamp_len(len[b], T);                                             \
        REAL* cur = (REAL*)malloc((size_t)C * sizeof(REAL));                            \
        REAL* nxt = (REAL*)malloc((size_t)C * sizeof(REAL));                            \
        int32_t* bp = (int32_t*)malloc((size_t)(T > 0 ? T : 1) * C * sizeof(int32_t));  \
        cur[0] = (REAL)0;                                                               \
        for (int q = 1; q < C; ++q) cur[q] = (REAL)NEG_INF;                             \
        for (int t = 0; t < L; ++t) {                                                   \
            const float* wt = w + ((size_t)b * T + t) * fr;                             \
            for (int d = 0; d < C; ++d) { nxt[d] = (REAL)NEG_INF; bp[(size_t)t * C + d] = -1; } \
            for (int q = 0; q < C; ++q)                                                 \
                for (int y = 0; y < V1; ++y) { /* increasing flat arc index */          \
                    volatile REAL v = cur[q] + (REAL)wt[q * V1 + y];                    \
                    int d = lo_next_state(V, order, q, y);                              \
                    if (v > nxt[d]) { nxt[d] = v; bp[(size_t)t * C + d] = q * V1 + y; } \
                }                                                                       \
            REAL* s = cur; cur = nxt; nxt = s;                                          \
        }                                                                               \
        int best = 0;                                                                   \
        for (int q = 1; q < C; ++q) if (cur[q] > cur[best]) best = q;                   \
        score[b] = cur[best];                                                           \
        for (int t = 0; t < T; ++t) labels[(size_t)b * T + t] = -1;                     \
        for (int t = 0; t <= T; ++t) states[(size_t)b * (T + 1) + t] = -1;              \
        states[(size_t)b * (T + 1) + L] = best;                                         \
        for (int t = L - 1; t >= 0; --t) {                                              \
            int arc = bp[(size_t)t * C + states[(size_t)b * (T + 1) + t + 1]];          \
            labels[(size_t)b * T + t] = arc % V1;                                       \
            states[(size_t)b * (T + 1) + t] = arc / V1;                                 \
        }                                                                               \
        free(cur); free(nxt); free(bp);                                                 \
    }                                                                                   \
    return 0;

int lo_viterbi_f32(const float* w, const int32_t* len, int B, int T, int V, int order,
                   int32_t* labels, int32_t* states, float* score)
{
    VITERBI_BODY(float)
}

int lo_viterbi_f64(const float* w, const int32_t* len, int B, int T, int V, int order,
                   int32_t* labels, int32_t* states, double* score)
{
    VITERBI_BODY(double)
}

/* ---------------------------------------------------------------------- */
/* Shared-embedding weight function (Section 3 "weight function", Table 2   */
/* names it with 512 hidden units; the paper prints no formula, the         */
/* benchmark definition supplies it):                                       */
/*   w[b][t][q][y] = sum_k h[k] * W[k][y],  h = tanh(f[b][t] + e[q]).       */
/* f, e, W arrive as bfloat16 bit patterns.  Reading used here: the sum     */
/* f + e is formed in float32, tanh is evaluated in float64, and when       */
/* round_h != 0 the hidden vector is rounded to bfloat16 (nearest even)     */
/* before the contraction, which accumulates in float64.                    */
/* ---------------------------------------------------------------------- */
static float bf16_to_f32(uint16_t v)
{
    uint32_t u = (uint32_t)v << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static double round_to_bf16(double x)
{
    float f = (float)x;  /* |x| <= 1, so the double->float step is harmless here */
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

static void hidden_row(const uint16_t* ft, const uint16_t* eq, int H, int round_h, double* h)
{
    for (int k = 0; k < H; ++k) {
        float x = bf16_to_f32(ft[k]) + bf16_to_f32(eq[k]);
        double v = tanh((double)x);
        h[k] = round_h ? round_to_bf16(v) : v;
    }
}

/* one frame of weights: wt[C][V1] float64 */
static void shared_emb_frame(const uint16_t* ft, const uint16_t* e, const double* Wd,
                             int C, int H, int V1, int round_h, double* wt)
{
#pragma omp parallel
    {
        double* h = (double*)malloc((size_t)H * sizeof(double));
#pragma omp for schedule(static)
        for (int q = 0; q < C; ++q) {
            hidden_row(ft, e + (size_t)q * H, H, round_h, h);
            double* o = wt + (size_t)q * V1;
            for (int y = 0; y < V1; ++y) o[y] = 0.0;
            for (int k = 0; k < H; ++k)
                for (int y = 0; y < V1; ++y) o[y] += h[k] * Wd[(size_t)k * V1 + y];
        }
        free(h);
    }
}

/* materialise the weights: out [B][T][C][V+1] float64 */
int lo_shared_emb_weights(const uint16_t* f, const uint16_t* e, const uint16_t* W,
                          int B, int T, int C, int H, int V1, int round_h, double* out)
{
    double* Wd = (double*)malloc((size_t)H * V1 * sizeof(double));
    for (size_t i = 0; i < (size_t)H * V1; ++i) Wd[i] = (double)bf16_to_f32(W[i]);
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t)
            shared_emb_frame(f + ((size_t)b * T + t) * H, e, Wd, C, H, V1, round_h,
                             out + ((size_t)b * T + t) * C * V1);
    free(Wd);
    return 0;
}

/*
 * Forward-backward with weights computed one frame at a time during the
 * topological visit (Section 4.1 "Remedy"), and the chain of the arc
 * marginals (Eq. 1) through the weight function to its inputs:
 *   dW[k][y]   = sum_{b,t,q} h[k] * gamma[q][y]
 *   dpre[q][k] = (sum_y gamma[q][y] W[k][y]) * (1 - h[k]^2)
 *   df[b][t]   = sum_q dpre[q],   de[q] = sum_{b,t} dpre[q]
 * with h the (possibly bfloat16-rounded) hidden vector: the rounding is
 * treated as the identity in the derivative.
 *   alpha out [B][T+1][C] (caller's scratch, also returned), D out [B],
 *   df out [B][T][H], de out [C][H], dW out [H][V+1]; any gradient pointer
 *   may be NULL (then only the forward pass runs when all three are NULL).
 */
int lo_fused_forward_backward(const uint16_t* f, const uint16_t* e, const uint16_t* W,
                              const int32_t* len, int B, int T, int V, int order, int H,
                              int round_h, double* alpha, double* D,
                              double* df, double* de, double* dW)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const size_t fr = (size_t)C * V1;
    double* Wd = (double*)malloc((size_t)H * V1 * sizeof(double));
    for (size_t i = 0; i < (size_t)H * V1; ++i) Wd[i] = (double)bf16_to_f32(W[i]);
    double* wt = (double*)malloc(fr * sizeof(double));
    double* mx = (double*)malloc((size_t)C * sizeof(double));
    double* tmp = (double*)malloc((size_t)V1 * sizeof(double));
    double* bcur = (double*)malloc((size_t)C * sizeof(double));
    double* bnew = (double*)malloc((size_t)C * sizeof(double));
    double* gam = (double*)malloc(fr * sizeof(double));
    double* h = (double*)malloc((size_t)H * sizeof(double));
    const int want_grad = (df || de || dW);
    if (df) memset(df, 0, (size_t)B * T * H * sizeof(double));
    if (de) memset(de, 0, (size_t)C * H * sizeof(double));
    if (dW) memset(dW, 0, (size_t)H * V1 * sizeof(double));

    for (int b = 0; b < B; ++b) {
        const int L = clamp_len(len[b], T);
        double* al = alpha + (size_t)b * (T + 1) * C;
        al[0] = 0.0;
        for (int q = 1; q < C; ++q) al[q] = NEG_INF;
        for (int t = 0; t < T; ++t) {
            if (t < L) {
                shared_emb_frame(f + ((size_t)b * T + t) * H, e, Wd, C, H, V1, round_h, wt);
                forward_step(al + (size_t)t * C, wt, C, V, order, al + (size_t)(t + 1) * C, mx);
            } else {
                memcpy(al + (size_t)(t + 1) * C, al + (size_t)t * C, (size_t)C * sizeof(double));
            }
        }
        D[b] = lse(al + (size_t)L * C, C);
        if (!want_grad) continue;
        for (int q = 0; q < C; ++q) bcur[q] = 0.0;
        for (int t = L - 1; t >= 0; --t) {
            const uint16_t* ft = f + ((size_t)b * T + t) * H;
            shared_emb_frame(ft, e, Wd, C, H, V1, round_h, wt);
            /* marginals of frame t, then beta_t */
            for (int q = 0; q < C; ++q)
                for (int y = 0; y < V1; ++y) {
                    double a = al[(size_t)t * C + q];
                    gam[q * V1 + y] = (a == NEG_INF) ? 0.0
                        : exp(a + wt[q * V1 + y] + bcur[lo_next_state(V, order, q, y)] - D[b]);
                }
            backward_step(bcur, wt, C, V, order, bnew, tmp);
            { double* s = bcur; bcur = bnew; bnew = s; }
            /* chain through the weight function */
            for (int q = 0; q < C; ++q) {
                const double* g = gam + (size_t)q * V1;
                hidden_row(ft, e + (size_t)q * H, H, round_h, h);
                for (int k = 0; k < H; ++k) {
                    double gw = 0.0;
                    for (int y = 0; y < V1; ++y) gw += g[y] * Wd[(size_t)k * V1 + y];
                    double dpre = gw * (1.0 - h[k] * h[k]);
                    if (df) df[((size_t)b * T + t) * H + k] += dpre;
                    if (de) de[(size_t)q * H + k] += dpre;
                    if (dW)
                        for (int y = 0; y < V1; ++y) dW[(size_t)k * V1 + y] += h[k] * g[y];
                }
            }
        }
    }
    free(Wd); free(wt); free(mx); free(tmp); free(bcur); free(bnew); free(gam); free(h);
    return 0;
}

/* ---------------------------------------------------------------------- */
/* Numerator (Section 2.1) with the weights computed on the fly by the      */
/* shared-embedding weight function (Section 4.1: nothing is materialised). */
/* Only the two arcs leaving every state (t,u) of the intersected lattice   */
/* are evaluated:                                                           */
/*   w0[t][u] = w[t][ctx(u)][0],  w1[t][u] = w[t][ctx(u)][ref[u]],          */
/* then the same recursion as lo_numerator on the (t,u) grid, and the chain */
/* of its arc marginals pb, pl through the weight function:                 */
/*   gw[k]  = pb W[k][0] + pl W[k][ref[u]],  dpre[k] = gw[k] (1 - h[k]^2),  */
/*   df[b][t] += dpre, de[ctx(u)] += dpre,                                  */
/*   dW[k][0] += h[k] pb, dW[k][ref[u]] += h[k] pl,                         */
/* h = the (possibly bfloat16-rounded) hidden vector of (t, ctx(u)).        */
/* Outputs as lo_numerator; df [B][T][H], de [C][H], dW [H][V+1] or NULL.   */
/* ---------------------------------------------------------------------- */
int lo_fused_numerator(const uint16_t* f, const uint16_t* e, const uint16_t* W,
                       const int32_t* len, const int32_t* refs, const int32_t* ulen,
                       int B, int T, int V, int order, int H, int Umax, int round_h,
                       int32_t* ctx, double* a, double* bb, double* N, double* pb, double* pl,
                       double* df, double* de, double* dW)
{
    const int C = lo_num_states(V, order);
    if (C < 0) return 1;
    const int V1 = V + 1;
    const int U1 = Umax + 1;
    double* Wd = (double*)malloc((size_t)H * V1 * sizeof(double));
    for (size_t i = 0; i < (size_t)H * V1; ++i) Wd[i] = (double)bf16_to_f32(W[i]);
    double* h = (double*)malloc((size_t)H * sizeof(double));
    double* w0 = (double*)malloc((size_t)(T > 0 ? T : 1) * U1 * sizeof(double));
    double* w1 = (double*)malloc((size_t)(T > 0 ? T : 1) * U1 * sizeof(double));
    if (df) memset(df, 0, (size_t)B * T * H * sizeof(double));
    if (de) memset(de, 0, (size_t)C * H * sizeof(double));
    if (dW) memset(dW, 0, (size_t)H * V1 * sizeof(double));
    for (int b = 0; b < B; ++b) {
        const int L = clamp_len(len[b], T);
        const int U = ulen[b];
        const int32_t* r = refs + (size_t)b * Umax;
        int32_t* cx = ctx + (size_t)b * U1;
        double* A = a + (size_t)b * (T + 1) * U1;
        double* Bk = bb + (size_t)b * (T + 1) * U1;
        double* PB = pb + (size_t)b * T * U1;
        double* PL = pl + (size_t)b * T * U1;
        for (size_t i = 0; i < (size_t)(T + 1) * U1; ++i) { A[i] = NEG_INF; Bk[i] = NEG_INF; }
        for (size_t i = 0; i < (size_t)T * U1; ++i) { PB[i] = 0.0; PL[i] = 0.0; }
        cx[0] = 0;
        for (int u = 1; u <= Umax; ++u)
            cx[u] = (u <= U) ? lo_next_state(V, order, cx[u - 1], r[u - 1]) : -1;
        /* the two arc weights of every state of the intersected lattice */
        for (int t = 0; t < L; ++t)
            for (int u = 0; u <= U; ++u) {
                hidden_row(f + ((size_t)b * T + t) * H, e + (size_t)cx[u] * H, H, round_h, h);
                double s0 = 0.0, s1 = 0.0;
                for (int k = 0; k < H; ++k) {
                    s0 += h[k] * Wd[(size_t)k * V1];
                    if (u < U) s1 += h[k] * Wd[(size_t)k * V1 + r[u]];
                }
                w0[(size_t)t * U1 + u] = s0;
                w1[(size_t)t * U1 + u] = (u < U) ? s1 : NEG_INF;
            }
        A[0] = 0.0;
        for (int t = 0; t < L; ++t)
            for (int u = 0; u <= U; ++u) {
                double c[2];
                c[0] = A[(size_t)t * U1 + u] + w0[(size_t)t * U1 + u];
                c[1] = (u >= 1) ? A[(size_t)t * U1 + u - 1] + w1[(size_t)t * U1 + u - 1] : NEG_INF;
                A[(size_t)(t + 1) * U1 + u] = lse(c, 2);
            }
        N[b] = A[(size_t)L * U1 + U];
        Bk[(size_t)L * U1 + U] = 0.0;
        for (int t = L - 1; t >= 0; --t)
            for (int u = 0; u <= U; ++u) {
                double c[2];
                c[0] = w0[(size_t)t * U1 + u] + Bk[(size_t)(t + 1) * U1 + u];
                c[1] = (u < U) ? w1[(size_t)t * U1 + u] + Bk[(size_t)(t + 1) * U1 + u + 1] : NEG_INF;
                Bk[(size_t)t * U1 + u] = lse(c, 2);
            }
        if (N[b] == NEG_INF) continue;
        for (int t = 0; t < L; ++t)
            for (int u = 0; u <= U; ++u) {
                const double av = A[(size_t)t * U1 + u];
                if (av == NEG_INF) continue;
                double p0 = 0.0, p1 = 0.0;
                const double nb = Bk[(size_t)(t + 1) * U1 + u];
                if (nb != NEG_INF) p0 = exp(av + w0[(size_t)t * U1 + u] + nb - N[b]);
                if (u < U) {
                    const double nl = Bk[(size_t)(t + 1) * U1 + u + 1];
                    if (nl != NEG_INF) p1 = exp(av + w1[(size_t)t * U1 + u] + nl - N[b]);
                }
                PB[(size_t)t * U1 + u] = p0;
                PL[(size_t)t * U1 + u] = p1;
                if ((df || de || dW) && (p0 != 0.0 || p1 != 0.0)) {
                    hidden_row(f + ((size_t)b * T + t) * H, e + (size_t)cx[u] * H, H, round_h, h);
                    for (int k = 0; k < H; ++k) {
                        double gw = p0 * Wd[(size_t)k * V1];
                        if (u < U) gw += p1 * Wd[(size_t)k * V1 + r[u]];
                        const double dpre = gw * (1.0 - h[k] * h[k]);
                        if (df) df[((size_t)b * T + t) * H + k] += dpre;
                        if (de) de[(size_t)cx[u] * H + k] += dpre;
                        if (dW) {
                            dW[(size_t)k * V1] += h[k] * p0;
                            if (u < U) dW[(size_t)k * V1 + r[u]] += h[k] * p1;
                        }
                    }
                }
            }
    }
    free(Wd); free(h); free(w0); free(w1);
    return 0;
}
