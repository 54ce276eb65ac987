/*
 * mdsd_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU statement of multi-draft speculative decoding's
 * sampling-verification step: SpecHub, RRS and RRS without replacement.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use
 * it.  It shares nothing with the HIP library: no header, no constant, no
 * helper.  Every function takes the uniforms it consumes as arguments, so a
 * run is a deterministic function of (rows, tokens, uniforms).
 *
 * Citations name the paper's sections / algorithms / equations:
 *   "Alg. 1"  Token-level RRS (with the without-replacement variant)
 *   "Alg. 2"  GetResidual
 *   "Alg. 3"  Sampling and Verification with SpecHub
 *   "Sec. 4"  SpecHub: definition of the sparse joint draft distribution Q
 *   "App. B.1" transport plan of the hub token
 *   "App. B.2" correctness proof (Theorem 2) and Corollary 1
 *
 * Readings taken where the paper is silent or garbled are marked READING.
 * Pins: tests/test_oracle_*.py (closed forms, the worked example of the
 * LP figure, exact output distributions, brute-force LP, Philox known
 * answers).  Parity unpinned: the handling of degenerate rows (draft mass
 * entirely on the hub; zero residual mass), which the paper does not define.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_FLAG_DEGENERATE_HUB 1 /* sum_{y!=a} q(y) == 0                    */
#define ORC_FLAG_ZERO_RESIDUAL  2 /* a residual had no mass; fallback taken  */
#define ORC_FLAG_Q_EXHAUSTED    4 /* RRSw: no draft mass left after zeroing  */
#define ORC_FLAG_BAD_PAIR       8 /* SpecHub pair does not contain the hub   */
#define ORC_FLAG_BAD_TOKEN     16 /* token id outside [0, V)                 */

#define ORC_OUTCOME_NONE      (-1)
#define ORC_OUTCOME_BAD_PAIR  (-2)
#define ORC_OUTCOME_BAD_TOKEN (-3)

static double dmax(double a, double b) { return a > b ? a : b; }
static double dmin(double a, double b) { return a < b ? a : b; }

/* ------------------------------------------------------------------ */
/* stored element -> double (exact)                                    */
/* ------------------------------------------------------------------ */
static double bf16_to_double(uint16_t h)
{
    uint32_t w = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* dtype: 0 = fp32, 1 = bf16 */
void orc_row_to_double(const void* row, int dtype, int V, double* out)
{
    if (dtype == 0) {
        const float* r = (const float*)row;
        for (int x = 0; x < V; ++x) out[x] = (double)r[x];
    } else {
        const uint16_t* r = (const uint16_t*)row;
        for (int x = 0; x < V; ++x) out[x] = bf16_to_double(r[x]);
    }
}

/* ------------------------------------------------------------------ */
/* softmax(logits / T)   (App. D uses softmax(u/T); Sec. 2 simplex)    */
/* ------------------------------------------------------------------ */
void orc_softmax(const double* logit, int V, double T, double* prob)
{
    double m = logit[0] / T;
    for (int x = 1; x < V; ++x) m = dmax(m, logit[x] / T);
    double Z = 0.0;
    for (int x = 0; x < V; ++x) {
        prob[x] = exp(logit[x] / T - m);
        Z += prob[x];
    }
    for (int x = 0; x < V; ++x) prob[x] /= Z;
}

/* lowest index among the maxima (READING: Alg. 3 gives no tie rule) */
int orc_argmax(const double* v, int V)
{
    int a = 0;
    for (int x = 1; x < V; ++x)
        if (v[x] > v[a]) a = x;
    return a;
}

/* ------------------------------------------------------------------ */
/* inverse CDF over non-negative weights w with uniform u in [0,1):    */
/* the smallest x whose running sum exceeds u * sum(w).                */
/* READING: strict ">" so that a zero-weight token is never returned;  */
/* if rounding leaves no such x, the last token with positive weight.  */
/* Returns -1 when sum(w) == 0.  *margin = distance of u*W to the      */
/* nearest boundary of the chosen token's interval, relative to W.     */
/* ------------------------------------------------------------------ */
int orc_icdf(const double* w, int V, double u, double* W_out, double* margin)
{
    double W = 0.0;
    for (int x = 0; x < V; ++x) W += w[x];
    if (W_out) *W_out = W;
    if (margin) *margin = INFINITY;
    if (!(W > 0.0)) return -1;
    double t = u * W, c = 0.0, lo = 0.0;
    int last_pos = -1;
    for (int x = 0; x < V; ++x) {
        if (w[x] > 0.0) last_pos = x;
        lo = c;
        c += w[x];
        if (c > t) {
            if (margin) *margin = dmin(t - lo, c - t) / W;
            return x;
        }
    }
    if (margin) *margin = 0.0;
    return last_pos;
}

/* one accept test "r < B/A", evaluated as r*A < B (READING: strict,      */
/* multiplicative, so A == 0 accepts exactly when B > 0).                 */
static int accept_test(double r, double A, double B, double* margin)
{
    if (A > 0.0) {
        double d = fabs(r - B / A);
        if (d < *margin) *margin = d;
    }
    return r * A < B;
}

/* ------------------------------------------------------------------ */
/* Alg. 2  GetResidual(p, q, a)                                        */
/* ------------------------------------------------------------------ */
static void get_residual(const double* p, const double* q, int V, int a,
                         double* p_res, double* q_res)
{
    for (int x = 0; x < V; ++x) {
        if (x == a) continue;
        p_res[x] = dmax(p[x] - q[x], 0.0);
        q_res[x] = dmax(q[x] - p[x], 0.0);
    }
    p_res[a] = p[a];
    q_res[a] = 0.0;
}

/* Sec. 4: the two populated lines of Q.  Q_xa[x] = Q(x,a) = q(x),        */
/* Q_ax[x] = Q(a,x) = q(a) q(x) / (1 - q(a)); both 0 at x = a.            */
/* READING: 1 - q(a) is formed as D = sum_{y != a} q(y), which is the     */
/* same number on the simplex and stays accurate when q(a) is near 1.     */
static double build_Q(const double* q, int V, int a, double* Q_xa, double* Q_ax)
{
    double D = 0.0;
    for (int x = 0; x < V; ++x)
        if (x != a) D += q[x];
    for (int x = 0; x < V; ++x) {
        Q_xa[x] = (x == a) ? 0.0 : q[x];
        Q_ax[x] = (x == a || !(D > 0.0)) ? 0.0 : q[a] * q[x] / D;
    }
    return D;
}

/* ------------------------------------------------------------------ */
/* Sampling the pair (x1, x2) ~ Q  (Alg. 3, "Sample draft tokens")     */
/* READING: the paper names no procedure.  Two stages: x ~ q with u0;  */
/* if x != a the pair is (x, a), which has probability q(x) = Q(x,a);  */
/* if x == a (probability q(a)) a second token x' ~ q restricted to    */
/* y != a with u1 gives (a, x') with probability q(a) q(x')/(1-q(a)).  */
/* ------------------------------------------------------------------ */
int orc_spechub_draft(const double* q, int V, int a, double u0, double u1,
                      int* x1, int* x2, double* margin)
{
    int flags = 0;
    double m0 = INFINITY, m1 = INFINITY;
    int x = orc_icdf(q, V, u0, NULL, &m0);
    if (x != a) {
        *x1 = x;
        *x2 = a;
    } else {
        double* w = (double*)malloc(sizeof(double) * (size_t)V);
        memcpy(w, q, sizeof(double) * (size_t)V);
        w[a] = 0.0;
        int y = orc_icdf(w, V, u1, NULL, &m1);
        free(w);
        if (y < 0) { /* all draft mass on the hub: pair (a, a) */
            y = a;
            m1 = INFINITY;
            flags |= ORC_FLAG_DEGENERATE_HUB;
        }
        *x1 = a;
        *x2 = y;
    }
    if (margin) *margin = dmin(m0, m1);
    return flags;
}

/* ------------------------------------------------------------------ */
/* Alg. 3, verification part, for one node.                            */
/*   (x1, x2): the sampled pair; r0: uniform of the non-hub test;      */
/*   r1: uniform of the hub test; u: uniform of the residual sample.   */
/* READING of the control flow (the printed listing falls through its  */
/* "Return ... with probability" lines): a pair (x, a) first tests x   */
/* against p(x)/Q(x,a), then a against p'(a)/sum Q'(.,a), where p'(a)  */
/* is what the pairs (a, .) left of p(a); a pair (a, x) first tests x  */
/* against p'(x)/Q(a,x), then a against p(a)/sum Q'(a,.).  This is the */
/* order of App. B.1's plan and of the proof of Theorem 2.             */
/* READING: the last residual has weight 0 on the hub (the proof shows */
/* sum Q'(a,.) + sum Q'(.,a) >= p(a), so p''(a) = 0 exactly).          */
/* Outputs: return value = accepted slot (0 or 1) or a negative code;  */
/*   *token; *resid_mass = sum of p''; w_out (optional, V) = p''.      */
/* ------------------------------------------------------------------ */
int orc_spechub_verify(const double* p, const double* q, int V, int a,
                       int x1, int x2, double r0, double r1, double u,
                       int* token, double* resid_mass, double* margin,
                       int* flags_out, double* w_out)
{
    int flags = 0, outcome = ORC_OUTCOME_NONE;
    double mg = INFINITY;
    size_t n = (size_t)V;
    double* buf = (double*)calloc(n * 7, sizeof(double));
    double *Q_xa = buf, *Q_ax = buf + n, *p1 = buf + 2 * n, *Qr_xa = buf + 3 * n,
           *p2 = buf + 4 * n, *Qr_ax = buf + 5 * n, *w = buf + 6 * n;
    *token = -1;

    double D = build_Q(q, V, a, Q_xa, Q_ax);
    /* p', Q'(*,a) = GetResidual(p, Q(*,a), a) */
    get_residual(p, Q_xa, V, a, p1, Qr_xa);
    /* p'', Q'(a,*) = GetResidual(p', Q(a,*), a) */
    get_residual(p1, Q_ax, V, a, p2, Qr_ax);
    double S_ax = 0.0, S_xa = 0.0; /* sum_x Q'(a,x), sum_x Q'(x,a) */
    for (int x = 0; x < V; ++x) {
        S_ax += Qr_ax[x];
        S_xa += Qr_xa[x];
    }
    for (int x = 0; x < V; ++x) w[x] = (x == a) ? 0.0 : p2[x];
    double W = 0.0;
    for (int x = 0; x < V; ++x) W += w[x];
    if (resid_mass) *resid_mass = W;
    if (w_out) memcpy(w_out, w, sizeof(double) * n);

    int decided = 0;
    if (x1 < 0 || x1 >= V || x2 < 0 || x2 >= V) {
        flags |= ORC_FLAG_BAD_TOKEN;
        outcome = ORC_OUTCOME_BAD_TOKEN;
        decided = 1;
    } else if (!(D > 0.0)) {
        /* READING: all draft mass on the hub -> Q is undefined; the node is
         * the single-draft case on token a with q(a) = 1, residual p - q. */
        flags |= ORC_FLAG_DEGENERATE_HUB;
        if (x1 != a || x2 != a) {
            flags |= ORC_FLAG_BAD_PAIR;
            outcome = ORC_OUTCOME_BAD_PAIR;
            decided = 1;
        } else if (accept_test(r0, q[a], p[a], &mg)) {
            outcome = 0;
            *token = a;
            decided = 1;
        }
    } else if (x2 == a && x1 != a) {
        if (accept_test(r0, Q_xa[x1], p[x1], &mg)) {
            outcome = 0;
            *token = x1;
            decided = 1;
        } else {
            double pa1 = dmax(p[a] - S_ax, 0.0); /* p'(a) after the pairs (a,.) */
            if (accept_test(r1, S_xa, pa1, &mg)) {
                outcome = 1;
                *token = a;
                decided = 1;
            }
        }
    } else if (x1 == a && x2 != a) {
        if (accept_test(r0, Q_ax[x2], p1[x2], &mg)) {
            outcome = 1;
            *token = x2;
            decided = 1;
        } else if (accept_test(r1, S_ax, p[a], &mg)) {
            outcome = 0;
            *token = a;
            decided = 1;
        }
    } else {
        flags |= ORC_FLAG_BAD_PAIR;
        outcome = ORC_OUTCOME_BAD_PAIR;
        decided = 1;
    }

    if (!decided) {
        double m2 = INFINITY;
        int y = orc_icdf(w, V, u, NULL, &m2);
        if (y < 0) { /* READING: no residual mass left -> sample p itself */
            flags |= ORC_FLAG_ZERO_RESIDUAL;
            y = orc_icdf(p, V, u, NULL, &m2);
        }
        mg = dmin(mg, m2);
        *token = y;
    }
    if (margin) *margin = mg;
    if (flags_out) *flags_out = flags;
    free(buf);
    return outcome;
}

/* ------------------------------------------------------------------ */
/* Alg. 1  Token-level RRS; without_replacement selects the red lines. */
/*   x[0..k-1] drafts, r[0..k-1] their uniforms, u the residual one.   */
/* READING: inside the reject branch the residual is formed with the   */
/* draft distribution before x_i is zeroed, then x_i is zeroed and q   */
/* renormalised.  A residual without mass (possible only when p <= q   */
/* everywhere, where rejection has probability 0) leaves p unchanged.  */
/* Outputs as above; P_out (optional, V) = the target distribution p   */
/* as it stands when the procedure returns (after i rejections when    */
/* x_{i+1} was accepted; the one "Return x ~ p" draws from otherwise); */
/* mass_out (optional, k) = sum max(p - q, 0) of each rejected round.  */
/* ------------------------------------------------------------------ */
int orc_rrs_verify(const double* p, const double* q, int V, int k,
                   const int* x, const double* r, double u,
                   int without_replacement, int* token, double* margin,
                   int* flags_out, double* P_out, double* mass_out)
{
    int flags = 0, outcome = ORC_OUTCOME_NONE, decided = 0;
    double mg = INFINITY;
    size_t n = (size_t)V;
    double* P = (double*)malloc(sizeof(double) * n * 2);
    double* Qc = P + n;
    memcpy(P, p, sizeof(double) * n);
    memcpy(Qc, q, sizeof(double) * n);
    *token = -1;
    for (int i = 0; i < k; ++i)
        if (x[i] < 0 || x[i] >= V) {
            flags |= ORC_FLAG_BAD_TOKEN;
            outcome = ORC_OUTCOME_BAD_TOKEN;
            decided = 1;
        }
    for (int i = 0; i < k && !decided; ++i) {
        int xi = x[i];
        if (accept_test(r[i], Qc[xi], P[xi], &mg)) {
            outcome = i;
            *token = xi;
            decided = 1;
            break;
        }
        double M = 0.0;
        for (int y = 0; y < V; ++y) M += dmax(P[y] - Qc[y], 0.0);
        if (mass_out) mass_out[i] = M;
        if (M > 0.0) {
            for (int y = 0; y < V; ++y) P[y] = dmax(P[y] - Qc[y], 0.0) / M;
        } else {
            flags |= ORC_FLAG_ZERO_RESIDUAL;
        }
        if (without_replacement) {
            Qc[xi] = 0.0;
            double s = 0.0;
            for (int y = 0; y < V; ++y) s += Qc[y];
            if (s > 0.0) {
                for (int y = 0; y < V; ++y) Qc[y] /= s;
            } else { /* READING: nothing left to draft from -> go to the end */
                flags |= ORC_FLAG_Q_EXHAUSTED;
                break;
            }
        }
    }
    if (P_out) memcpy(P_out, P, sizeof(double) * n);
    if (!decided) {
        double m2 = INFINITY;
        int y = orc_icdf(P, V, u, NULL, &m2);
        mg = dmin(mg, m2);
        *token = y;
    }
    if (margin) *margin = mg;
    if (flags_out) *flags_out = flags;
    free(P);
    return outcome;
}

/* Alg. 1, first step: k drafts from q, independently (RRS) or without  */
/* replacement (RRSw: earlier picks get weight 0; the inverse CDF       */
/* rescales by the remaining mass, which is the renormalised q).        */
/* READING: if no mass remains the previous token is repeated.          */
int orc_rrs_draft(const double* q, int V, int k, const double* u,
                  int without_replacement, int* x, double* margin)
{
    int flags = 0;
    double mg = INFINITY;
    double* w = (double*)malloc(sizeof(double) * (size_t)V);
    memcpy(w, q, sizeof(double) * (size_t)V);
    for (int i = 0; i < k; ++i) {
        double m = INFINITY;
        int y = orc_icdf(w, V, u[i], NULL, &m);
        if (y < 0) {
            flags |= ORC_FLAG_Q_EXHAUSTED;
            y = (i > 0) ? x[i - 1] : 0;
            m = INFINITY;
        }
        x[i] = y;
        mg = dmin(mg, m);
        if (without_replacement) w[y] = 0.0;
    }
    free(w);
    if (margin) *margin = mg;
    return flags;
}

/* ------------------------------------------------------------------ */
/* Token tree (Sec. 2, token-tree figure; Sec. 5 "binary trees of      */
/* depth d with 2^d - 1 nodes").  Nodes in BFS order, root 0; the      */
/* children of n are first_child[n] .. first_child[n]+k-1, or, when    */
/* first_child is NULL, k*n+1 .. k*n+k while those are < N.            */
/* ------------------------------------------------------------------ */
static int child0(const int32_t* first_child, int n, int k, int N)
{
    if (first_child) return first_child[n];
    long c = (long)k * n + 1;
    return (c + k <= (long)N) ? (int)c : -1;
}

/* Walk: from the root follow accepted children; every visited node emits
 * its token; stop at the first node without an accepted child.           */
void orc_tree_walk(const int32_t* outcome, const int32_t* token, int N, int k,
                   const int32_t* first_child, int max_depth,
                   int32_t* accept_depth, int32_t* emitted)
{
    int n = 0, depth = 0;
    for (int i = 0; i < max_depth; ++i) emitted[i] = -1;
    for (;;) {
        if (depth < max_depth) emitted[depth] = token[n];
        int c0 = child0(first_child, n, k, N);
        if (c0 < 0 || outcome[n] < 0 || depth + 1 >= max_depth) break;
        n = c0 + outcome[n];
        ++depth;
    }
    *accept_depth = depth;
}

/* ------------------------------------------------------------------ */
/* Batch drivers: rows as stored ([B,N,ld] of fp32 or bf16; kind 0 =   */
/* probabilities used as given, 1 = logits -> softmax(l / T)).         */
/* method: 0 SpecHub, 1 RRS, 2 RRSw.  u is [B,N,k+1] (SpecHub: k = 2). */
/* tokens is [B,N], indexed by child node; the root's entry is unused. */
/* Leaves are the k = 0 case of Alg. 1: token ~ p with the last        */
/* uniform slot.                                                       */
/* ------------------------------------------------------------------ */
typedef struct {
    const void* target;
    const void* draft;
    int64_t ld_t, ld_d;
    int dtype, kind;
    double temp_target, temp_draft;
    int B, N, V, k, depth;
    const int32_t* first_child;
} orc_problem;

static const void* row_ptr(const void* base, int dtype, int64_t ld, int64_t r)
{
    size_t es = dtype == 0 ? 4 : 2;
    return (const char*)base + (size_t)(r * ld) * es;
}

static void load_row(const void* base, int dtype, int kind, int64_t ld, int64_t r,
                     int V, double T, double* stored, double* prob)
{
    orc_row_to_double(row_ptr(base, dtype, ld, r), dtype, V, stored);
    if (kind == 1)
        orc_softmax(stored, V, T, prob);
    else
        memcpy(prob, stored, sizeof(double) * (size_t)V);
}

int orc_batch_verify(const orc_problem* pb, int method, const int32_t* tokens,
                     const float* u, int32_t* outcome, int32_t* token_out,
                     double* resid_mass, double* margin, int32_t* flags,
                     int32_t* accept_depth, int32_t* emitted,
                     double* resid_prob /* optional [B,N,V] */, int nthreads)
{
    const int B = pb->B, N = pb->N, V = pb->V, k = pb->k;
    if (method == 0 && k != 2) return -1;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int64_t r = 0; r < (int64_t)B * N; ++r) {
        int n = (int)(r % N);
        size_t nv = (size_t)V;
        double* buf = (double*)malloc(sizeof(double) * nv * 5);
        double *ps = buf, *p = buf + nv, *qs = buf + 2 * nv, *q = buf + 3 * nv,
               *res = buf + 4 * nv;
        const float* ur = u + r * (k + 1);
        int tok = -1, fl = 0, oc = ORC_OUTCOME_NONE;
        double mg = INFINITY, rm = 0.0;
        load_row(pb->target, pb->dtype, pb->kind, pb->ld_t, r, V, pb->temp_target, ps, p);
        int c0 = child0(pb->first_child, n, k, N);
        if (c0 < 0) { /* leaf: bonus token ~ p */
            tok = orc_icdf(p, V, (double)ur[k], &rm, &mg);
            memcpy(res, p, sizeof(double) * nv);
        } else {
            load_row(pb->draft, pb->dtype, pb->kind, pb->ld_d, r, V, pb->temp_draft, qs, q);
            const int32_t* xt = tokens + (r - n) + c0;
            if (method == 0) {
                int a = orc_argmax(qs, V); /* hub: argmax of the stored draft row */
                oc = orc_spechub_verify(p, q, V, a, xt[0], xt[1], (double)ur[0],
                                        (double)ur[1], (double)ur[2], &tok, &rm, &mg,
                                        &fl, res);
            } else {
                int xi[16];
                double ri[16];
                for (int i = 0; i < k; ++i) {
                    xi[i] = xt[i];
                    ri[i] = (double)ur[i];
                }
                double mass[16];
                for (int i = 0; i < k; ++i) mass[i] = 1.0;
                oc = orc_rrs_verify(p, q, V, k, xi, ri, (double)ur[k], method == 2,
                                    &tok, &mg, &fl, res, mass);
                /* mass of the unnormalised k-fold residual: the product of the
                 * per-round masses (a round without mass changes nothing) */
                rm = 1.0;
                for (int i = 0; i < k; ++i)
                    if (mass[i] > 0.0) rm *= mass[i];
            }
        }
        outcome[r] = oc;
        token_out[r] = tok;
        if (resid_mass) resid_mass[r] = rm;
        if (margin) margin[r] = mg;
        if (flags) flags[r] = fl;
        if (resid_prob) {
            double s = 0.0;
            for (int y = 0; y < V; ++y) s += res[y];
            for (int y = 0; y < V; ++y)
                resid_prob[(size_t)r * nv + (size_t)y] = s > 0.0 ? res[y] / s : 0.0;
        }
        free(buf);
    }
    if (accept_depth && emitted)
        for (int b = 0; b < B; ++b)
            orc_tree_walk(outcome + (size_t)b * N, token_out + (size_t)b * N, N, k,
                          pb->first_child, pb->depth, accept_depth + b,
                          emitted + (size_t)b * pb->depth);
    return 0;
}

/* u is [B,N,k] (SpecHub: [B,N,2]); tokens [B,N] child-indexed, root = -1;
 * hub [B,N] (SpecHub only, -1 on leaves) may be NULL.                    */
int orc_batch_draft(const orc_problem* pb, int method, const float* u,
                    int32_t* tokens, int32_t* hub, double* margin, int32_t* flags,
                    int nthreads)
{
    const int B = pb->B, N = pb->N, V = pb->V, k = pb->k;
    if (method == 0 && k != 2) return -1;
    (void)nthreads;
    for (int b = 0; b < B; ++b) tokens[(size_t)b * N] = -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int64_t r = 0; r < (int64_t)B * N; ++r) {
        int n = (int)(r % N);
        int c0 = child0(pb->first_child, n, k, N);
        if (hub) hub[r] = -1;
        if (margin) margin[r] = INFINITY;
        if (flags) flags[r] = 0;
        if (c0 < 0) continue;
        size_t nv = (size_t)V;
        double* qs = (double*)malloc(sizeof(double) * nv * 2);
        double* q = qs + nv;
        load_row(pb->draft, pb->dtype, pb->kind, pb->ld_d, r, V, pb->temp_draft, qs, q);
        int32_t* xt = tokens + (r - n) + c0;
        const float* ur = u + r * k;
        double mg = INFINITY;
        int fl;
        if (method == 0) {
            int a = orc_argmax(qs, V), x1, x2;
            fl = orc_spechub_draft(q, V, a, (double)ur[0], (double)ur[1], &x1, &x2, &mg);
            xt[0] = x1;
            xt[1] = x2;
            if (hub) hub[r] = a;
        } else {
            int xi[16];
            double ui[16];
            for (int i = 0; i < k; ++i) ui[i] = (double)ur[i];
            fl = orc_rrs_draft(q, V, k, ui, method == 2, xi, &mg);
            for (int i = 0; i < k; ++i) xt[i] = xi[i];
        }
        if (margin) margin[r] = mg;
        if (flags) flags[r] = fl;
        free(qs);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random         */
/* numbers: as easy as 1, 2, 3", SC'11).  Written from the published   */
/* round function: two 32x32->64 multiplies, swap-and-xor with the     */
/* key, key bumped by the Weyl constants every round.                  */
/* ------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t m0 = (uint64_t)0xD2511F53u * c0;
        uint64_t m1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(m1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)m1;
        uint32_t n2 = (uint32_t)(m0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)m0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniforms for `rows` rows of `slots` values: element (row, s) is word
 * s & 3 of Philox(counter = (row_lo, row_hi, s >> 2, stream), key =
 * (seed_lo, seed_hi)), mapped to [0,1) as (word >> 8) * 2^-24, which is
 * exact in fp32.  If words is not NULL it receives the raw 32-bit words. */
void orc_philox_uniform(uint64_t seed, uint32_t stream, int64_t rows, int slots,
                        float* out, uint32_t* words)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t r = 0; r < rows; ++r)
        for (int s = 0; s < slots; ++s) {
            uint32_t ctr[4] = { (uint32_t)((uint64_t)r), (uint32_t)((uint64_t)r >> 32),
                                (uint32_t)(s >> 2), stream };
            uint32_t o[4];
            orc_philox4x32_10(ctr, key, o);
            uint32_t wv = o[s & 3];
            if (words) words[r * slots + s] = wv;
            if (out) out[r * slots + s] = (float)(wv >> 8) * (1.0f / 16777216.0f);
        }
}
