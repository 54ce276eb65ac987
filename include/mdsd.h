/*
 * mdsd.h -- C ABI of the MI355X (gfx950) sampling-verification library for
 * multi-draft speculative decoding: SpecHub and the RRS / RRS-without-
 * replacement baselines ("SpecHub: Provable Acceleration to Multi-Draft
 * Speculative Decoding").
 *
 * One call handles a batch of B token trees of N nodes each.  Every tree node
 * owns one target row p (V elements) and, if it has children, one draft row q
 * (Sec. 2: p = p(.|prefix), q = q(.|prefix) on the probability simplex).  A
 * node's k children carry the k draft tokens sampled at that node; verifying
 * the node decides which child, if any, is accepted (Sec. 2, token-tree
 * figure).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     allocates nothing, frees nothing and never synchronises: work is queued
 *     on `stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and the call returns at once.  Calls are stateless and re-entrant.
 *   - Return value: MDSD_OK, or a negative MDSD_E_* code for anything the
 *     host can detect; in that case nothing was launched.  Data-dependent
 *     problems (a token id outside [0,V), a SpecHub pair without the hub, a
 *     draft row whose whole mass sits on the hub, a residual without mass) are
 *     reported per node in `outcome` / `flags`, never by trapping.
 *   - B = 0 is an empty batch: the call looks at nothing else, launches
 *     nothing and returns MDSD_OK.
 *   - Trees: nodes in breadth-first order, root = node 0.  With first_child
 *     == NULL the tree is the complete k-ary tree with `depth` levels
 *     (N = (k^depth - 1)/(k - 1); Sec. 5.3 "binary trees of depth d with
 *     2^d - 1 nodes"); the children of n are k*n+1 .. k*n+k.  Otherwise
 *     first_child[n] is the index of node n's first child (its k children are
 *     consecutive) or -1 for a leaf, and `depth` bounds the walk.
 *     Preconditions on the table, which the library cannot check as a whole:
 *     every node but the root is the child of exactly one node (child ranges
 *     do not overlap), and children come after their parent (first_child[n]
 *     > n).  Per entry the kernels and the walk apply one rule: an entry
 *     that is <= n or leaves no room for k children (first_child[n] + k > N)
 *     makes node n a leaf, so no access leaves the arrays and every walk
 *     ends; with overlapping ranges each node is still verified on its own
 *     rows, but which tokens a shared child stands for is the caller's
 *     business.
 *   - Rows: element (b, n, x) of `target` lives at target[(b*N + n)*ld_t + x].
 *     dtype selects fp32 or bf16 storage.  kind = MDSD_PROBS: rows are
 *     probabilities and are used as given (no renormalisation); kind =
 *     MDSD_LOGITS: rows are logits and p = softmax(row / temp_target),
 *     q = softmax(row / temp_draft) (App. D; Sec. 5.1 temperatures), computed
 *     in fp32 inside the kernels.  Row start addresses of target and draft
 *     must have the same offset modulo 16 bytes (true whenever both bases are
 *     16-byte aligned and ld_t == ld_d); any V >= 2 and any element-aligned
 *     base is accepted.  Draft rows of leaves are never read.
 *   - Tokens: `tokens` is [B,N] int32 indexed by CHILD node: tokens[b][c] is
 *     the draft token that child c stands for; the root's entry is unused.
 *   - Uniforms are inputs ([0,1), fp32), so results are a deterministic
 *     function of the arguments.  mdsd_philox_uniform makes them.
 */
#ifndef MDSD_H
#define MDSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MDSD_FP32 0
#define MDSD_BF16 1

#define MDSD_PROBS 0
#define MDSD_LOGITS 1

#define MDSD_MAX_K 8

/* status codes */
#define MDSD_OK 0
#define MDSD_E_NULL (-1)      /* a required pointer is NULL                     */
#define MDSD_E_SHAPE (-2)     /* B < 0, N < 1, V < 2, ld < V, depth < 1, tree/N mismatch */
#define MDSD_E_K (-3)         /* k outside 1..MDSD_MAX_K, or SpecHub with k != 2 (Sec. 4) */
#define MDSD_E_TEMP (-4)      /* kind == logits and a temperature is not > 0    */
#define MDSD_E_DTYPE (-5)     /* unknown dtype or kind                          */
#define MDSD_E_ALIGN (-6)     /* pointer not element-aligned (workspace: 4 bytes), or target/draft rows differ modulo 16 bytes */
#define MDSD_E_WORKSPACE (-7) /* a workspace was given and is smaller than mdsd_workspace_bytes() */
#define MDSD_E_LAUNCH (-8)    /* the HIP runtime refused a launch               */
#define MDSD_E_UNSUPPORTED (-9) /* an output this entry point cannot give was asked for */

/* per-node outcome codes (values >= 0 are the accepted child slot) */
#define MDSD_NONE (-1)      /* no child accepted; token drawn from the residual (a leaf: from p) */
#define MDSD_BAD_PAIR (-2)  /* SpecHub: the two tokens are not {hub, non-hub}   */
#define MDSD_BAD_TOKEN (-3) /* a draft token id is outside [0, V)               */
#define MDSD_UNVISITED (-4) /* *_verify_path only: the walk never reached this node */

/* per-node flag bits */
#define MDSD_FLAG_DEGENERATE_HUB 1 /* draft mass outside the hub is 0: node handled as single-draft on the hub */
#define MDSD_FLAG_ZERO_RESIDUAL 2  /* a residual had no mass; the previous distribution was kept */
#define MDSD_FLAG_Q_EXHAUSTED 4    /* RRSw: no draft mass left after zeroing rejected tokens */
#define MDSD_FLAG_BAD_PAIR 8
#define MDSD_FLAG_BAD_TOKEN 16

/*
 * Statistics of one draft row that both SpecHub calls need: the hub a (Sec. 4: the token of
 * highest draft probability) and the two numbers that normalise q around it.  With
 * pb->draft_stats set, spechub_draft writes one record per node (leaves: hub = -1) and
 * spechub_verify reads them instead of scanning the draft row for them again; a node whose
 * first acceptance test (Alg. 3, the non-hub token) succeeds then never reads its draft row.
 * The records must come from spechub_draft on the same draft rows, dtype, kind and
 * temp_draft: the library cannot check that.  A hub outside [0,V) makes the node
 * MDSD_BAD_PAIR.  Results depend on the pointer only through fp32 rounding of rest_mass (a
 * different summation order).
 * rrs_draft and rrsw_draft write records too (hub = -1, rest_mass = the mass of the whole row,
 * before any token is removed) and rrs_verify / rrsw_verify read them the same way.  Records
 * must come from the draft call of the same method.
 */
typedef struct mdsd_row_stats {
    float max_stored; /* largest stored element of the row (a logit, or a probability)        */
    float rest_mass;  /* sum over y != hub of exp((l(y) - max_stored)/temp_draft) for logits,
                         of q(y) for probabilities: the draft mass outside the hub, times the
                         softmax normaliser when the hub's weight is 1                        */
    int32_t hub;      /* argmax of the stored row, lowest index on ties; -1 on leaves         */
    int32_t reserved; /* written as 0                                                         */
} mdsd_row_stats;

typedef struct mdsd_problem {
    const void* target;         /* device, [B,N,ld_t] rows of the target model            */
    const void* draft;          /* device, [B,N,ld_d] rows of the draft model             */
    int64_t ld_t, ld_d;         /* row strides in elements, >= V                          */
    int32_t dtype;              /* MDSD_FP32 | MDSD_BF16                                  */
    int32_t kind;               /* MDSD_PROBS | MDSD_LOGITS                               */
    float temp_target;          /* used iff kind == MDSD_LOGITS; > 0                      */
    float temp_draft;
    int32_t B, N, V;            /* trees, nodes per tree, vocabulary size                 */
    int32_t k;                  /* children per internal node (drafts per step)           */
    int32_t depth;              /* levels of the tree = max tokens emitted per tree       */
    const int32_t* first_child; /* device [N] or NULL (complete k-ary tree)               */
    mdsd_row_stats* draft_stats; /* device [B,N] or NULL: what spechub_draft learnt
                                   about each draft row, handed on to spechub_verify (below) */
} mdsd_problem;

typedef struct mdsd_result {
    int32_t* outcome;      /* device [B,N], required: accepted child slot or MDSD_* code       */
    int32_t* token;        /* device [B,N], required: the token this node emits (the accepted
                              child's token, else the residual / bonus sample)                 */
    float* resid_mass;     /* device [B,N] or NULL: mass of the node's residual in units of p.
                              SpecHub: sum_x p''(x) (= 1 - total acceptance, whatever the tokens);
                              RRS/RRSw: mass of max(p - c q, 0) when the node returned, i.e. the
                              probability mass the rejections so far left (the product of the
                              rejected rounds' sums of max(p_i - q_i, 0) in Alg. 1; 1 when the
                              first draft was accepted); leaf: sum p.
                              Non-NULL disables SpecHub's early exit.                          */
    int32_t* flags;        /* device [B,N] or NULL: MDSD_FLAG_* bits                           */
    float* resid_prob;     /* device [B,N,V] or NULL (diagnostic): SpecHub: norm(p''); RRS/RRSw:
                              the target distribution as it stood when the node returned (after
                              the rejections made so far); leaf: p                             */
    int32_t* accept_depth; /* device [B] or NULL: number of accepted draft tokens on the path  */
    int32_t* emitted;      /* device [B,depth] or NULL: emitted tokens, -1 padded; tokens per
                              step = accept_depth + 1 (Sec. 5.3 batch efficiency)              */
} mdsd_result;

/*
 * Workspace.  No call needs one: ws may always be NULL.  spechub_verify, rrs_verify and
 * rrsw_verify put a non-NULL workspace to use when they are also asked for the walk
 * (out->accept_depth and out->emitted): it holds one int32 arrival counter per tree, with which
 * the verify kernel walks each tree itself as soon as the tree's last node is done, instead of
 * running the walk as a second launch behind it (same results; one launch less per step, which
 * pays for batches of up to about 3000 tree nodes: beyond that the counting costs more than the
 * launch it saves, and ws = NULL is the faster call).
 *   - mdsd_workspace_bytes(pb) = 4 * pb->B bytes; ws must be 4-byte aligned device memory;
 *     a smaller ws_bytes is MDSD_E_WORKSPACE.
 *   - The counters must be ZERO when the call starts.  Every call leaves them zero again, so a
 *     workspace zero-filled once after its allocation can be handed to call after call.  (If a
 *     call was cut short -- the process went on after a failed launch or a device error -- fill
 *     it with zeros again; counters that do not start at zero give a wrong or missing walk,
 *     never an access outside the arrays.)
 *   - Calls that overlap in time (different streams) need workspaces of their own.
 * The draft calls, the *_verify_path calls and mdsd_tree_walk ignore ws.
 */
size_t mdsd_workspace_bytes(const mdsd_problem* pb);

/*
 * spechub_draft -- sample, for every internal node, the pair (x1, x2) ~ Q of
 * Sec. 4: with hub a = argmax q, Q(x,a) = q(x) and Q(a,x) = q(a) q(x)/(1-q(a))
 * for x != a, 0 elsewhere (Alg. 3, "Sample draft tokens").  Two-stage sampler:
 * x ~ q with u[.,.,0]; if x != a the pair is (x, a); otherwise the second
 * token is drawn with u[.,.,1] from q restricted to tokens other than a.
 * The hub is the lowest index among the maxima of the stored draft row.
 *   u      device [B,N,2] fp32 in [0,1)
 *   tokens device [B,N] out: tokens[b][first_child(n)+j] = x_{j+1}; root = -1
 *   hub    device [B,N] out or NULL: the hub of each internal node, -1 on leaves
 *   flags  device [B,N] out or NULL
 * Requires pb->k == 2.  Reads only pb->draft.
 */
int spechub_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* hub,
                  int32_t* flags, void* ws, size_t ws_bytes, void* stream);

/*
 * spechub_verify -- Alg. 3 (with Alg. 2 GetResidual and the transport plan of
 * App. B.1) for every node, then the tree walk.
 *   pair (x, a): accept x if u0 * q(x) < p(x); else accept a if
 *                u1 * sum_y max(q - p, 0) < max(p(a) - S, 0), where
 *                S = sum_{y != a} max(Q(a,y) - max(p(y) - q(y), 0), 0);
 *   pair (a, x): accept x if u0 * Q(a,x) < max(p(x) - q(x), 0); else accept a
 *                if u1 * S < p(a);
 *   otherwise draw the token with u2 from norm(p''), p''(y) = max(p(y) - q(y)
 *   - Q(a,y), 0) for y != a and 0 at a (App. B.2).  Leaves draw from p with u2.
 *   tokens device [B,N] (see above); u device [B,N,3] = (u0, u1, u2) per node.
 * Requires pb->k == 2.
 */
int spechub_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u,
                   const mdsd_result* out, void* ws, size_t ws_bytes, void* stream);

/*
 * spechub_verify_static -- spechub_verify with the tree walk inside its kernel, for callers that
 * cannot allocate or carry a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The arrival counters live in a device array of the library's
 * own (MDSD_STATIC_MAX_TREES int32, 256 KiB per GPU, held until the process ends); the call
 * allocates nothing, frees nothing and queues one kernel on `stream`.
 *   - Same arguments and results as spechub_verify with a workspace; out->accept_depth and
 *     out->emitted are required (MDSD_E_NULL without them).
 *   - pb->B > MDSD_STATIC_MAX_TREES is refused with MDSD_E_WORKSPACE.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 *     (different streams) race on it and may give wrong or missing walks; calls on one stream,
 *     one after another, are fine.  Every call leaves the counters zero for the next.
 *   - The first call on a device looks up the array's address on that device (no allocation);
 *     the device must be current, as for every call.
 */
#define MDSD_STATIC_MAX_TREES 65536
int spechub_verify_static(const mdsd_problem* pb, const int32_t* tokens, const float* u,
                          const mdsd_result* out, void* stream);

/*
 * rrs_draft / rrsw_draft -- Alg. 1, first step: k tokens per internal node from
 * q, independently (RRS) or without replacement (RRSw; Sec. 3.3 gives both Q).
 *   u device [B,N,k]; tokens device [B,N] out, child-indexed; flags or NULL.
 */
int rrs_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* flags,
              void* ws, size_t ws_bytes, void* stream);
int rrsw_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* flags,
               void* ws, size_t ws_bytes, void* stream);

/*
 * rrs_verify / rrsw_verify -- Alg. 1 for every node, then the tree walk.
 * Round i = 1..k: accept x_i if u_{i-1} * q_i(x_i) < p_i(x_i); else
 * p_{i+1} = norm(max(p_i - q_i, 0)) and, without replacement, q_{i+1} = norm(q_i
 * with q_i(x_i) = 0).  After k rejections the token is drawn from p_{k+1}
 * with u_k.  Leaves draw from p with u_k.
 *   u device [B,N,k+1].
 */
int rrs_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u,
               const mdsd_result* out, void* ws, size_t ws_bytes, void* stream);
int rrsw_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u,
                const mdsd_result* out, void* ws, size_t ws_bytes, void* stream);

/*
 * spechub_verify_path / rrs_verify_path / rrsw_verify_path -- the same verification
 * restricted to the nodes that decide what the step emits (Sec. 2: verification follows the
 * accepted tokens down the tree and stops at the first node that accepts none; the nodes
 * beside that path have no effect on the output).  One workgroup per tree starts at the root,
 * verifies a node exactly as the calls above do (same arguments, same uniforms, same
 * arithmetic, so the same outcome and token), moves to the accepted child and stops like
 * mdsd_tree_walk.  A step then reads accept_depth + 1 target rows per tree instead of N.
 *   out->accept_depth and out->emitted are required (they are the result);
 *   out->outcome, out->token (required), out->flags, out->resid_mass (optional) hold the
 *   visited nodes' values, every other node MDSD_UNVISITED / -1 / 0 / 0;
 *   out->resid_prob must be NULL (MDSD_E_UNSUPPORTED).
 * SpecHub uses pb->draft_stats as spechub_verify does.
 */
int spechub_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u,
                        const mdsd_result* out, void* ws, size_t ws_bytes, void* stream);
int rrs_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u,
                    const mdsd_result* out, void* ws, size_t ws_bytes, void* stream);
int rrsw_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u,
                     const mdsd_result* out, void* ws, size_t ws_bytes, void* stream);

/*
 * mdsd_tree_walk -- the walk alone (Sec. 2: follow accepted children from the
 * root; every visited node emits its token; stop at the first node without an
 * accepted child).  The verify calls run it themselves when out->accept_depth
 * and out->emitted are given.
 */
int mdsd_tree_walk(const mdsd_problem* pb, const int32_t* outcome, const int32_t* token,
                   int32_t* accept_depth, int32_t* emitted, void* stream);

/*
 * mdsd_philox_uniform -- counter-based uniforms (Philox4x32-10, Salmon et al.,
 * SC'11).  out[row*slots + s] = (w >> 8) * 2^-24 with w = word (s & 3) of
 * Philox(counter = (row_lo, row_hi, s >> 2, stream_id), key = (seed_lo,
 * seed_hi)).  out: device [rows, slots] fp32; words: device [rows, slots]
 * uint32 or NULL (the raw words, for tests).  rows = 0 returns MDSD_OK at once.
 */
int mdsd_philox_uniform(uint64_t seed, uint32_t stream_id, int64_t rows, int32_t slots,
                        float* out, uint32_t* words, void* stream);

/* Text for a status code (static storage). */
const char* mdsd_strerror(int code);

/* Library version, major*100 + minor. */
int mdsd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MDSD_H */
