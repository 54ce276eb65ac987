// Host side of the sampling-verification library (gfx950): validation of a problem, the choice
// of a kernel family (spechub_resident.hip, rrs_resident.hip, verify_generic_*.hip,
// draft_*.hip; the device code they share is in node_common.h), the tree walk and Philox
// kernels, and the C entry points.
#include "launch.h"
#include "launch_half.h"
#include "launch_small.h"

#include <atomic>

namespace mdsd {

// ---------------------------------------------------------------- tree walk
// The walk as a launch of its own (see group_walk and wave_walk in node_common.h).  Trees of at most
// 64 nodes: a group of W lanes per tree (W = the power of two from N up), 64 / W trees per wavefront.
// Larger trees (W = 0): one wavefront per tree.
__global__ __launch_bounds__(256) void tree_walk_kernel(const int32_t* outcome, const int32_t* token, int B, int N,
                                                        int W, int k, int depth, const int32_t* first_child,
                                                        int32_t* accept_depth, int32_t* emitted)
{
    const int wave = blockIdx.x * (blockDim.x / 64) + (int)(threadIdx.x / 64);
    if (W == 0) {
        if (wave < B) wave_walk<false>(outcome, token, wave, N, k, depth, first_child, accept_depth, emitted);
        return;
    }
    const int per_wave = 64 / W;
    if ((int64_t)wave * per_wave >= B) return;  // the whole wavefront: the shuffles below need every lane of the others
    const int b = wave * per_wave + (int)(threadIdx.x & 63) / W;
    group_walk<false>(outcome, token, b < B ? b : 0, b < B, W, N, k, depth, first_child, accept_depth, emitted);
}

// ---------------------------------------------------------------- Philox4x32-10
// Salmon, Moraes, Dror, Shaw, SC'11: ten rounds of two 32x32->64 multiplies,
// swap and xor with the key; the key advances by the two Weyl constants.
__global__ void philox_uniform_kernel(uint32_t k0, uint32_t k1, uint32_t stream_id, int64_t rows,
                                      int slots, float* out, uint32_t* words)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int blocks_per_row = (slots + 3) >> 2;
    if (i >= rows * blocks_per_row) return;
    const int64_t row = i / blocks_per_row;
    const int blk = (int)(i - row * blocks_per_row);
    uint32_t c0 = (uint32_t)row, c1 = (uint32_t)((uint64_t)row >> 32), c2 = (uint32_t)blk, c3 = stream_id;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0;
        c1 = l1;
        c2 = n2;
        c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    const uint32_t w[4] = {c0, c1, c2, c3};
    for (int j = 0; j < 4; ++j) {
        const int s = blk * 4 + j;
        if (s < slots) {
            if (out) out[row * slots + s] = (float)(w[j] >> 8) * (1.0f / 16777216.0f);
            if (words) words[row * slots + s] = w[j];
        }
    }
}
// ---------------------------------------------------------------- host side
static int complete_tree_nodes(int k, int depth, int64_t* n_internal)
{
    int64_t n = 0, level = 1, internal = 0;
    for (int d = 0; d < depth; ++d) {
        if (d == depth - 1) internal = n;
        n += level;
        level *= k;
        if (n > INT_MAX) return -1;
    }
    *n_internal = internal;
    return (int)n;
}

// what validate returns for a batch of no trees: the entry points then return MDSD_OK at once
static constexpr int kEmptyBatch = 1;

static int validate(const mdsd_problem* pb, int method, bool need_target, Params* P)
{
    if (!pb) return MDSD_E_NULL;
    if (pb->B == 0) return kEmptyBatch;
    if (!pb->draft || (need_target && !pb->target)) return MDSD_E_NULL;
    if (pb->dtype != MDSD_FP32 && pb->dtype != MDSD_BF16) return MDSD_E_DTYPE;
    if (pb->kind != MDSD_PROBS && pb->kind != MDSD_LOGITS) return MDSD_E_DTYPE;
    if (pb->B < 1 || pb->N < 1 || pb->V < 2 || pb->depth < 1) return MDSD_E_SHAPE;
    if (pb->ld_d < pb->V || (need_target && pb->ld_t < pb->V)) return MDSD_E_SHAPE;
    if (pb->k < 1 || pb->k > MDSD_MAX_K) return MDSD_E_K;
    if (method == kSpecHub && pb->k != 2) return MDSD_E_K;
    if (pb->kind == MDSD_LOGITS) {
        if (!(pb->temp_draft > 0.f)) return MDSD_E_TEMP;
        if (need_target && !(pb->temp_target > 0.f)) return MDSD_E_TEMP;
    }
    const int es = pb->dtype == MDSD_FP32 ? 4 : 2;
    const int per_chunk = 16 / es;
    // vocabulary bound of the per-slab partial sums kept in LDS
    if ((int64_t)pb->V + per_chunk > (int64_t)kMaxSlabs * 64 * per_chunk) return MDSD_E_SHAPE;
    if ((int64_t)pb->B * pb->N > INT_MAX) return MDSD_E_SHAPE;
    const uintptr_t at = (uintptr_t)pb->target, ad = (uintptr_t)pb->draft;
    if ((ad % es) != 0 || (need_target && (at % es) != 0)) return MDSD_E_ALIGN;
    if (need_target) {
        // every pair of rows must share its offset modulo 16 bytes
        if ((at & 15) != (ad & 15)) return MDSD_E_ALIGN;
        if (pb->B * (int64_t)pb->N > 1 && ((pb->ld_t * es) & 15) != ((pb->ld_d * es) & 15)) return MDSD_E_ALIGN;
    }
    int64_t n_internal = 0;
    if (!pb->first_child) {
        const int n = complete_tree_nodes(pb->k, pb->depth, &n_internal);
        if (n != pb->N) return MDSD_E_SHAPE;
    }
    P->target = pb->target;
    P->draft = pb->draft;
    P->ld_t = pb->ld_t;
    P->ld_d = pb->ld_d;
    P->temp_target = pb->temp_target;
    P->temp_draft = pb->temp_draft;
    P->scale_t = pb->kind == MDSD_LOGITS && need_target ? kLog2e / pb->temp_target : 0.f;
    P->scale_d = pb->kind == MDSD_LOGITS ? kLog2e / pb->temp_draft : 0.f;
    P->B = pb->B;
    P->N = pb->N;
    P->V = pb->V;
    P->k = pb->k;
    P->depth = pb->depth;
    P->n_internal = (int)n_internal;
    P->first_child = pb->first_child;
    return MDSD_OK;
}

// chunks per lane that hold a whole row in registers; 0 = stream the row in every pass
static int resident_chunks(const mdsd_problem* pb)
{
    const int per_chunk = pb->dtype == MDSD_FP32 ? 4 : 8;
    // worst case head of per_chunk - 1 masked elements in front of the row
    const int64_t nchunk = ((int64_t)pb->V + 2 * per_chunk - 2) / per_chunk;
    const int64_t per_lane = (nchunk + kWG - 1) / kWG;
    if (per_lane <= 4) return 4;
    if (per_lane <= 8) return 8;
    if (per_lane <= 16) return 16;
    return 0;
}
// Short rows go to a build of the generic kernels with fewer threads per node (1, 2 or 4 wavefronts:
// four chunks per lane) instead of one 512-thread workgroup most of whose wavefronts would hold no
// part of the row; 0 = the main build
static int small_build(const mdsd_problem* pb)
{
    const int per_chunk = pb->dtype == MDSD_FP32 ? 4 : 8;
    const int64_t nchunk = ((int64_t)pb->V + 2 * per_chunk - 2) / per_chunk;
    if (nchunk <= mdsd_wave::kMaxChunks) return 1;
    if (nchunk <= mdsd_pair::kMaxChunks) return 2;
    if (nchunk <= mdsd_quad::kMaxChunks) return 4;
    return 0;
}
// true when some element of some row may need masking: a row that does not start on a
// 16-byte boundary, or a vocabulary that is not a whole number of 16-byte chunks
static bool rows_need_mask(const mdsd_problem* pb)
{
    const int es = pb->dtype == MDSD_FP32 ? 4 : 2;
    const uintptr_t at = (uintptr_t)pb->target, ad = (uintptr_t)pb->draft;
    return (at & 15) || (ad & 15) || ((pb->ld_t * es) & 15) || ((pb->ld_d * es) & 15) || (pb->V % (16 / es));
}
// One workgroup per node.  Complete trees with more than one node: (trees, nodes), which
// node_of_block() reads without a division (a one-node tree keeps gridDim.y == 1, which is how the
// kernels tell the two numberings apart; there the single node is node 0 of tree blockIdx.x
// either way).  Explicit topologies, and trees of more nodes than a grid's second dimension
// holds: one dimension.
// Rows too long for registers (nit == 0) keep the one-dimensional numbering as well: there
// the workgroups that run side by side would read rows a whole tree apart, which measured 4 %
// slower than rows next to each other (config 4).
static dim3 node_grid(const Params& P, int nit)
{
    if (P.first_child == nullptr && P.N > 1 && P.N <= 65535 && nit > 0) return dim3((unsigned)P.B, (unsigned)P.N);
    return dim3((unsigned)(P.B * P.N));
}

// tree nodes per batch from which the 256-thread verify kernels take over from the 512-thread ones
constexpr int64_t kHalfWidthMinNodes = 2300;

// path == false: one workgroup per node.  path == true: one workgroup per tree.
static void launch_verify(int method, const mdsd_problem* pb, const Params& P, bool path, hipStream_t st)
{
    const bool lg = pb->kind == MDSD_LOGITS;
    int nit = resident_chunks(pb);
    const dim3 grid = path ? dim3((unsigned)P.B) : node_grid(P, nit), block(kWG);
    switch (small_build(pb)) {
    case 1: mdsd_wave::launch_verify(method, pb->dtype, lg, path, grid, st, P); return;
    case 2: mdsd_pair::launch_verify(method, pb->dtype, lg, path, grid, st, P); return;
    case 4: mdsd_quad::launch_verify(method, pb->dtype, lg, path, grid, st, P); return;
    default: break;
    }
    // Rows of eight chunks per lane, the draft call's records at hand, and a batch that fills the chip
    // several times over: 256 threads per node with sixteen chunks per lane, four nodes per CU
    // instead of three (config-3 rows, 31 nodes per tree: B = 80 41.8 -> 41.1 us, B = 128 58.7 -> 56.6 us,
    // B = 1024 437 -> 410 us; B = 64 33.3 -> 34.3 us and B = 32 21.5 -> 23.5 us, hence the bound)
    const bool half_width = lg && nit == 8 && !path && P.stats_in != nullptr &&
                            (int64_t)P.B * P.N >= kHalfWidthMinNodes;
    if (half_width && method == kSpecHub) {
        mdsd_half::launch_spechub(pb->dtype, rows_need_mask(pb), grid, st, P);
        return;
    }
    if (half_width && method != kSpecHub && mdsd_half::rrs_covers(pb->dtype, rows_need_mask(pb))) {
        mdsd_half::launch_rrs(method == kRRSw, pb->dtype, rows_need_mask(pb), grid, st, P);
        return;
    }
    if (method == kSpecHub && lg && nit > 0) {
        launch_spechub_resident(pb->dtype, nit, rows_need_mask(pb), path, grid, block, st, P);
        return;
    }
    if (method != kSpecHub && lg && P.stats_in != nullptr && !path &&
        rrs_resident_covers(pb->dtype, nit, rows_need_mask(pb))) {
        // logit rows in registers, the draft call's records at hand
        launch_rrs_resident(method == kRRSw, pb->dtype, nit, rows_need_mask(pb), grid, block, st, P);
        return;
    }
    // The generic RRS rounds hold many registers beside two resident rows (8 chunks per lane and
    // row: more than 200, one workgroup per CU): from that size on the rows are streamed, which
    // measures faster (config 3, rrsw_verify: 117 -> 82 us).
    if (method != kSpecHub && nit >= 8) nit = 0;
    if (method == kSpecHub)
        launch_verify_generic_spechub(pb->dtype, lg, nit, path, grid, block, st, P);
    else if (method == kRRS)
        launch_verify_generic_rrs(pb->dtype, lg, nit, path, grid, block, st, P);
    else
        launch_verify_generic_rrsw(pb->dtype, lg, nit, path, grid, block, st, P);
}

static void launch_draft(int method, const mdsd_problem* pb, const Params& P, hipStream_t st)
{
    const bool lg = pb->kind == MDSD_LOGITS;
    int nit = resident_chunks(pb);
    // Rows of sixteen chunks per lane are streamed: the draft kernel with such a row in registers
    // fits two workgroups on a CU, the streaming one four, and its one-sweep statistics are the
    // cheaper (V = 50304, B = 64: spechub_draft 33.7 -> 24.7 us, rrsw_draft 47.2 -> 26.8 us).  At
    // eight chunks per lane the row in registers wins (V = 32000: 18.8 against 19.4 us).
    if (nit == 16 && lg) nit = 0;  // (rows of probabilities have no one-sweep form and stay in registers)
    const dim3 grid = node_grid(P, nit), block(kWG);
    switch (small_build(pb)) {
    case 1: mdsd_wave::launch_draft(method, pb->dtype, lg, st, P); return;
    case 2: mdsd_pair::launch_draft(method, pb->dtype, lg, st, P); return;
    case 4: mdsd_quad::launch_draft(method, pb->dtype, lg, st, P); return;
    default: break;
    }
    const int es = pb->dtype == MDSD_FP32 ? 4 : 2;
    const bool masked = ((uintptr_t)pb->draft & 15) || ((pb->ld_d * es) & 15) || (pb->V % (16 / es));
    if (method == kSpecHub)
        launch_draft_spechub(pb->dtype, lg, nit, masked, grid, block, st, P);
    else if (method == kRRS)
        launch_draft_rrs(pb->dtype, lg, nit, masked, grid, block, st, P);
    else
        launch_draft_rrsw(pb->dtype, lg, nit, masked, grid, block, st, P);
}

static int walk(const mdsd_problem* pb, const int32_t* outcome, const int32_t* token,
                int32_t* accept_depth, int32_t* emitted, hipStream_t st)
{
    int W = 0;  // lanes per tree
    if (pb->N <= 64) {
        W = 1;
        while (W < pb->N) W *= 2;
    }
    const int64_t waves = W ? ((int64_t)pb->B * W + 63) / 64 : (int64_t)pb->B;
    const int waves_per_block = 4;
    hipLaunchKernelGGL(tree_walk_kernel, dim3((unsigned)((waves + waves_per_block - 1) / waves_per_block)),
                       dim3(64 * waves_per_block), 0, st, outcome, token, pb->B, pb->N, W, pb->k, pb->depth,
                       pb->first_child, accept_depth, emitted);
    return hipGetLastError() == hipSuccess ? MDSD_OK : MDSD_E_LAUNCH;
}

// bytes of workspace the full verify calls take when they walk the trees themselves
static size_t walk_workspace_bytes(int B) { return B > 0 ? (size_t)B * sizeof(int32_t) : 0; }

// tree_count: per-tree arrival counters (zero on entry) when the kernel is to walk the trees
// itself, nullptr when the walk is a launch of its own
static int verify_entry(int method, const mdsd_problem* pb, const int32_t* tokens, const float* u,
                        const mdsd_result* out, bool path, int32_t* tree_count, void* stream)
{
    Params P = {};
    const int rc = validate(pb, method, true, &P);
    if (rc == kEmptyBatch) return MDSD_OK;
    if (rc != MDSD_OK) return rc;
    if (!tokens || !u || !out || !out->outcome || !out->token) return MDSD_E_NULL;
    if ((out->accept_depth == nullptr) != (out->emitted == nullptr)) return MDSD_E_NULL;
    if (path && !out->accept_depth) return MDSD_E_NULL;
    if (path && out->resid_prob) return MDSD_E_UNSUPPORTED;
    const bool walk_inside = !path && out->accept_depth && tree_count;
    P.accept_depth = out->accept_depth;
    P.emitted = out->emitted;
    P.tree_count = walk_inside ? tree_count : nullptr;
    P.tokens = tokens;
    P.u = u;
    P.outcome = out->outcome;
    P.token = out->token;
    P.resid_mass = out->resid_mass;
    P.flags = out->flags;
    P.resid_prob = out->resid_prob;
    P.stats_in = pb->draft_stats;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();
    launch_verify(method, pb, P, path, st);
    if (hipGetLastError() != hipSuccess) return MDSD_E_LAUNCH;
    if (path || walk_inside) return MDSD_OK;  // the walk is part of the kernel
    if (out->accept_depth) return walk(pb, out->outcome, out->token, out->accept_depth, out->emitted, st);
    return MDSD_OK;
}

// the full verify calls: a workspace, when given, holds the trees' arrival counters
static int verify_with_workspace(int method, const mdsd_problem* pb, const int32_t* tokens, const float* u,
                                 const mdsd_result* out, void* ws, size_t ws_bytes, void* stream)
{
    if (ws && pb && ws_bytes < walk_workspace_bytes(pb->B)) return MDSD_E_WORKSPACE;
    if (ws && ((uintptr_t)ws & 3)) return MDSD_E_ALIGN;
    return verify_entry(method, pb, tokens, u, out, false, (int32_t*)ws, stream);
}

// ---------------------------------------------------------------- arrival counters owned by the library
// For callers that cannot allocate a workspace (code under HIP graph capture, serving loops that
// must not call hipMalloc): the arrival counters of up to MDSD_STATIC_MAX_TREES trees in a
// file-scope device array, zero when the code object is loaded and left zero by every call.  Each
// GPU holds its own copy at its own address; the array's name is a host-side stand-in, so the
// address on the current device is asked for once per device and used from then on.
static __device__ __align__(256) int32_t scratch[MDSD_STATIC_MAX_TREES];

static constexpr int kMaxDevices = 64;
static std::atomic<int32_t*> scratch_on_device[kMaxDevices];

static int static_tree_counters(int32_t** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MDSD_E_LAUNCH;
    int32_t* ptr = scratch_on_device[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        // two threads asking at once get the same answer
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return MDSD_E_LAUNCH;
        }
        scratch_on_device[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return MDSD_OK;
}

static int draft_entry(int method, const mdsd_problem* pb, const float* u, int32_t* tokens,
                       int32_t* hub, int32_t* flags, void* stream)
{
    Params P = {};
    const int rc = validate(pb, method, false, &P);
    if (rc == kEmptyBatch) return MDSD_OK;
    if (rc != MDSD_OK) return rc;
    if (!u || !tokens) return MDSD_E_NULL;
    P.u = u;
    P.tokens_out = tokens;
    P.hub_out = hub;
    P.flags = flags;
    P.stats_out = pb->draft_stats;
    hipStream_t st = (hipStream_t)stream;
    (void)hipGetLastError();
    launch_draft(method, pb, P, st);
    return hipGetLastError() == hipSuccess ? MDSD_OK : MDSD_E_LAUNCH;
}

}  // namespace mdsd

// ---------------------------------------------------------------- C ABI
extern "C" {

size_t mdsd_workspace_bytes(const mdsd_problem* pb)
{
    // every intermediate of a node lives in registers and LDS; the workspace holds one arrival
    // counter per tree for the verify calls that walk the trees inside their kernel
    return pb ? mdsd::walk_workspace_bytes(pb->B) : 0;
}

int spechub_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* hub, int32_t* flags,
                  void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::draft_entry(mdsd::kSpecHub, pb, u, tokens, hub, flags, stream);
}

int rrs_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* flags, void* ws,
              size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::draft_entry(mdsd::kRRS, pb, u, tokens, nullptr, flags, stream);
}

int rrsw_draft(const mdsd_problem* pb, const float* u, int32_t* tokens, int32_t* flags, void* ws,
               size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::draft_entry(mdsd::kRRSw, pb, u, tokens, nullptr, flags, stream);
}

int spechub_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                   void* ws, size_t ws_bytes, void* stream)
{
    return mdsd::verify_with_workspace(mdsd::kSpecHub, pb, tokens, u, out, ws, ws_bytes, stream);
}

int spechub_verify_static(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                          void* stream)
{
    if (!pb) return MDSD_E_NULL;
    if (pb->B > MDSD_STATIC_MAX_TREES) return MDSD_E_WORKSPACE;
    if (!out || !out->accept_depth || !out->emitted) return MDSD_E_NULL;
    int32_t* counters = nullptr;
    const int rc = mdsd::static_tree_counters(&counters);
    if (rc != MDSD_OK) return rc;
    return mdsd::verify_entry(mdsd::kSpecHub, pb, tokens, u, out, false, counters, stream);
}

int rrs_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
               void* ws, size_t ws_bytes, void* stream)
{
    return mdsd::verify_with_workspace(mdsd::kRRS, pb, tokens, u, out, ws, ws_bytes, stream);
}

int rrsw_verify(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                void* ws, size_t ws_bytes, void* stream)
{
    return mdsd::verify_with_workspace(mdsd::kRRSw, pb, tokens, u, out, ws, ws_bytes, stream);
}

int spechub_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                        void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kSpecHub, pb, tokens, u, out, true, nullptr, stream);
}

int rrs_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                    void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kRRS, pb, tokens, u, out, true, nullptr, stream);
}

int rrsw_verify_path(const mdsd_problem* pb, const int32_t* tokens, const float* u, const mdsd_result* out,
                     void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    return mdsd::verify_entry(mdsd::kRRSw, pb, tokens, u, out, true, nullptr, stream);
}

int mdsd_tree_walk(const mdsd_problem* pb, const int32_t* outcome, const int32_t* token,
                   int32_t* accept_depth, int32_t* emitted, void* stream)
{
    if (!pb) return MDSD_E_NULL;
    if (pb->B == 0) return MDSD_OK;
    if (!outcome || !token || !accept_depth || !emitted) return MDSD_E_NULL;
    if (pb->B < 1 || pb->N < 1 || pb->depth < 1) return MDSD_E_SHAPE;
    if (pb->k < 1 || pb->k > MDSD_MAX_K) return MDSD_E_K;
    (void)hipGetLastError();
    return mdsd::walk(pb, outcome, token, accept_depth, emitted, (hipStream_t)stream);
}

int mdsd_philox_uniform(uint64_t seed, uint32_t stream_id, int64_t rows, int32_t slots, float* out,
                        uint32_t* words, void* stream)
{
    if (rows < 0 || slots < 1) return MDSD_E_SHAPE;
    if (rows == 0) return MDSD_OK;
    if (!out && !words) return MDSD_E_NULL;
    const int64_t n = rows * ((slots + 3) >> 2);
    const int threads = 256;
    const int64_t blocks = (n + threads - 1) / threads;
    if (blocks > INT_MAX) return MDSD_E_SHAPE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(mdsd::philox_uniform_kernel, dim3((unsigned)blocks), dim3(threads), 0,
                       (hipStream_t)stream, (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, rows,
                       (int)slots, out, words);
    return hipGetLastError() == hipSuccess ? MDSD_OK : MDSD_E_LAUNCH;
}

const char* mdsd_strerror(int code)
{
    switch (code) {
    case MDSD_OK: return "ok";
    case MDSD_E_NULL: return "a required pointer is NULL";
    case MDSD_E_SHAPE: return "bad shape: B, N, V, ld, depth or tree/N mismatch";
    case MDSD_E_K: return "k out of range (SpecHub needs k == 2)";
    case MDSD_E_TEMP: return "temperature must be > 0";
    case MDSD_E_DTYPE: return "unknown dtype or kind";
    case MDSD_E_ALIGN: return "pointer not element-aligned, or target/draft rows differ modulo 16 bytes";
    case MDSD_E_WORKSPACE: return "workspace smaller than mdsd_workspace_bytes()";
    case MDSD_E_LAUNCH: return "HIP launch failed";
    case MDSD_E_UNSUPPORTED: return "output not available from this entry point";
    default: return "unknown status";
    }
}

int mdsd_version(void) { return 104; }

}  // extern "C"
