"""GPU parity: the HIP library against the fp64 oracle, through the C ABI, on
the same seeded rows, tokens and Philox uniforms (see tests/parity.py for the
bar).  Sizes span several slabs and ragged tails; the large configurations run
at full size on the GPU and are compared on sampled sequences."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_05289_amd import binding as B
from paper_2411_05289_amd import workloads as W
from parity import DRAFT, METHODS, VERIFY, VERIFY_PATH, check_case, oracle_kwargs, tokens_per_step, uniforms, _np

pytestmark = pytest.mark.gpu
DEV = "cuda"
ALL = ["spechub", "rrs", "rrsw"]


def note(request, out):
    print("\n[parity] %s: %s" % (request.node.name, out), flush=True)


# ----------------------------------------------------------------- Philox
def test_philox_words_match_oracle():
    for seed, stream, rows, slots in ((0, 1, 1000, 3), (2 ** 40 + 5, 7, 257, 9), (1, 0, 5, 1)):
        u, w = B.philox_uniform(seed, stream, rows, slots, device=DEV, want_words=True)
        uo, wo = oracle.philox_uniform(seed, stream, rows, slots, want_words=True)
        assert (_np(w).view(np.uint32) == wo).all()
        assert (_np(u) == uo).all()


# ----------------------------------------------------------------- the five configurations
@pytest.mark.parametrize("method", ALL)
def test_config1_tiny_probs(method, request):
    wl = W.config(1, device=DEV)
    note(request, check_case(method, wl, seed=0))


@pytest.mark.parametrize("method", ALL)
def test_config2_fp32_logits(method, request):
    wl = W.config(2, device=DEV)
    note(request, check_case(method, wl, seed=0))
    # more trees of the same recipe, so that every branch of the method is visited
    wl = W.config(2, device=DEV, B=24, seed=3)
    note(request, check_case(method, wl, seed=3, full_outputs=False))


@pytest.mark.parametrize("method", ALL)
def test_config3_bf16_headline(method, request):
    wl = W.config(3, device=DEV)
    note(request, check_case(method, wl, seed=0))


@pytest.mark.parametrize("method", ALL)
def test_config4_large_vocab_sampled(method, request):
    wl = W.config(4, device=DEV)
    seqs = [0, 1, 37, 100, 255]
    note(request, check_case(method, wl, seed=0, seqs=seqs))


@pytest.mark.parametrize("method", ["rrs", "rrsw"])
def test_config5_four_drafts_sampled(method, request):
    wl = W.config(5, device=DEV)                     # k = 4, depth 3; every 4th sequence near-uniform
    note(request, check_case(method, wl, seed=0, seqs=[0, 3, 7, 64, 127]))


def test_config5_spechub_sampled(request):
    wl = W.config(5, device=DEV, k=2, depth=4)
    note(request, check_case("spechub", wl, seed=0, seqs=[0, 3, 7, 64, 127]))


# ----------------------------------------------------------------- ragged and misaligned rows
@pytest.mark.parametrize("method", ALL)
@pytest.mark.parametrize("V,dtype", [(2, torch.float32), (7, torch.float32), (50, torch.float32),
                                     (1003, torch.float32), (5, torch.bfloat16), (777, torch.bfloat16),
                                     (4099, torch.bfloat16)])
def test_ragged_vocabularies(method, V, dtype, request):
    """ld = V: row starts fall on every 16-byte phase, tails are partial chunks."""
    k, depth = 2, 3
    if method == "rrsw" and V < 3:
        pytest.skip("cannot draw two distinct tokens plus a residual from V = 2")
    N = W.tree_nodes(k, depth)
    t, d = W.llm_like_logits(16, N, V, logit_std=2.0, draft_noise_std=1.0, dtype=dtype, seed=V, device=DEV)
    wl = W.Workload("ragged_V%d" % V, 16, N, V, k, depth, "fp32" if dtype == torch.float32 else "bf16",
                    "logits", 0.9, 1.1, t, d)
    note(request, check_case(method, wl, seed=V))


@pytest.mark.parametrize("method", ALL)
def test_padded_rows_and_offset_base(method, request):
    """ld > V and a base pointer that is not 16-byte aligned."""
    k, depth, V, ld, Bn = 2, 3, 300, 312, 8
    N = W.tree_nodes(k, depth)
    t, d = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.5, dtype=torch.bfloat16, seed=9, device=DEV)
    big_t = torch.full((Bn * N * ld + 3,), 77.0, dtype=torch.bfloat16, device=DEV)
    big_d = torch.full((Bn * N * ld + 3,), -77.0, dtype=torch.bfloat16, device=DEV)
    tv = big_t[3:].view(Bn, N, ld)[:, :, :V]
    dv = big_d[3:].view(Bn, N, ld)[:, :, :V]
    tv.copy_(t)
    dv.copy_(d)
    wl = W.Workload("padded", Bn, N, V, k, depth, "bf16", "logits", 1.0, 1.0, tv, dv)
    # the oracle reads contiguous copies of the same values
    pb = B.Problem.from_workload(wl)
    u_v = B.philox_uniform(4, 2, Bn * N, k + 1, device=DEV).view(Bn, N, k + 1)
    u_d = B.philox_uniform(4, 1, Bn * N, k, device=DEV).view(Bn, N, k)
    from parity import DRAFT, VERIFY
    g_d = DRAFT[method](pb, u_d)
    wl_c = W.Workload("padded_c", Bn, N, V, k, depth, "bf16", "logits", 1.0, 1.0, t.contiguous(), d.contiguous())
    pb_c = B.Problem.from_workload(wl_c)
    g_dc = DRAFT[method](pb_c, u_d)
    assert (g_d["tokens"] == g_dc["tokens"]).all()
    a = VERIFY[method](pb, g_d["tokens"], u_v, resid_mass=True)
    c = VERIFY[method](pb_c, g_d["tokens"], u_v, resid_mass=True)
    for key in ("outcome", "token", "accept_depth", "emitted"):
        assert (a[key] == c[key]).all(), key
    # a different 16-byte phase regroups the partial sums: same value up to rounding
    assert torch.allclose(a["resid_mass"], c["resid_mass"], rtol=1e-5, atol=5e-7)
    note(request, check_case(method, wl_c, seed=4))


@pytest.mark.parametrize("method", ALL)
def test_random_shapes_strides_and_temperatures(method, request):
    """Seeded random cases: vocabulary size (ragged tails, one slab to many), k, depth, storage
    type, logits or probabilities, both temperatures, row padding and a base address that is
    not 16-byte aligned, straight against the oracle."""
    rng = np.random.default_rng({"spechub": 1, "rrs": 2, "rrsw": 3}[method])
    totals = {}
    for case in range(24):
        V = int(rng.choice([rng.integers(2, 40), rng.integers(40, 700), rng.integers(700, 9000)]))
        k = 2 if method == "spechub" else int(rng.integers(1, 6))
        depth = int(rng.integers(1, 4 if k <= 3 else 3))
        N = W.tree_nodes(k, depth)
        Bn = int(rng.integers(1, 7))
        bf16 = bool(rng.integers(0, 2))
        logits = bool(rng.integers(0, 4))             # one case in four: probabilities
        dtype = torch.bfloat16 if bf16 and logits else torch.float32
        pad, off = int(rng.integers(0, 18)), int(rng.integers(0, 8))
        if logits:
            t, d = W.llm_like_logits(Bn, N, V, logit_std=float(rng.uniform(0.5, 4.0)),
                                     draft_noise_std=float(rng.uniform(0.2, 2.5)), dtype=dtype,
                                     seed=100 + case, device=DEV)
            temps = (float(rng.uniform(0.3, 2.0)), float(rng.uniform(0.3, 2.0)))
        else:
            t, d = W.dirichlet_rows(Bn, N, V, seed=100 + case, device=DEV)
            temps = (1.0, 1.0)
        ld = V + pad
        big_t = torch.zeros((Bn * N * ld + off,), dtype=dtype, device=DEV)
        big_d = torch.zeros((Bn * N * ld + off,), dtype=dtype, device=DEV)
        tv = big_t[off:].view(Bn, N, ld)[:, :, :V]
        dv = big_d[off:].view(Bn, N, ld)[:, :, :V]
        tv.copy_(t)
        dv.copy_(d)
        wl = W.Workload("random%d" % case, Bn, N, V, k, depth, "bf16" if dtype == torch.bfloat16 else "fp32",
                        "logits" if logits else "probs", temps[0], temps[1], tv, dv)
        out = check_case(method, wl, seed=200 + case, full_outputs=V <= 3000)
        for key, val in out.items():
            if isinstance(val, (int, np.integer)):
                totals[key] = totals.get(key, 0) + int(val)
    note(request, totals)


# ----------------------------------------------------------------- temperatures
@pytest.mark.parametrize("method", ALL)
@pytest.mark.parametrize("T", [0.3, 0.7, 2.0])
def test_temperatures(method, T, request):
    wl = W.config(2, device=DEV, B=8, V=4000, seed=11)
    wl.temp_target = T
    wl.temp_draft = T
    note(request, check_case(method, wl, seed=int(T * 10)))


@pytest.mark.parametrize("V,Bn", [(4096, 6), (70016, 2)], ids=["in_registers", "streamed"])
def test_rows_with_isolated_peaks(V, Bn, request):
    """bf16 rows whose largest logits sit far above the rest at even and at odd token indices
    (a shift taken from part of the row would overflow or underflow the weights), and
    rows holding -inf (masked tokens): the softmax must still be the exact one.  Once with rows
    that stay in registers, once with rows long enough to be streamed."""
    wl = W.config(3, device=DEV, B=Bn, V=V, seed=31)
    g = torch.Generator(device="cpu").manual_seed(31)
    # the target's peaks leave every other weight at zero in fp32; the draft's stay moderate, so
    # that its mass outside the hub does not vanish in fp32 while it is positive in fp64
    for rows, peak in ((wl.target, 300.0), (wl.draft, 40.0)):
        Bn, N, V = rows.shape
        for b in range(Bn):
            for n in range(N):
                kind = (b * N + n) % 4
                if kind == 0:      # one dominant token at an even index
                    rows[b, n, 2 * int(torch.randint(0, V // 2, (1,), generator=g))] = peak
                elif kind == 1:    # at an odd index
                    rows[b, n, 2 * int(torch.randint(0, V // 2, (1,), generator=g)) + 1] = peak
                elif kind == 2:    # a block of masked tokens
                    lo = int(torch.randint(0, V - 600, (1,), generator=g))
                    rows[b, n, lo:lo + 555] = float("-inf")
                # kind 3: left as generated
    note(request, check_case("spechub", wl, seed=31))


@pytest.mark.parametrize("method", ALL)
def test_largest_supported_vocabulary(method, request):
    """bf16 rows of 2048 slabs minus one chunk, the longest the per-slab sums in LDS allow
    (one more chunk is refused with MDSD_E_SHAPE)."""
    V = 2048 * 64 * 8 - 8
    wl = W.config(3, device=DEV, B=2, V=V, depth=2, seed=41)
    note(request, check_case(method, wl, seed=41, full_outputs=False))
    too_long = W.config(3, device=DEV, B=1, V=V + 8, depth=2, seed=41)
    with pytest.raises(B.MdsdError) as err:
        B.spechub_draft(B.Problem.from_workload(too_long),
                        torch.zeros((1, too_long.N, 2), dtype=torch.float32, device=DEV))
    assert err.value.code == -2


@pytest.mark.parametrize("method", ALL)
@pytest.mark.parametrize("V,K", [(32000, 5), (32000, 20), (32000, 50), (4096, 5), (4096, 50), (70016, 20)])
def test_rows_masked_down_to_a_few_tokens(method, V, K, request):
    """bf16 rows with every logit at -inf except K tokens (what top-k filtering leaves), at even
    and odd indices: most 32-bit words of such a row hold no finite upper half, so a softmax
    shift estimated from whole words finds nothing to refer to in most waves.  Normalisers, leaf
    draws and the draft records must still be those of the exact softmax (rows in registers at
    V = 4096 and 32000, streamed at 70016)."""
    k, depth, Bn = 2, 3, 6
    N = W.tree_nodes(k, depth)
    t, d = W.topk_masked_logits(Bn, N, V, K, seed=V + K, device=DEV)
    wl = W.Workload("topk_V%d_K%d" % (V, K), Bn, N, V, k, depth, "bf16", "logits", 1.0, 1.0, t, d)
    note(request, check_case(method, wl, seed=K))


# ----------------------------------------------------------------- every dispatched kernel variant
# (dtype, kind, V, row offset in elements): between them these reach every instantiation the
# launchers can choose: rows in registers with 4, 8 or 16 chunks per lane, with and without masked
# first / last chunks, fp32 and bf16, logits and probabilities, the streamed forms, and the
# builds for short rows with one, two or four wavefronts per node (rows of up to 256, 512 and
# 1024 16-byte chunks).
_VARIANTS = [
    ("fp32", "logits", 1000, 0),     # one wavefront per node: fp32 logits, four chunks per lane
    ("fp32", "logits", 301, 1),      # ... masked
    ("bf16", "logits", 2040, 0),     # ... bf16 logits, the longest aligned row of that build
    ("bf16", "logits", 777, 3),      # ... masked
    ("fp32", "probs", 513, 0),       # ... fp32 probabilities
    ("bf16", "probs", 2042, 0),      # two wavefronts per node: the shortest row, bf16 probabilities
    ("fp32", "logits", 1023, 0),     # ... fp32 logits, masked
    ("bf16", "logits", 3000, 0),     # ... bf16 logits
    ("fp32", "probs", 2044, 0),      # ... the longest aligned fp32 row
    ("bf16", "logits", 4090, 0),     # four wavefronts per node: the shortest row
    ("bf16", "logits", 5001, 3),     # ... masked
    ("bf16", "probs", 8184, 0),      # ... the longest aligned row, bf16 probabilities
    ("fp32", "logits", 3001, 0),     # ... fp32 logits
    ("fp32", "probs", 4000, 0),      # ... fp32 probabilities
    ("bf16", "probs", 8200, 0),      # the 512-thread build again: bf16 probabilities, registers
    ("fp32", "logits", 4100, 0),     # ... fp32 logits
    ("fp32", "logits", 12000, 0),    # fp32, 8 chunks per lane, no masking
    ("fp32", "logits", 12001, 0),    # ... masked (ld = V is odd: rows start on every 4-byte phase)
    ("fp32", "logits", 30000, 1),    # fp32, 16 chunks per lane, masked (base one element off)
    ("fp32", "logits", 40000, 0),    # fp32, streamed
    ("bf16", "logits", 20001, 0),    # bf16, 8 chunks per lane, masked
    ("bf16", "logits", 50304, 0),    # bf16, 16 chunks per lane, no masking
    ("bf16", "logits", 50257, 0),    # ... masked
    ("bf16", "logits", 65520, 0),    # the longest row that stays in registers
    ("bf16", "probs", 1000, 0),      # bf16 probabilities: one wavefront per node
    ("bf16", "probs", 4099, 3),      # ... masked
    ("bf16", "probs", 40000, 0),     # ... 16 chunks per lane / streamed
    ("bf16", "probs", 70016, 0),     # ... streamed
    ("fp32", "probs", 20000, 0),     # fp32 probabilities, 16 chunks per lane
    ("fp32", "probs", 40000, 0),     # ... streamed
]


@pytest.mark.parametrize("method", ALL)
@pytest.mark.parametrize("dtype,kind,V,off", _VARIANTS, ids=["%s_%s_V%d_off%d" % v for v in _VARIANTS])
def test_dispatched_variants(method, dtype, kind, V, off, request):
    k, depth, Bn = (2, 3, 3) if method == "spechub" else (3, 2, 4)
    N = W.tree_nodes(k, depth)
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    if kind == "logits":
        t, d = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.5, dtype=td, seed=V, device=DEV)
        temps = (0.9, 1.2)
    else:
        # probabilities rounded to the storage type: used as given, not renormalised
        lt, ld = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.5, dtype=torch.float32, seed=V, device=DEV)
        t, d = torch.softmax(lt.double(), -1).to(td), torch.softmax(ld.double(), -1).to(td)
        temps = (1.0, 1.0)
    if off:
        big_t = torch.zeros((Bn * N * V + off,), dtype=td, device=DEV)
        big_d = torch.zeros((Bn * N * V + off,), dtype=td, device=DEV)
        tv, dv = big_t[off:].view(Bn, N, V), big_d[off:].view(Bn, N, V)
        tv.copy_(t)
        dv.copy_(d)
        t, d = tv, dv
    wl = W.Workload("variant_%s_%s_V%d" % (dtype, kind, V), Bn, N, V, k, depth, dtype, kind, temps[0], temps[1], t, d)
    note(request, check_case(method, wl, seed=V % 1000, full_outputs=V <= 20001))


# ----------------------------------------------------------------- large batches
_LARGE = [
    ("bf16", 32000, 0),     # the headline row: 256 threads per node, sixteen chunks per lane
    ("bf16", 20001, 0),     # ... masked (RRS / RRSw: the generic kernel)
    ("fp32", 12000, 0),     # fp32
    ("fp32", 12001, 1),     # ... masked
]


@pytest.mark.parametrize("method", ALL)
@pytest.mark.parametrize("dtype,V,off", _LARGE, ids=["%s_V%d_off%d" % v for v in _LARGE])
def test_batches_of_more_than_2300_nodes(method, dtype, V, off, request):
    """From 2300 tree nodes per batch the verify calls that have the draft call's records run their
    rows of eight chunks per lane on 256-thread kernels; sampled sequences against the oracle."""
    k, depth = (2, 3) if method == "spechub" else (3, 2)
    N = W.tree_nodes(k, depth)
    Bn = 2300 // N + 3
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    t, d = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.5, dtype=td, seed=V + 1, device=DEV)
    if off:
        big_t = torch.zeros((Bn * N * V + off,), dtype=td, device=DEV)
        big_d = torch.zeros((Bn * N * V + off,), dtype=td, device=DEV)
        tv, dv = big_t[off:].view(Bn, N, V), big_d[off:].view(Bn, N, V)
        tv.copy_(t)
        dv.copy_(d)
        t, d = tv, dv
    wl = W.Workload("large_%s_V%d" % (dtype, V), Bn, N, V, k, depth, dtype, "logits", 0.9, 1.1, t, d)
    assert wl.B * wl.N >= 2300
    note(request, check_case(method, wl, seed=V % 1000, seqs=[0, 1, Bn // 2, Bn - 1], full_outputs=False))


# ----------------------------------------------------------------- general topology
@pytest.mark.parametrize("V", [2500, 12000])
@pytest.mark.parametrize("method", ALL)
def test_unbalanced_tree(method, V, request):
    """first_child given: an unbalanced binary tree (left spine deeper than the right)."""
    fc = [1, 3, -1, 5, -1, 7, -1, -1, -1]      # 0->(1,2) 1->(3,4) 3->(5,6) 5->(7,8)
    N, k, depth, Bn = len(fc), 2, 5, 12
    t, d = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.0, dtype=torch.bfloat16, seed=21, device=DEV)
    wl = W.Workload("unbalanced", Bn, N, V, k, depth, "bf16", "logits", 1.0, 1.0, t, d,
                    first_child=torch.tensor(fc, dtype=torch.int32, device=DEV))
    note(request, check_case(method, wl, seed=21))


@pytest.mark.parametrize("method", ["rrs", "rrsw"])
def test_unbalanced_ternary_tree(method, request):
    """first_child given, three children per internal node: 0->(1,2,3) 1->(4,5,6) 3->(7,8,9)
    6->(10,11,12); nodes 2, 4, 5 and the last level are leaves."""
    fc = [1, 4, -1, 7, -1, -1, 10, -1, -1, -1, -1, -1, -1]
    N, k, depth, V, Bn = len(fc), 3, 4, 3000, 10
    t, d = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.0, dtype=torch.bfloat16, seed=22, device=DEV)
    wl = W.Workload("unbalanced3", Bn, N, V, k, depth, "bf16", "logits", 1.0, 1.0, t, d,
                    first_child=torch.tensor(fc, dtype=torch.int32, device=DEV))
    note(request, check_case(method, wl, seed=22))


def test_first_child_entries_that_cannot_be_children_count_as_leaves():
    """An entry that does not point past its own node, or leaves no room for k children, makes
    the node a leaf in the verify kernels and in the walk alike (so the walk always ends)."""
    good = [1, 3, -1, -1, -1]
    for bad in ([1, 3, -1, 0, -1], [1, 3, -1, 3, -1], [1, 3, -1, 4, -1], [1, 3, 1, -1, -1]):
        N, k, depth, V, Bn = 5, 2, 4, 500, 4
        t, d = W.llm_like_logits(Bn, N, V, logit_std=3.0, draft_noise_std=1.0, dtype=torch.float32, seed=23, device=DEV)
        u_v = B.philox_uniform(23, 2, Bn * N, k + 1, device=DEV).view(Bn, N, k + 1)
        u_d = B.philox_uniform(23, 1, Bn * N, k, device=DEV).view(Bn, N, k)
        res = []
        for fc in (good, bad):
            pb = B.Problem(t, d, B.LOGITS, k, depth, first_child=torch.tensor(fc, dtype=torch.int32, device=DEV))
            tok = B.spechub_draft(B.Problem(t, d, B.LOGITS, k, depth,
                                            first_child=torch.tensor(good, dtype=torch.int32, device=DEV)), u_d)["tokens"]
            res.append(B.spechub_verify(pb, tok, u_v, flags=True, walk=True))
            torch.cuda.synchronize()
        for key in ("outcome", "token", "accept_depth", "emitted"):
            assert torch.equal(res[0][key], res[1][key]), (bad, key)


@pytest.mark.parametrize("V", [600, 4000, 9000], ids=["one_wave_per_node", "two_waves_per_node", "eight_waves_per_node"])
@pytest.mark.parametrize("method", ALL)
def test_trees_of_more_than_64_nodes(method, V, request):
    """127-node trees: the walk (as a launch of its own and inside the verify kernel) goes node
    by node from memory instead of holding the tree in one wavefront's lanes."""
    wl = W.config(3, device=DEV, B=5, V=V, depth=7, seed=61)
    assert wl.N == 127
    note(request, check_case(method, wl, seed=61, full_outputs=False))


def test_workspace_is_checked():
    wl = W.config(3, device=DEV, B=4, V=600, depth=3, seed=62)
    pb = B.Problem.from_workload(wl)
    assert B.workspace_bytes(pb) == 4 * wl.B
    u_d, u_v = uniforms(wl, 62)
    tokens = B.spechub_draft(pb, u_d)["tokens"]
    small = torch.zeros((wl.B - 1,), dtype=torch.int32, device=DEV)
    with pytest.raises(B.MdsdError) as err:
        B.spechub_verify(pb, tokens, u_v, workspace=small)
    assert err.value.code == -7
    # without the walk outputs the workspace is left alone
    ws = B.alloc_workspace(pb)
    a = B.spechub_verify(pb, tokens, u_v, workspace=ws, walk=False)
    b = B.spechub_verify(pb, tokens, u_v, walk=False)
    assert torch.equal(a["outcome"], b["outcome"]) and not ws.any()


# ----------------------------------------------------------------- degenerate and invalid inputs
def _tiny_probs(p_rows, q_rows, k=2, depth=2):
    p = torch.tensor(p_rows, dtype=torch.float32, device=DEV).view(1, -1, len(p_rows[0]))
    q = torch.tensor(q_rows, dtype=torch.float32, device=DEV).view(1, -1, len(q_rows[0]))
    return B.Problem(p, q, B.PROBS, k, depth)


def test_point_mass_draft_is_single_draft_case():
    p = [[0.2, 0.5, 0.1, 0.2]] * 3
    q = [[0.0, 1.0, 0.0, 0.0]] * 3
    pb = _tiny_probs(p, q)
    u_d = torch.tensor([[[0.4, 0.4]] * 3], dtype=torch.float32, device=DEV)
    g = B.spechub_draft(pb, u_d)
    assert _np(g["tokens"])[0].tolist() == [-1, 1, 1]
    assert _np(g["flags"])[0, 0] & B.FLAG_DEGENERATE_HUB
    for r0, want_oc, want_tok in ((0.49, 0, 1), (0.51, -1, None)):
        u = torch.tensor([[[r0, 0.5, 0.55]] * 3], dtype=torch.float32, device=DEV)
        v = B.spechub_verify(pb, g["tokens"], u, resid_mass=True)
        assert _np(v["outcome"])[0, 0] == want_oc
        o = oracle.spechub_verify(np.array(p[0]), np.array(q[0]), 1, 1, 1, r0, 0.5, float(np.float32(0.55)))
        assert _np(v["token"])[0, 0] == o["token"]
        assert _np(v["flags"])[0, 0] & B.FLAG_DEGENERATE_HUB
        if want_tok is not None:
            assert _np(v["token"])[0, 0] == want_tok


def test_invalid_tokens_and_pairs_are_flagged():
    p = [[0.2, 0.5, 0.3]] * 3
    q = [[0.3, 0.4, 0.3]] * 3
    pb = _tiny_probs(p, q)
    u = torch.full((1, 3, 3), 0.5, dtype=torch.float32, device=DEV)
    for toks, code, flag in (([-1, 0, 2], B.BAD_PAIR, B.FLAG_BAD_PAIR), ([-1, 7, 1], B.BAD_TOKEN, B.FLAG_BAD_TOKEN),
                             ([-1, 1, 1], B.BAD_PAIR, B.FLAG_BAD_PAIR)):
        t = torch.tensor([toks], dtype=torch.int32, device=DEV)
        v = B.spechub_verify(pb, t, u)
        assert _np(v["outcome"])[0, 0] == code and _np(v["flags"])[0, 0] & flag
        assert _np(v["accept_depth"])[0] == 0
    t = torch.tensor([[-1, 0, -5]], dtype=torch.int32, device=DEV)
    for fn in (B.rrs_verify, B.rrsw_verify):
        v = fn(pb, t, u)
        assert _np(v["outcome"])[0, 0] == B.BAD_TOKEN


@pytest.mark.parametrize("V,dtype,kind", [(4096, torch.bfloat16, "resident"), (70016, torch.bfloat16, "streamed")])
def test_unusable_draft_record_is_flagged(V, dtype, kind):
    """A draft record whose hub lies outside the vocabulary makes that node MDSD_BAD_PAIR (never a
    wild read); every other node is verified as with the good records.  Invalid draft tokens
    are flagged on the paths that take the records, too."""
    wl = W.config(3, device=DEV, B=3, V=V, depth=3, seed=51)
    pb = B.Problem.from_workload(wl).with_draft_stats()
    rows = wl.B * wl.N
    u_d = B.philox_uniform(51, 1, rows, 2, device=DEV).view(wl.B, wl.N, 2)
    u_v = B.philox_uniform(51, 2, rows, 3, device=DEV).view(wl.B, wl.N, 3)
    tokens = B.spechub_draft(pb, u_d)["tokens"]
    good = B.spechub_verify(pb, tokens, u_v)
    hubs = pb.draft_stats.view(torch.int32)[..., 2]
    hubs[1, 0] = V + 5
    hubs[2, 1] = -3
    bad = B.spechub_verify(pb, tokens, u_v)
    oc_g, oc_b, fl_b = _np(good["outcome"]), _np(bad["outcome"]), _np(bad["flags"])
    assert oc_b[1, 0] == B.BAD_PAIR and fl_b[1, 0] & B.FLAG_BAD_PAIR
    assert oc_b[2, 1] == B.BAD_PAIR and fl_b[2, 1] & B.FLAG_BAD_PAIR
    keep = np.ones_like(oc_g, dtype=bool)
    keep[1, 0] = keep[2, 1] = False
    assert (oc_b[keep] == oc_g[keep]).all() and (_np(bad["token"])[keep] == _np(good["token"])[keep]).all()
    # invalid tokens with records at hand (SpecHub and RRS take their own paths for them)
    pb2 = B.Problem.from_workload(wl).with_draft_stats()
    t2 = B.spechub_draft(pb2, u_d)["tokens"].clone()
    t2[0, 1] = V + 1
    v = B.spechub_verify(pb2, t2, u_v)
    assert _np(v["outcome"])[0, 0] == B.BAD_TOKEN
    pb3 = B.Problem.from_workload(wl).with_draft_stats()
    t3 = B.rrs_draft(pb3, u_d)["tokens"].clone()
    t3[0, 2] = -9
    v = B.rrs_verify(pb3, t3, u_v)
    assert _np(v["outcome"])[0, 0] == B.BAD_TOKEN and _np(v["flags"])[0, 0] & B.FLAG_BAD_TOKEN
    assert (_np(v["outcome"])[1:] >= -1).all()


@pytest.mark.parametrize("method", ["rrs", "rrsw"])
def test_repeated_draft_tokens(method):
    """Duplicates handed to the verifiers (RRS draws them; RRSw must treat the second as massless)."""
    rng = np.random.default_rng(5)
    V, k, depth = 40, 3, 2
    N = W.tree_nodes(k, depth)
    p = rng.dirichlet(np.full(V, 0.4), size=(6, N)).astype(np.float32)
    q = rng.dirichlet(np.full(V, 0.4), size=(6, N)).astype(np.float32)
    toks = np.full((6, N), -1, np.int32)
    for b in range(6):
        x = int(np.argmax(q[b, 0] - p[b, 0]))     # surely over-sampled: likely rejected
        toks[b, 1:] = [x, x, (x + 1) % V]
    u = np.full((6, N, k + 1), 0.97, np.float32)
    pb = B.Problem(torch.from_numpy(p).to(DEV), torch.from_numpy(q).to(DEV), B.PROBS, k, depth)
    g = {"rrs": B.rrs_verify, "rrsw": B.rrsw_verify}[method](pb, torch.from_numpy(toks).to(DEV),
                                                              torch.from_numpy(u).to(DEV), resid_mass=True)
    o = oracle.batch_verify(METHODS[method], p, q, toks, u, dtype=oracle.FP32, kind=oracle.PROBS, k=k, depth=depth)
    near = o["margin"] < 1e-6
    assert ((_np(g["outcome"]) == o["outcome"]) | near).all()
    assert ((_np(g["token"]) == o["token"]) | near).all()


@pytest.mark.parametrize("method", ALL)
def test_empty_batch(method):
    """No trees: every call succeeds and returns empty outputs."""
    k, depth, V = 2, 3, 64
    N = W.tree_nodes(k, depth)
    rows = torch.empty((0, N, V), dtype=torch.bfloat16, device=DEV)
    pb = B.Problem(rows, rows.clone(), B.LOGITS, k, depth).with_draft_stats()
    d = DRAFT[method](pb, torch.empty((0, N, k), dtype=torch.float32, device=DEV))
    assert d["tokens"].shape == (0, N)
    u_v = torch.empty((0, N, k + 1), dtype=torch.float32, device=DEV)
    for call in (VERIFY[method], VERIFY_PATH[method]):
        v = call(pb, d["tokens"], u_v, flags=True, walk=True)
        assert v["outcome"].shape == (0, N) and v["accept_depth"].shape == (0,) and v["emitted"].shape == (0, depth)
    assert B.philox_uniform(1, 0, 0, 4, device=DEV).numel() == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("V,Bn", [(4104, 6), (40000, 3)], ids=["in_registers", "streamed"])
def test_draft_mass_below_the_fp32_range_is_flagged(V, Bn):
    """Rows so peaked (temperature 0.03) that, once the dominant token is removed, what is left is
    below 2^-126 of it: the kernels' fp32 weights then hold no mass.  rrsw_draft repeats the token
    and flags the node, spechub_draft gives the pair (a, a) and flags it, both verifiers still
    return a valid outcome; where the rest is inside the range the tokens are the oracle's (on
    streamed rows the one-sweep statistics must notice that they cannot hold such a row)."""
    wl = W.config(2, device=DEV, B=Bn, V=V, k=2, depth=3, seed=300)
    wl.temp_target, wl.temp_draft = 0.02, 0.03
    pb = B.Problem.from_workload(wl)
    u_d, u_v = uniforms(wl, 300)
    rows = W.rows_as_numpy(wl.draft).astype(np.float64)
    w = np.exp((rows - rows.max(axis=-1, keepdims=True)) / np.float64(np.float32(wl.temp_draft)))
    internal = np.arange(wl.N) < W.internal_nodes(wl.k, wl.depth)
    seen = {"gone": 0, "kept": 0}
    for method, flag in (("rrsw", B.FLAG_Q_EXHAUSTED), ("spechub", B.FLAG_DEGENERATE_HUB)):
        g = DRAFT[method](pb, u_d)
        o = oracle.batch_draft(METHODS[method], W.rows_as_numpy(wl.draft), _np(u_d), temp_draft=wl.temp_draft,
                               nthreads=8, **oracle_kwargs(wl))
        g_tok, g_flags = _np(g["tokens"]), _np(g["flags"])
        for b in range(wl.B):
            for n in np.nonzero(internal)[0]:
                c0 = wl.k * n + 1
                first = o["tokens"][b, c0] if method == "rrsw" else int(np.argmax(w[b, n]))
                rest = np.delete(w[b, n], first).sum()         # relative to the largest weight, 1
                if method == "rrsw" and w[b, n, first] < 1.0:
                    continue                                   # the dominant token was not drawn first
                if np.delete(w[b, n], first).max() < 2.0 ** -150:   # every other weight rounds to 0
                    seen["gone"] += 1
                    assert g_flags[b, n] & flag, (method, b, n, rest)
                    assert g_tok[b, c0] == g_tok[b, c0 + 1] == first, (method, b, n)
                elif rest > 1e-30 and o["margin"][b, n] > 1e-6:
                    seen["kept"] += 1
                    assert (g_tok[b, c0:c0 + 2] == o["tokens"][b, c0:c0 + 2]).all(), (method, b, n)
                    assert g_flags[b, n] == 0
        v = VERIFY[method](pb, g["tokens"], u_v, flags=True, walk=True)
        assert (_np(v["outcome"]) >= -1).all() and (_np(v["token"]) >= 0).all()
    assert seen["gone"] > 0 and seen["kept"] > 0, seen


# ----------------------------------------------------------------- determinism
def test_bitwise_reproducible():
    wl = W.config(3, device=DEV, B=8)
    pb = B.Problem.from_workload(wl)
    u_d = B.philox_uniform(3, 1, wl.B * wl.N, 2, device=DEV).view(wl.B, wl.N, 2)
    u_v = B.philox_uniform(3, 2, wl.B * wl.N, 3, device=DEV).view(wl.B, wl.N, 3)
    d1, d2 = B.spechub_draft(pb, u_d), B.spechub_draft(pb, u_d)
    assert (d1["tokens"] == d2["tokens"]).all()
    v1 = B.spechub_verify(pb, d1["tokens"], u_v, resid_mass=True)
    v2 = B.spechub_verify(pb, d1["tokens"], u_v, resid_mass=True)
    for key in v1:
        assert torch.equal(v1[key], v2[key]), key


# ----------------------------------------------------------------- the marshalled step bench.py times
@pytest.mark.parametrize("method", ALL)
def test_step_plan_gives_what_the_separate_calls_give(method):
    """StepPlan.run() (the launches bench.py times) with the walk in the verify kernel, as a launch
    of its own and by the batch-size rule, run twice each on one plan, against draft, verify and
    walk called one by one through the allocating binding."""
    wl = W.config(3, device=DEV, B=12, V=9000, seed=11)
    pb = B.Problem.from_workload(wl).with_draft_stats()   # the plan hands the draft call's records to verify
    u_d, u_v = uniforms(wl, 5)
    want_d = DRAFT[method](pb, u_d)
    want = VERIFY[method](pb, want_d["tokens"], u_v, flags=True, walk=True)
    for placement in (True, False, None):
        plan = B.StepPlan(method, pb, u_d, u_v, walk_in_verify=placement)
        assert plan.walk_in_verify == (True if placement is None else placement)   # 12 * 31 nodes: a small batch
        for rep in range(2):
            for t in plan.out.values():
                if t is not None:
                    t.fill_(-9)
            out = plan.run()
            torch.cuda.synchronize()
            assert torch.equal(plan.tokens, want_d["tokens"]), (placement, rep)
            for key in ("outcome", "token", "flags", "accept_depth", "emitted"):
                assert torch.equal(out[key], want[key]), (placement, rep, key)
    big = B.Problem.from_workload(W.config(3, device=DEV, B=160, V=1000, seed=1))
    u_d, u_v = uniforms(W.config(3, device=DEV, B=160, V=1000, seed=1), 5)
    assert B.StepPlan(method, big, u_d, u_v).walk_in_verify is False   # 160 * 31 nodes: beyond the rule's 3000


@pytest.mark.parametrize("shape", ["headline", "small_trees", "long_rows"])
def test_walk_inside_the_verify_kernel_over_many_launches(shape):
    """The arrival counters hand outcomes from workgroup to workgroup inside one launch; a mistake
    in that hand-over would show now and then, not every time.  2000 launches back to back on
    rotating inputs, each compared on the device with what the walk as a launch of its own gave."""
    if shape == "headline":
        wls = [W.config(3, device=DEV, seed=s, B=32) for s in range(3)]
    elif shape == "small_trees":
        wls = [W.toy_pairs(0.25, 0.7, 200, repeats=4, seed=s, device=DEV) for s in range(3)]
    else:
        wls = [W.config(5, device=DEV, seed=s, B=8, k=2, depth=4) for s in range(2)]
    plans, want = [], []
    for i, wl in enumerate(wls):
        pb = B.Problem.from_workload(wl)
        u_d, u_v = uniforms(wl, i)
        ref = B.StepPlan("spechub", pb, u_d, u_v, walk_in_verify=False).run()
        torch.cuda.synchronize()
        want.append({key: ref[key].clone() for key in ("accept_depth", "emitted", "outcome", "token")})
        plans.append(B.StepPlan("spechub", pb, u_d, u_v, walk_in_verify=True))
    bad = torch.zeros((), dtype=torch.int64, device=DEV)
    for i in range(2000):
        pl, w = plans[i % len(plans)], want[i % len(plans)]
        pl.out["accept_depth"].fill_(-7)
        pl.out["emitted"].fill_(-7)
        out = pl.run()
        for key in w:
            bad += (out[key] != w[key]).sum()
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    assert not any(bool(pl.workspace.any()) for pl in plans)   # every counter back at zero


# ----------------------------------------------------------------- Monte-Carlo tokens/step
@pytest.mark.parametrize("method", ALL)
def test_tokens_per_step_within_3_sigma(method, request):
    """Batch efficiency (tokens per step = accept depth + 1, Sec. 5.3) of the GPU against the
    oracle's on the same inputs, and both against each other's Monte-Carlo spread."""
    wl = W.config(3, device=DEV, B=96, V=8000, seed=5)
    pb = B.Problem.from_workload(wl)
    from parity import DRAFT, VERIFY, uniforms, oracle_kwargs
    from paper_2411_05289_amd.workloads import rows_as_numpy
    u_d, u_v = uniforms(wl, 77)
    g_d = DRAFT[method](pb, u_d)
    g_v = VERIFY[method](pb, g_d["tokens"], u_v)
    ok = oracle_kwargs(wl)
    # an independent stream of uniforms for the oracle: a statistical, not bitwise, comparison
    u_d2 = oracle.philox_uniform(78, 1, wl.B * wl.N, wl.k).reshape(wl.B, wl.N, wl.k)
    u_v2 = oracle.philox_uniform(78, 2, wl.B * wl.N, wl.k + 1).reshape(wl.B, wl.N, wl.k + 1)
    t_np, d_np = rows_as_numpy(wl.target), rows_as_numpy(wl.draft)
    o_d = oracle.batch_draft(METHODS[method], d_np, u_d2, temp_draft=wl.temp_draft, nthreads=8, **ok)
    o_v = oracle.batch_verify(METHODS[method], t_np, d_np, o_d["tokens"], u_v2, temp_target=wl.temp_target,
                              temp_draft=wl.temp_draft, nthreads=8, **ok)
    tg, to = _np(g_v["accept_depth"]) + 1.0, o_v["accept_depth"] + 1.0
    sigma = np.sqrt(tg.var(ddof=1) / tg.size + to.var(ddof=1) / to.size)
    note(request, dict(gpu=tokens_per_step(tg - 1), oracle=tokens_per_step(to - 1), sigma=float(sigma)))
    assert abs(tg.mean() - to.mean()) < 3 * sigma
