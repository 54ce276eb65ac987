"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on Llama-2 / Vicuna logits over CNN DailyMail, OpenWebText
and MT-Bench (Sec. 5.1); none of that exists here, so these generators stand in
for it: vocabulary sizes of those model families, complete k-ary token trees of
the paper's depths (Sec. 5.3), heavy-tailed target rows and a noisy copy as the
draft.  This module only *makes inputs* (rows, tree shapes); it contains none of
the method's arithmetic and is the one module that both the HIP library's tests
and the CPU oracle's tests consume.

Tensors are torch tensors on the requested device; ``rows_as_numpy`` gives the
stored bits to CPU code (float32, or uint16 holding bf16).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


def tree_nodes(k: int, depth: int) -> int:
    """Nodes of a complete k-ary tree with `depth` levels, root included
    (Sec. 5.3: a binary tree of depth d has 2^d - 1 nodes)."""
    return depth if k == 1 else (k ** depth - 1) // (k - 1)


def internal_nodes(k: int, depth: int) -> int:
    return tree_nodes(k, depth - 1) if depth > 1 else 0


@dataclass
class Workload:
    name: str
    B: int
    N: int
    V: int
    k: int
    depth: int
    dtype: str            # "fp32" | "bf16"  (storage of the rows)
    kind: str             # "probs" | "logits"
    temp_target: float
    temp_draft: float
    target: torch.Tensor  # [B, N, V]
    draft: torch.Tensor   # [B, N, V] (leaf rows are never read)
    seed: int = 0
    first_child: Optional[torch.Tensor] = None
    notes: dict = field(default_factory=dict)

    @property
    def n_internal(self) -> int:
        if self.first_child is not None:
            return int((self.first_child >= 0).sum().item())
        return internal_nodes(self.k, self.depth)

    def algorithmic_bytes(self) -> int:
        """Each needed row once: target rows of all nodes, draft rows of internal nodes."""
        es = 4 if self.dtype == "fp32" else 2
        return self.B * self.V * es * (self.N + self.n_internal)


def rows_as_numpy(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _coprime_multiplier(V: int) -> int:
    a = int(V * 0.6180339887) | 1
    while math.gcd(a, V) != 1:
        a += 2
    return a


def llm_like_logits(B, N, V, *, logit_std, draft_noise_std, zipf_s=1.1, dtype=torch.bfloat16,
                    seed=0, device="cpu", chunk_rows=256):
    """Target logits N(0, logit_std^2) minus zipf_s * ln(rank), where rank is a
    per-row pseudo-random permutation of 1..V (an affine map modulo V); draft
    logits = target logits + N(0, draft_noise_std^2).  `logit_std` and
    `draft_noise_std` are floats or per-sequence tensors [B].  Rows are rounded
    to `dtype` before anyone sees them; the draft noise is added to the
    unrounded target."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    target = torch.empty((B, N, V), dtype=dtype, device=dev)
    draft = torch.empty((B, N, V), dtype=dtype, device=dev)
    ls = torch.as_tensor(logit_std, dtype=torch.float32, device=dev).expand(B).contiguous()
    ds = torch.as_tensor(draft_noise_std, dtype=torch.float32, device=dev).expand(B).contiguous()
    A = _coprime_multiplier(V)
    x = torch.arange(V, device=dev, dtype=torch.int64)
    seqs_per_chunk = max(1, chunk_rows // N)
    for b0 in range(0, B, seqs_per_chunk):
        b1 = min(B, b0 + seqs_per_chunk)
        nb = b1 - b0
        g = torch.randn((nb, N, V), generator=gen, device=dev, dtype=torch.float32)
        g2 = torch.randn((nb, N, V), generator=gen, device=dev, dtype=torch.float32)
        shift = torch.randint(0, V, (nb, N, 1), generator=gen, device=dev, dtype=torch.int64)
        rank = ((A * x).view(1, 1, V) + shift) % V + 1
        bias = -zipf_s * torch.log(rank.to(torch.float32))
        lt = g * ls[b0:b1].view(nb, 1, 1) + bias
        target[b0:b1] = lt.to(dtype)
        draft[b0:b1] = (lt + g2 * ds[b0:b1].view(nb, 1, 1)).to(dtype)
    return target, draft


def topk_masked_logits(B, N, V, K, *, overlap=0.6, dtype=torch.bfloat16, seed=0, device="cpu"):
    """Rows as a top-k / top-p filter leaves them: every logit is -inf except K tokens per row, at
    random positions (even and odd indices alike).  The draft row keeps about `overlap` of the
    target row's tokens and puts the rest of its K tokens elsewhere."""
    g = torch.Generator().manual_seed(seed)
    target = torch.full((B, N, V), float("-inf"), dtype=torch.float32)
    draft = torch.full((B, N, V), float("-inf"), dtype=torch.float32)
    for b in range(B):
        for n in range(N):
            perm = torch.randperm(V, generator=g)
            keep_t = perm[:K]
            n_common = max(1, min(K, int(round(overlap * K))))
            keep_d = torch.cat([keep_t[:n_common], perm[K:2 * K - n_common]])
            vals = 3.0 * torch.randn(K, generator=g)
            target[b, n, keep_t] = vals
            draft[b, n, keep_d[:n_common]] = vals[:n_common] + torch.randn(n_common, generator=g)
            draft[b, n, keep_d[n_common:]] = 3.0 * torch.randn(K - n_common, generator=g)
    return target.to(dtype).to(device), draft.to(dtype).to(device)


def dirichlet_rows(B, N, V, *, alpha=0.3, mix=0.7, seed=0, device="cpu"):
    """p ~ Dirichlet(alpha); q = mix * p + (1 - mix) * Dirichlet(alpha); both
    renormalised in fp64, then rounded to fp32."""
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.full(V, alpha), size=(B, N))
    q = mix * p + (1 - mix) * rng.dirichlet(np.full(V, alpha), size=(B, N))
    p /= p.sum(-1, keepdims=True)
    q /= q.sum(-1, keepdims=True)
    return (torch.from_numpy(p.astype(np.float32)).to(device),
            torch.from_numpy(q.astype(np.float32)).to(device))


def toy_pairs(T: float, lam: float, pairs: int, *, repeats: int = 1, seed: int = 0, device="cpu") -> "Workload":
    """The toy experiment of App. D as a batch: V = 50, one draft step (a root with its two
    children), logits u_p, u_q ~ N(0,1) per pair, target = softmax(u_p / T), draft =
    softmax((lam u_p + (1 - lam) u_q) / T).  (The appendix prints uniform logits; the
    table it reports is reproduced with normal ones.)  Every pair is repeated `repeats` times
    in a row, so that different uniforms meet the same distributions."""
    V, k, depth = 50, 2, 2
    N = tree_nodes(k, depth)
    gen = torch.Generator().manual_seed(seed)
    up = torch.randn((pairs, 1, V), generator=gen, dtype=torch.float32)
    uq = torch.randn((pairs, 1, V), generator=gen, dtype=torch.float32)
    t = up.expand(pairs, N, V).repeat_interleave(repeats, dim=0).contiguous()
    d = (lam * up + (1.0 - lam) * uq).expand(pairs, N, V).repeat_interleave(repeats, dim=0).contiguous()
    return Workload("toy_V50_T%g_lam%g" % (T, lam), pairs * repeats, N, V, k, depth, "fp32", "logits",
                    float(T), float(T), t.to(device), d.to(device), seed,
                    notes={"pairs": pairs, "repeats": repeats})


CONFIG_NAMES = {
    1: "tiny_V16_k2_4096rows_probs_fp32",
    2: "V32000_B1_bin_d4_fp32_logits",
    3: "V32000_B64_bin_d5_bf16_logits",
    4: "V128256_B256_bin_d5_bf16_T0.7",
    5: "V152064_B128_bf16_nearuniform25",
}


def config(i: int, *, device="cpu", seed=0, B=None, k=None, depth=None, V=None) -> Workload:
    """The five configurations the benchmark and the parity tests use.  B, k,
    depth and V can be overridden to get a smaller case of the same recipe."""
    if i == 1:
        V, B, k, depth = V or 16, B or 4096, k or 2, depth or 2
        N = tree_nodes(k, depth)
        p, q = dirichlet_rows(B, N, V, seed=seed, device=device)
        return Workload(CONFIG_NAMES[1], B, N, V, k, depth, "fp32", "probs", 1.0, 1.0, p, q, seed)
    if i == 2:
        V, B, k, depth = V or 32000, B or 1, k or 2, depth or 4
        N = tree_nodes(k, depth)
        t, d = llm_like_logits(B, N, V, logit_std=3.0, draft_noise_std=1.5, dtype=torch.float32,
                               seed=seed, device=device)
        return Workload(CONFIG_NAMES[2], B, N, V, k, depth, "fp32", "logits", 1.0, 1.0, t, d, seed)
    if i == 3:
        V, B, k, depth = V or 32000, B or 64, k or 2, depth or 5
        N = tree_nodes(k, depth)
        gen = torch.Generator().manual_seed(seed + 1000)
        sig = 0.5 + 2.0 * torch.rand(B, generator=gen)
        t, d = llm_like_logits(B, N, V, logit_std=3.0, draft_noise_std=sig, seed=seed, device=device)
        return Workload(CONFIG_NAMES[3], B, N, V, k, depth, "bf16", "logits", 1.0, 1.0, t, d, seed,
                        notes={"draft_noise_std": sig})
    if i == 4:
        V, B, k, depth = V or 128256, B or 256, k or 2, depth or 5
        N = tree_nodes(k, depth)
        t, d = llm_like_logits(B, N, V, logit_std=3.0, draft_noise_std=1.5, seed=seed, device=device)
        return Workload(CONFIG_NAMES[4], B, N, V, k, depth, "bf16", "logits", 0.7, 0.7, t, d, seed)
    if i == 5:
        # k = 4, depth 3 for RRS / RRSw; pass k=2, depth=4 for SpecHub
        V, B, k, depth = V or 152064, B or 128, k or 4, depth or 3
        N = tree_nodes(k, depth)
        std = torch.full((B,), 3.0)
        std[3::4] = 0.5          # every fourth sequence: near-uniform rows (rank bias kept)
        t, d = llm_like_logits(B, N, V, logit_std=std, draft_noise_std=2.0, seed=seed, device=device)
        return Workload(CONFIG_NAMES[5], B, N, V, k, depth, "bf16", "logits", 1.0, 1.0, t, d, seed,
                        notes={"logit_std": std})
    raise ValueError("config index must be 1..5")
