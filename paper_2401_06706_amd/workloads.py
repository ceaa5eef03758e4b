"""Seeded synthetic workloads for the MCSD verification step.

This module only *describes and draws inputs*: the draft tree (Sec. 3.3 of the
paper: a k-ary tree of candidate tokens, level i having k_1*...*k_i nodes), the
KV cache / query tensors, the two logit arrays and the random numbers the
method consumes (candidate ids drawn from the draft distribution, Sec. 3.1-3.2
and Eq. (1); uniforms for the accept test and the endpoint draw).  It contains
none of the verification or attention arithmetic, imports neither the oracle
nor the HIP binding, and is shared by the tests, the smoke check and the bench.

The synthetic shapes stand in for the paper's LLaMA/Vicuna + Alpaca/WMT runs
(Sec. 4.1), which need weights and datasets that are not available here:
attention geometry of LLaMA-7B/13B/2-70B, the 32000-entry LLaMA vocabulary and
the k-configurations of Tables 2, 3, 6.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

WITH_REPLACEMENT = 0
WITHOUT_REPLACEMENT = 1
NAIVE = 2                    # verification only: multi-candidate naive sampling (ablation rule)

SEED_BASE = 0x4D435344  # "MCSD"


# --------------------------------------------------------------------------- tree
@dataclass(frozen=True)
class DraftTree:
    """Draft tree in level order.  Node ids 0..N-1 exclude the root (the last
    context token); ``parent[i] == -1`` marks a child of the root.  Row ids used
    by the logit arrays are ``0`` for the root and ``1 + i`` for node ``i``."""

    kconfig: Tuple[int, ...]
    parent: np.ndarray          # int32 [N]
    depth: np.ndarray           # int32 [N], 1-based level of each node
    q_row: np.ndarray           # int32 [1+N]: row in the draft-logit array, -1 for leaves
    children: List[List[int]]   # children[row] = node ids whose parent is row-1 (row 0 = root)

    @property
    def N(self) -> int:
        return int(self.parent.shape[0])

    @property
    def P(self) -> int:
        """Number of rows that have children (root + internal nodes)."""
        return int((self.q_row >= 0).sum())

    @property
    def gamma(self) -> int:
        return len(self.kconfig)

    @property
    def n_leaves(self) -> int:
        return 1 + self.N - self.P


def parse_kconfig(s: str) -> Tuple[int, ...]:
    """'4x2x2' -> (4, 2, 2) (notation of Tables 2-3)."""
    ks = tuple(int(t) for t in s.lower().replace("×", "x").split("x"))
    if not ks or any(k < 1 for k in ks):
        raise ValueError(f"bad k-config {s!r}")
    return ks


def build_tree(kconfig: Sequence[int]) -> DraftTree:
    """Level-order tree: every node of level i-1 gets k_i children, children of
    one parent are consecutive and appear in sampling order."""
    kconfig = tuple(int(k) for k in kconfig)
    parent: List[int] = []
    depth: List[int] = []
    prev_level = [-1]
    for lvl, k in enumerate(kconfig, start=1):
        cur = []
        for par in prev_level:
            for _ in range(k):
                cur.append(len(parent))
                parent.append(par)
                depth.append(lvl)
        prev_level = cur
    return tree_from_parent(np.asarray(parent, dtype=np.int32), kconfig)


def tree_from_parent(parent: np.ndarray, kconfig: Tuple[int, ...] = ()) -> DraftTree:
    parent = np.asarray(parent, dtype=np.int32)
    n = parent.shape[0]
    depth = np.zeros(n, dtype=np.int32)
    children: List[List[int]] = [[] for _ in range(n + 1)]
    for i in range(n):
        par = int(parent[i])
        if not (-1 <= par < i):
            raise ValueError("parent[i] must satisfy -1 <= parent[i] < i")
        depth[i] = 1 if par < 0 else depth[par] + 1
        children[par + 1].append(i)
    q_row = np.full(n + 1, -1, dtype=np.int32)
    nxt = 0
    for row in range(n + 1):
        if children[row]:
            q_row[row] = nxt
            nxt += 1
    return DraftTree(kconfig=kconfig, parent=parent, depth=depth, q_row=q_row, children=children)


# ------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # 1-based position in the list of synthetic configs
    B: int
    H_q: int
    H_kv: int
    d: int
    dtype: str                      # "fp32" | "bf16" storage type of Q, K, V, O
    prefix: Tuple[int, int]         # (lo, hi) inclusive; lo == hi -> fixed prefix length
    kconfig: Tuple[int, ...]
    V: int
    sigma_q: float                  # std of the noise added to the target logits to get draft logits
    variant: int                    # WITH_REPLACEMENT | WITHOUT_REPLACEMENT
    n_greedy: int = 0               # the first n_greedy sequences run at temperature 0
    description: str = ""

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def tree(self) -> DraftTree:
        return build_tree(self.kconfig)

    def with_(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1", 1, B=1, H_q=1, H_kv=1, d=64, dtype="fp32", prefix=(32, 32),
                   kconfig=(2, 2), V=64, sigma_q=1.0, variant=WITH_REPLACEMENT,
                   description="tiny fp32: 1 head, d 64, prefix 32, tree 2x2, vocab 64"),
    "c2": Workload("c2", 2, B=1, H_q=32, H_kv=32, d=128, dtype="bf16", prefix=(512, 512),
                   kconfig=(4, 2, 2), V=32000, sigma_q=1.0, variant=WITH_REPLACEMENT,
                   description="LLaMA-7B-shaped MHA, prefix 512, tree 4x2x2, with replacement"),
    "c3": Workload("c3", 3, B=1, H_q=40, H_kv=40, d=128, dtype="bf16", prefix=(2048, 2048),
                   kconfig=(8, 2, 1, 1), V=32000, sigma_q=2.0, variant=WITHOUT_REPLACEMENT,
                   description="LLaMA-13B-shaped MHA, prefix 2048, tree 8x2x1x1, without replacement"),
    "c4": Workload("c4", 4, B=16, H_q=32, H_kv=32, d=128, dtype="bf16", prefix=(256, 4096),
                   kconfig=(4, 2, 2, 1, 1), V=32000, sigma_q=1.0, variant=WITHOUT_REPLACEMENT,
                   n_greedy=8,
                   description="batched serving step: 16 seqs, prefix U[256,4096], tree 4x2x2x1x1, "
                               "8 greedy + 8 sampled sequences"),
    "c5": Workload("c5", 5, B=4, H_q=64, H_kv=8, d=128, dtype="bf16", prefix=(16384, 16384),
                   kconfig=(4, 4, 2, 1), V=32000, sigma_q=1.0, variant=WITHOUT_REPLACEMENT,
                   description="LLaMA-2-70B-shaped GQA 64/8, batch 4, prefix 16384, tree 4x4x2x1"),
}


# ------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of finite fp32 values to bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_storage(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    """N(0,1) samples in the storage type: float32 array for fp32, uint16 bit
    patterns for bf16.  Drawn in chunks so the fp32 staging buffer stays small."""
    n = int(np.prod(shape))
    if dtype == "fp32":
        return rng.standard_normal(n, dtype=np.float32).reshape(shape)
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


def open_uniform(rng: np.random.Generator, shape) -> np.ndarray:
    """fp32 uniforms on the open interval (0,1): j / 2^24 with j in [1, 2^24)."""
    j = rng.integers(1, 1 << 24, size=shape, dtype=np.int64)
    return (j.astype(np.float64) / float(1 << 24)).astype(np.float32)


# ------------------------------------------------------------------------ inputs
@dataclass
class AttnInputs:
    B: int
    N: int
    H_q: int
    H_kv: int
    d: int
    dtype: str
    L_stride: int
    scale: float
    q: np.ndarray            # [B][N][H_q][d]         storage type
    k_prefix: np.ndarray     # [B][H_kv][L_stride][d] storage type
    v_prefix: np.ndarray
    prefix_len: np.ndarray   # int32 [B]
    k_tree: np.ndarray       # [B][H_kv][N][d]
    v_tree: np.ndarray
    parent: np.ndarray       # int32 [N]

    def algorithmic_bytes(self) -> int:
        """K and V actually attended (prefix + tree) plus Q in and O out."""
        e = 4 if self.dtype == "fp32" else 2
        kv = 2 * self.H_kv * self.d * e * (int(self.prefix_len.sum()) + self.B * self.N)
        qo = 2 * self.B * self.N * self.H_q * self.d * e
        return kv + qo

    def flops(self) -> int:
        """4*d flops per (query row, attended key) pair, tree keys counted by depth."""
        depth = tree_from_parent(self.parent).depth
        per_seq = [self.H_q * (self.N * int(L) + int(depth.sum())) for L in self.prefix_len]
        return 4 * self.d * int(sum(per_seq))


@dataclass
class VerifyInputs:
    B: int
    N: int
    V: int
    P: int
    variant: int
    tree: DraftTree
    target_logits: np.ndarray   # float32 [B][1+N][V]
    draft_logits: np.ndarray    # float32 [B][P][V]
    cand_tok: np.ndarray        # int32 [B][N]
    u_accept: np.ndarray        # float32 [B][N]
    u_endpoint: np.ndarray      # float32 [B][1+N]
    temperature: np.ndarray     # float32 [B]

    def design_bytes(self) -> int:
        """Logit bytes read when every row owner is evaluated once: both rows of a
        parent, the target row of a leaf; greedy sequences never read draft rows."""
        rows = 0
        for b in range(self.B):
            rows += (1 + self.N) + (0 if self.temperature[b] == 0.0 else self.P)
        return rows * self.V * 4


def gen_attn_inputs(w: Workload, rng: Optional[np.random.Generator] = None,
                    L_stride: Optional[int] = None) -> AttnInputs:
    rng = rng or np.random.default_rng(w.seed)
    tree = w.tree
    lo, hi = w.prefix
    prefix_len = rng.integers(lo, hi + 1, size=w.B, dtype=np.int64).astype(np.int32)
    if L_stride is None:
        L_stride = hi
    N = tree.N
    q = _normal_storage(rng, (w.B, N, w.H_q, w.d), w.dtype)
    k_prefix = _normal_storage(rng, (w.B, w.H_kv, L_stride, w.d), w.dtype)
    v_prefix = _normal_storage(rng, (w.B, w.H_kv, L_stride, w.d), w.dtype)
    k_tree = _normal_storage(rng, (w.B, w.H_kv, N, w.d), w.dtype)
    v_tree = _normal_storage(rng, (w.B, w.H_kv, N, w.d), w.dtype)
    return AttnInputs(B=w.B, N=N, H_q=w.H_q, H_kv=w.H_kv, d=w.d, dtype=w.dtype,
                      L_stride=L_stride, scale=float(1.0 / np.sqrt(w.d)),
                      q=q, k_prefix=k_prefix, v_prefix=v_prefix, prefix_len=prefix_len,
                      k_tree=k_tree, v_tree=v_tree, parent=tree.parent.copy())


def _softmax64(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def draw_candidates(rng: np.random.Generator, q: np.ndarray, k: int, variant: int) -> np.ndarray:
    """k candidate ids from the draft distribution q: i.i.d. (Alg. 1's input) or
    sequentially without replacement, candidate i from q-bar_{i-1} of Eq. (1)
    (Alg. 2's input).  Inverse-CDF draws in token-id order."""
    q = np.asarray(q, dtype=np.float64).copy()
    out = np.empty(k, dtype=np.int32)
    for i in range(k):
        cdf = np.cumsum(q)
        x = int(np.searchsorted(cdf, rng.random() * cdf[-1], side="right"))
        if x >= q.shape[0]:     # only by rounding of the last partial sum
            x = int(np.flatnonzero(q)[-1])
        out[i] = x
        if variant == WITHOUT_REPLACEMENT:
            q[x] = 0.0
    return out


def gen_verify_inputs(w: Workload, rng: Optional[np.random.Generator] = None,
                      variant: Optional[int] = None,
                      temperature: Optional[Sequence[float]] = None,
                      draw_candidates_on_host: bool = True) -> VerifyInputs:
    """Target logits z ~ N(0, 3^2); draft logits z + N(0, sigma_q^2); one
    independent row pair per row owner.  Candidates of a sampled sequence are
    drawn from softmax(draft row / T); a greedy sequence proposes the top-k
    draft tokens in descending order (what a draft model at temperature 0
    producing k distinct candidates amounts to)."""
    rng = rng or np.random.default_rng(w.seed + 1000)
    variant = w.variant if variant is None else variant
    tree = w.tree
    N, P, V = tree.N, tree.P, w.V
    if temperature is None:
        temperature = [0.0] * w.n_greedy + [1.0] * (w.B - w.n_greedy)
    temperature = np.asarray(temperature, dtype=np.float32)
    assert temperature.shape == (w.B,)
    target = (3.0 * rng.standard_normal((w.B, 1 + N, V), dtype=np.float32)).astype(np.float32)
    draft = np.empty((w.B, P, V), dtype=np.float32)
    for row in range(1 + N):
        r = int(tree.q_row[row])
        if r >= 0:
            noise = rng.standard_normal((w.B, V), dtype=np.float32)
            draft[:, r, :] = target[:, row, :] + np.float32(w.sigma_q) * noise
    cand = np.zeros((w.B, N), dtype=np.int32)
    for b in range(w.B if draw_candidates_on_host else 0):    # otherwise the GPU sampler fills them in
        T = float(temperature[b])
        for row in range(1 + N):
            kids = tree.children[row]
            if not kids:
                continue
            zq = draft[b, tree.q_row[row]]
            if T == 0.0:
                order = np.lexsort((np.arange(V), -zq.astype(np.float64)))
                cand[b, kids] = order[: len(kids)].astype(np.int32)
            else:
                cand[b, kids] = draw_candidates(rng, _softmax64(zq / np.float32(T)), len(kids), variant)
    u_acc = open_uniform(rng, (w.B, N))
    u_end = open_uniform(rng, (w.B, 1 + N))
    return VerifyInputs(B=w.B, N=N, V=V, P=P, variant=variant, tree=tree,
                        target_logits=target, draft_logits=draft, cand_tok=cand,
                        u_accept=u_acc, u_endpoint=u_end, temperature=temperature)
