"""Moves a synthetic workload (numpy, from workloads.py) into device tensors and
builds the argument structs of the C ABI.  Allocation and copies only: torch is
used for device memory and streams, every computation runs in libmcsd's kernels.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

from . import binding as mcsd
from .workloads import AttnInputs, VerifyInputs


def _to_device(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


@dataclass
class AttnCall:
    args: mcsd.AttnArgs
    tensors: Dict[str, torch.Tensor]

    @property
    def out(self) -> torch.Tensor:
        return self.tensors["out"]

    def out_numpy(self) -> np.ndarray:
        """Output as float64 (exact conversion from the storage type)."""
        return self.out.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def make_attn_call(ai: AttnInputs, device="cuda:0", parent_per_seq: bool = False) -> AttnCall:
    t = {
        "q": _to_device(ai.q, ai.dtype, device),
        "k_prefix": _to_device(ai.k_prefix, ai.dtype, device),
        "v_prefix": _to_device(ai.v_prefix, ai.dtype, device),
        "k_tree": _to_device(ai.k_tree, ai.dtype, device),
        "v_tree": _to_device(ai.v_tree, ai.dtype, device),
        "prefix_len": torch.from_numpy(ai.prefix_len.astype(np.int32)).to(device),
    }
    parent = ai.parent.astype(np.int32)
    if parent_per_seq:
        parent = np.ascontiguousarray(np.broadcast_to(parent, (ai.B, ai.N)))
    t["parent"] = torch.from_numpy(parent).to(device)
    t["out"] = torch.zeros_like(t["q"])
    dt = mcsd.DTYPE_FP32 if ai.dtype == "fp32" else mcsd.DTYPE_BF16
    desc = mcsd.attn_desc(ai.B, ai.N, ai.H_q, ai.H_kv, ai.d, dt, ai.L_stride, ai.scale, parent_per_seq)
    ws_bytes = mcsd.mcsd_attn_workspace_bytes(desc)
    t["workspace"] = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=device)
    args = mcsd.attn_args(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_len"], t["k_tree"], t["v_tree"],
                          t["parent"], t["out"], ai.scale, t["workspace"])
    return AttnCall(args, t)


@dataclass
class VerifyCall:
    args: mcsd.VerifyArgs
    tensors: Dict[str, torch.Tensor]

    def results(self) -> Dict[str, np.ndarray]:
        names = ["n_accepted", "accepted_path", "out_tokens", "acc_child", "endpoint", "flags", "ratio",
                 "residual_out"]
        return {n: self.tensors[n].detach().cpu().numpy() for n in names if self.tensors.get(n) is not None}


def make_verify_call(vi: VerifyInputs, device="cuda:0", want_ratio: bool = True,
                     want_residual: bool = False, near_tie_eps: float = 1e-6) -> VerifyCall:
    B, N, V = vi.B, vi.N, vi.V
    G = vi.tree.gamma
    i32 = dict(dtype=torch.int32, device=device)
    t: Dict[str, Optional[torch.Tensor]] = {
        "target_logits": torch.from_numpy(vi.target_logits).to(device),
        "draft_logits": torch.from_numpy(vi.draft_logits).to(device),
        "q_row": torch.from_numpy(vi.tree.q_row.astype(np.int32)).to(device),
        "parent": torch.from_numpy(vi.tree.parent.astype(np.int32)).to(device),
        "cand_tok": torch.from_numpy(vi.cand_tok.astype(np.int32)).to(device),
        "u_accept": torch.from_numpy(vi.u_accept).to(device),
        "u_endpoint": torch.from_numpy(vi.u_endpoint).to(device),
        "temperature": torch.from_numpy(vi.temperature).to(device),
        "n_accepted": torch.full((B,), -7, **i32),
        "accepted_path": torch.full((B, G), -7, **i32),
        "out_tokens": torch.full((B, G + 1), -7, **i32),
        "acc_child": torch.full((B, 1 + N), -7, **i32),
        "endpoint": torch.full((B, 1 + N), -7, **i32),
        "flags": torch.full((B, 1 + N), -7, **i32),
        "ratio": torch.full((B, N), -7.0, dtype=torch.float32, device=device) if want_ratio else None,
        "residual_out": torch.full((B, 1 + N, V), -7.0, dtype=torch.float32, device=device)
        if want_residual else None,
    }
    args = mcsd.verify_args(t["target_logits"], t["draft_logits"], t["q_row"], t["parent"], t["cand_tok"],
                            t["u_accept"], t["u_endpoint"], t["temperature"], t["n_accepted"],
                            t["accepted_path"], t["out_tokens"], t["acc_child"], t["endpoint"], t["flags"],
                            vi.variant, ratio=t["ratio"], residual_out=t["residual_out"],
                            near_tie_eps=near_tie_eps)
    return VerifyCall(args, t)


@dataclass
class DraftCall:
    args: "mcsd.DraftArgs"
    tensors: Dict[str, Optional[torch.Tensor]]

    def results(self) -> Dict[str, np.ndarray]:
        return {n: self.tensors[n].detach().cpu().numpy() for n in ("cand_tok", "flags")}


def make_draft_call(vi: VerifyInputs, u_draw: np.ndarray, device="cuda:0", near_tie_eps: float = 1e-6,
                    cand_tok: Optional[torch.Tensor] = None) -> DraftCall:
    """Draft-side sampling for the trees of `vi` (its draft logits, tree, temperatures and variant) with
    the uniforms u_draw [B][N].  `cand_tok` may be the candidate tensor of a verification call, which
    then consumes the sampler's output on the same stream."""
    B, N = vi.B, vi.N
    t: Dict[str, Optional[torch.Tensor]] = {
        "draft_logits": torch.from_numpy(vi.draft_logits).to(device),
        "q_row": torch.from_numpy(vi.tree.q_row.astype(np.int32)).to(device),
        "parent": torch.from_numpy(vi.tree.parent.astype(np.int32)).to(device),
        "u_draw": torch.from_numpy(np.ascontiguousarray(u_draw, dtype=np.float32)).to(device),
        "temperature": torch.from_numpy(vi.temperature).to(device),
        "cand_tok": cand_tok if cand_tok is not None else torch.full((B, N), -7, dtype=torch.int32, device=device),
        "flags": torch.full((B, N), -7, dtype=torch.int32, device=device),
    }
    args = mcsd.draft_args(t["draft_logits"], t["q_row"], t["parent"], t["u_draw"], t["temperature"],
                           t["cand_tok"], t["flags"], vi.variant, near_tie_eps=near_tie_eps)
    return DraftCall(args, t)


def leaf_paths(parent: np.ndarray):
    """Root-to-leaf node paths of a tree given by its parent array: list of lists of node ids."""
    n = parent.shape[0]
    has_child = np.zeros(n, dtype=bool)
    has_child[parent[parent >= 0]] = True
    paths = []
    for leaf in np.flatnonzero(~has_child):
        path, v = [], int(leaf)
        while v >= 0:
            path.append(v)
            v = int(parent[v])
        paths.append(path[::-1])
    return paths


def make_replicated_attn_call(tree_call: AttnCall, ai: AttnInputs, device="cuda:0") -> AttnCall:
    """The same attention problem WITHOUT tree attention (the arrangement Sec. 3.3 starts from):
    every candidate sequence (root-to-leaf path) becomes a sequence of its own with a private copy
    of the prefix cache and its candidates as a chain.  Built on the device from the tensors of
    `tree_call` by copies and gathers only.  Replica r = b * n_leaves + leaf index; all leaves
    must have the same depth (true for k-configuration trees)."""
    paths = leaf_paths(ai.parent)
    depth = len(paths[0])
    if any(len(p) != depth for p in paths):
        raise ValueError("leaves of different depth")
    n_leaves = len(paths)
    idx = torch.tensor(paths, dtype=torch.long, device=device)           # [n_leaves][depth]
    t0 = tree_call.tensors
    B = ai.B
    t = {
        # q [B][N][H_q][d] -> [B][n_leaves][depth][H_q][d]
        "q": t0["q"][:, idx].reshape(B * n_leaves, depth, ai.H_q, ai.d).contiguous(),
        # k_tree [B][H_kv][N][d] -> [B][n_leaves][H_kv][depth][d]
        "k_tree": t0["k_tree"][:, :, idx].permute(0, 2, 1, 3, 4).reshape(B * n_leaves, ai.H_kv, depth, ai.d).contiguous(),
        "v_tree": t0["v_tree"][:, :, idx].permute(0, 2, 1, 3, 4).reshape(B * n_leaves, ai.H_kv, depth, ai.d).contiguous(),
        "k_prefix": t0["k_prefix"].repeat_interleave(n_leaves, dim=0),
        "v_prefix": t0["v_prefix"].repeat_interleave(n_leaves, dim=0),
        "prefix_len": t0["prefix_len"].repeat_interleave(n_leaves),
        "parent": torch.arange(-1, depth - 1, dtype=torch.int32, device=device),
    }
    t["out"] = torch.zeros_like(t["q"])
    dt = mcsd.DTYPE_FP32 if ai.dtype == "fp32" else mcsd.DTYPE_BF16
    desc = mcsd.attn_desc(B * n_leaves, depth, ai.H_q, ai.H_kv, ai.d, dt, ai.L_stride, ai.scale)
    t["workspace"] = torch.empty(max(mcsd.mcsd_attn_workspace_bytes(desc), 256), dtype=torch.uint8, device=device)
    args = mcsd.attn_args(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_len"], t["k_tree"], t["v_tree"],
                          t["parent"], t["out"], ai.scale, t["workspace"])
    call = AttnCall(args, t)
    call.paths = paths
    return call


def make_paged_attn_call(tree_call: AttnCall, ai: AttnInputs, page_size: int, seed: int = 0, spare_pages: int = 3,
                         device="cuda:0"):
    """The attention problem of `tree_call` with its prefix cache scattered into a page pool in a
    random page order (device copies only).  Returns (AttnCall, PagedKV, block_table numpy)."""
    B, H_kv, Ls, d = ai.B, ai.H_kv, ai.L_stride, ai.d
    per_seq = (Ls + page_size - 1) // page_size
    n_pages = B * per_seq + spare_pages
    rng = np.random.default_rng(seed)
    table = rng.permutation(n_pages)[: B * per_seq].reshape(B, per_seq).astype(np.int32)
    t0 = tree_call.tensors
    padded = per_seq * page_size
    def scatter(cache):
        pool = torch.full((n_pages, H_kv, page_size, d), float("nan"), dtype=cache.dtype, device=device)
        c = cache
        if padded != Ls:
            c = torch.cat([cache, torch.zeros((B, H_kv, padded - Ls, d), dtype=cache.dtype, device=device)], dim=2)
        pages = c.reshape(B, H_kv, per_seq, page_size, d).permute(0, 2, 1, 3, 4).reshape(B * per_seq, H_kv, page_size, d)
        pool[torch.from_numpy(table.reshape(-1).astype(np.int64)).to(device)] = pages
        return pool
    t = dict(t0)
    t["k_pool"], t["v_pool"] = scatter(t0["k_prefix"]), scatter(t0["v_prefix"])
    t["block_table"] = torch.from_numpy(table).to(device)
    t["out"] = torch.zeros_like(t0["out"])
    t["workspace"] = torch.empty_like(t0["workspace"])
    args, paged = mcsd.paged_attn_args(t["q"], t["k_pool"], t["v_pool"], t["block_table"], t["prefix_len"],
                                       t["k_tree"], t["v_tree"], t["parent"], t["out"], ai.scale, Ls, t["workspace"])
    del t["k_prefix"], t["v_prefix"]
    return AttnCall(args, t), paged, table
