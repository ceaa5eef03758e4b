"""ctypes loader for the CPU oracle (oracle/mcsd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
cpu_baseline leg of the bench.  It marshals numpy arrays into the C functions
and does no arithmetic of its own.  It never imports the HIP binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mcsd_oracle.c")
_LIB = os.path.join(_HERE, "libmcsd_oracle.so")

FP32, BF16 = 0, 1
WITH_REPLACEMENT, WITHOUT_REPLACEMENT = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c = ctypes
        L.mcsd_oracle_max_threads.restype = c.c_int
        L.mcsd_oracle_tree_attn.restype = c.c_int
        L.mcsd_oracle_tree_attn.argtypes = [c.c_int] * 6 + [c.c_long, c.c_double] + [c.c_void_p] * 8 + \
            [c.c_long, c.c_void_p, c.c_int]
        L.mcsd_oracle_verify_parent.restype = c.c_int
        L.mcsd_oracle_verify_parent.argtypes = [c.c_int, c.c_int, c.c_int, c.c_double] + [c.c_void_p] * 4 + \
            [c.c_double] + [c.c_void_p] * 5
        L.mcsd_oracle_verify.restype = c.c_int
        L.mcsd_oracle_verify.argtypes = [c.c_int] * 5 + [c.c_void_p] * 16 + [c.c_int, c.c_int]
        L.mcsd_oracle_draft_parent.restype = c.c_int
        L.mcsd_oracle_draft_parent.argtypes = [c.c_int, c.c_int, c.c_int, c.c_double] + [c.c_void_p] * 4
        L.mcsd_oracle_draft_sample.restype = c.c_int
        L.mcsd_oracle_tree_build.restype = c.c_int
        L.mcsd_oracle_tree_build.argtypes = [c.c_void_p, c.c_int, c.c_int] + [c.c_void_p] * 3
        L.mcsd_oracle_kv_commit.restype = c.c_int
        L.mcsd_oracle_kv_commit.argtypes = [c.c_int] * 6 + [c.c_long, c.c_int, c.c_int] + [c.c_void_p] * 10
        L.mcsd_oracle_draft_sample.argtypes = [c.c_int] * 5 + [c.c_void_p] * 7 + [c.c_int]
        _lib = L
    return _lib


def max_threads() -> int:
    return int(lib().mcsd_oracle_max_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _storage(a: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == FP32 else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"expected {want} storage, got {a.dtype}")
    return a


def tree_attn(q, k_prefix, v_prefix, prefix_len, k_tree, v_tree, parent, scale: float,
              dtype: int, sel: Optional[np.ndarray] = None, n_threads: int = 1) -> np.ndarray:
    """q [B][N][H_q][d]; k/v_prefix [B][H_kv][L_stride][d]; k/v_tree [B][H_kv][N][d];
    storage float32 (dtype FP32) or uint16 bf16 bit patterns (dtype BF16).
    Returns fp64 [B][N][H_q][d], or [n_sel][d] for sel = int32 [n_sel][3] of (b, node, head)."""
    q = _storage(q, dtype)
    k_prefix, v_prefix = _storage(k_prefix, dtype), _storage(v_prefix, dtype)
    k_tree, v_tree = _storage(k_tree, dtype), _storage(v_tree, dtype)
    B, N, H_q, d = q.shape
    H_kv, L_stride = k_prefix.shape[1], k_prefix.shape[2]
    prefix_len = np.ascontiguousarray(prefix_len, dtype=np.int32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    if sel is not None:
        sel = np.ascontiguousarray(sel, dtype=np.int32).reshape(-1, 3)
        out = np.empty((sel.shape[0], d), dtype=np.float64)
        n_sel = sel.shape[0]
    else:
        out = np.empty((B, N, H_q, d), dtype=np.float64)
        n_sel = 0
    rc = lib().mcsd_oracle_tree_attn(B, N, H_q, H_kv, d, dtype, L_stride, float(scale), _ptr(q),
                                     _ptr(k_prefix), _ptr(v_prefix), _ptr(prefix_len), _ptr(k_tree),
                                     _ptr(v_tree), _ptr(parent), _ptr(sel), n_sel, _ptr(out),
                                     int(n_threads))
    if rc != 0:
        raise ValueError(f"mcsd_oracle_tree_attn failed: {rc}")
    return out


@dataclass
class ParentResult:
    accepted: int            # index into the candidate list, -1 if none
    endpoint: int            # endpoint token, -1 if a candidate was accepted
    ratio: np.ndarray        # fp64 [k], NaN where not reached
    margin: float
    residual: Optional[np.ndarray]


def verify_parent(z_p, z_q, tok: Sequence[int], u_acc: Sequence[float], u_end: float,
                  variant: int, T: float = 1.0, want_residual: bool = True) -> ParentResult:
    z_p = np.ascontiguousarray(z_p, dtype=np.float32)
    z_q = np.ascontiguousarray(z_q, dtype=np.float32)
    V = z_p.shape[0]
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    k = tok.shape[0]
    u_acc = np.ascontiguousarray(u_acc, dtype=np.float32)
    assert u_acc.shape[0] == k and z_q.shape[0] == V
    acc = ctypes.c_int32(-1)
    endp = ctypes.c_int32(-1)
    margin = ctypes.c_double(0.0)
    ratio = np.full(max(k, 1), np.nan, dtype=np.float64)
    residual = np.empty(V, dtype=np.float64) if want_residual else None
    rc = lib().mcsd_oracle_verify_parent(V, k, int(variant), float(T), _ptr(z_p), _ptr(z_q), _ptr(tok),
                                         _ptr(u_acc), float(u_end), ctypes.byref(acc),
                                         ctypes.byref(endp), _ptr(ratio), ctypes.byref(margin),
                                         _ptr(residual))
    if rc != 0:
        raise ValueError(f"mcsd_oracle_verify_parent failed: {rc}")
    return ParentResult(int(acc.value), int(endp.value), ratio[:k], float(margin.value), residual)


@dataclass
class VerifyResult:
    acc_child: np.ndarray      # int32 [B][1+N]
    endpoint: np.ndarray       # int32 [B][1+N]
    ratio: np.ndarray          # fp64  [B][N]
    margin: np.ndarray         # fp64  [B][1+N]
    residual: Optional[np.ndarray]   # fp64 [B][1+N][V]
    n_accepted: np.ndarray     # int32 [B]
    accepted_path: np.ndarray  # int32 [B][gamma_max]
    out_tokens: np.ndarray     # int32 [B][gamma_max+1]


def verify(target_logits, draft_logits, q_row, parent, cand_tok, u_accept, u_endpoint,
           temperature, variant: int, gamma_max: int, want_residual: bool = False,
           n_threads: int = 1) -> VerifyResult:
    target_logits = np.ascontiguousarray(target_logits, dtype=np.float32)
    draft_logits = np.ascontiguousarray(draft_logits, dtype=np.float32)
    B, rows, V = target_logits.shape
    N = rows - 1
    P = draft_logits.shape[1]
    q_row = np.ascontiguousarray(q_row, dtype=np.int32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    cand_tok = np.ascontiguousarray(cand_tok, dtype=np.int32).reshape(B, N)
    u_accept = np.ascontiguousarray(u_accept, dtype=np.float32).reshape(B, N)
    u_endpoint = np.ascontiguousarray(u_endpoint, dtype=np.float32).reshape(B, 1 + N)
    temperature = np.ascontiguousarray(temperature, dtype=np.float32).reshape(B)
    acc_child = np.empty((B, 1 + N), dtype=np.int32)
    endpoint = np.empty((B, 1 + N), dtype=np.int32)
    ratio = np.empty((B, N), dtype=np.float64)
    margin = np.empty((B, 1 + N), dtype=np.float64)
    residual = np.empty((B, 1 + N, V), dtype=np.float64) if want_residual else None
    n_accepted = np.empty(B, dtype=np.int32)
    accepted_path = np.empty((B, gamma_max), dtype=np.int32)
    out_tokens = np.empty((B, gamma_max + 1), dtype=np.int32)
    rc = lib().mcsd_oracle_verify(B, N, V, P, int(variant), _ptr(target_logits), _ptr(draft_logits),
                                  _ptr(q_row), _ptr(parent), _ptr(cand_tok), _ptr(u_accept),
                                  _ptr(u_endpoint), _ptr(temperature), _ptr(acc_child), _ptr(endpoint),
                                  _ptr(ratio), _ptr(margin), _ptr(residual), _ptr(n_accepted),
                                  _ptr(accepted_path), _ptr(out_tokens), int(gamma_max), int(n_threads))
    if rc != 0:
        raise ValueError(f"mcsd_oracle_verify failed: {rc}")
    return VerifyResult(acc_child, endpoint, ratio, margin, residual, n_accepted, accepted_path,
                        out_tokens)


def draft_parent(z_q, u, k: int, variant: int, T: float = 1.0):
    """Candidates of one parent (Sec. 3.1; Eq. (1) for variant 1): (tokens int32 [k], margin fp64 [k])."""
    z_q = np.ascontiguousarray(z_q, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float32).reshape(-1)
    assert u.shape[0] >= k
    tok = np.empty(max(k, 1), dtype=np.int32)
    margin = np.empty(max(k, 1), dtype=np.float64)
    rc = lib().mcsd_oracle_draft_parent(int(z_q.shape[0]), int(k), int(variant), float(T), _ptr(z_q), _ptr(u),
                                        _ptr(tok), _ptr(margin))
    if rc != 0:
        raise ValueError(f"mcsd_oracle_draft_parent failed: {rc}")
    return tok[:k], margin[:k]


def draft_sample(draft_logits, q_row, parent, u_draw, temperature, variant: int, n_threads: int = 1):
    """Candidates of whole trees: (cand_tok int32 [B][N], margin fp64 [B][N])."""
    draft_logits = np.ascontiguousarray(draft_logits, dtype=np.float32)
    B, P, V = draft_logits.shape
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    N = parent.shape[0]
    q_row = np.ascontiguousarray(q_row, dtype=np.int32)
    u_draw = np.ascontiguousarray(u_draw, dtype=np.float32).reshape(B, N)
    temperature = np.ascontiguousarray(temperature, dtype=np.float32).reshape(B)
    cand = np.full((B, N), -1, dtype=np.int32)
    margin = np.full((B, N), np.inf, dtype=np.float64)
    rc = lib().mcsd_oracle_draft_sample(B, N, V, P, int(variant), _ptr(draft_logits), _ptr(q_row), _ptr(parent),
                                        _ptr(u_draw), _ptr(temperature), _ptr(cand), _ptr(margin), int(n_threads))
    if rc != 0:
        raise ValueError(f"mcsd_oracle_draft_sample failed: {rc}")
    return cand, margin


def tree_build(kconfig, max_nodes: int = 128):
    """(parent int32 [N], depth int32 [N], q_row int32 [1+N]) of the k-ary candidate tree."""
    kc = np.ascontiguousarray(kconfig, dtype=np.int32)
    parent = np.empty(max_nodes, dtype=np.int32)
    depth = np.empty(max_nodes, dtype=np.int32)
    q_row = np.empty(max_nodes + 1, dtype=np.int32)
    n = lib().mcsd_oracle_tree_build(_ptr(kc), int(kc.shape[0]), int(max_nodes), _ptr(parent), _ptr(depth), _ptr(q_row))
    if n < 0:
        raise ValueError("mcsd_oracle_tree_build: bad k-configuration or too many nodes")
    return parent[:n].copy(), depth[:n].copy(), q_row[:n + 1].copy()


def kv_commit(k_prefix, v_prefix, k_tree, v_tree, n_accepted, accepted_path, out_tokens, prefix_len, root_row=False):
    """Arrays [n_layers][B][H_kv][L_stride | N][d] (any 2- or 4-byte element type); with root_row
    the tree arrays have 1 + N rows, row 0 = the root, which is committed ahead of the path.
    Returns new (k_prefix, v_prefix, prefix_len, next_root, full); the inputs are not modified."""
    k_prefix, v_prefix = np.array(k_prefix, copy=True, order="C"), np.array(v_prefix, copy=True, order="C")
    k_tree, v_tree = np.ascontiguousarray(k_tree), np.ascontiguousarray(v_tree)
    n_layers, B, H_kv, L_stride, d = k_prefix.shape
    N = k_tree.shape[3] - (1 if root_row else 0)
    assert k_tree.shape == (n_layers, B, H_kv, N + (1 if root_row else 0), d) and v_tree.shape == k_tree.shape and v_prefix.shape == k_prefix.shape
    assert k_prefix.dtype == k_tree.dtype == v_prefix.dtype == v_tree.dtype
    n_accepted = np.ascontiguousarray(n_accepted, dtype=np.int32).reshape(B)
    accepted_path = np.ascontiguousarray(accepted_path, dtype=np.int32)
    gamma_max = accepted_path.shape[1]
    out_tokens = np.ascontiguousarray(out_tokens, dtype=np.int32).reshape(B, gamma_max + 1)
    prefix_len = np.array(prefix_len, dtype=np.int32, copy=True).reshape(B)
    next_root = np.empty(B, dtype=np.int32)
    full = np.empty(B, dtype=np.int32)
    rc = lib().mcsd_oracle_kv_commit(n_layers, B, N, H_kv, d, k_prefix.dtype.itemsize, L_stride, gamma_max, 1 if root_row else 0,
                                     _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(n_accepted),
                                     _ptr(accepted_path), _ptr(out_tokens), _ptr(prefix_len), _ptr(next_root),
                                     _ptr(full))
    if rc != 0:
        raise ValueError(f"mcsd_oracle_kv_commit failed: {rc}")
    return k_prefix, v_prefix, prefix_len, next_root, full


def gather_pages(pool: np.ndarray, block_table: np.ndarray, L_stride: int) -> np.ndarray:
    """Definition of the paged prefix layout: pool [n_pages][H_kv][page_size][d], block_table
    [B][pages per sequence]; logical row r of sequence b is pool[block_table[b][r // page_size]][:, r % page_size].
    Returns the contiguous cache [B][H_kv][L_stride][d]."""
    n_pages, H_kv, page_size, d = pool.shape
    B = block_table.shape[0]
    out = np.empty((B, H_kv, L_stride, d), dtype=pool.dtype)
    for b in range(B):
        for r in range(L_stride):
            out[b, :, r, :] = pool[block_table[b, r // page_size], :, r % page_size, :]
    return out
