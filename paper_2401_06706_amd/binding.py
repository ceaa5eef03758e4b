"""ctypes binding of libmcsd.so: argument marshalling only.

Every function here fills the C structs of include/mcsd.h from torch tensors
(device pointers, shapes) and calls the entry point of the same name; all
computation happens in the HIP kernels.  There is no fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmcsd.so")

DTYPE_FP32, DTYPE_BF16 = 0, 1
WITH_REPLACEMENT, WITHOUT_REPLACEMENT, NAIVE = 0, 1, 2
MAX_NODES, MAX_VOCAB = 128, 65536

FLAG_NEAR_TIE_ACCEPT, FLAG_NEAR_TIE_ENDPOINT, FLAG_BAD_TOKEN = 1, 2, 4
FLAG_ZERO_DRAFT_PROB, FLAG_ZERO_RESIDUAL, FLAG_NONFINITE, FLAG_BAD_TREE = 8, 16, 32, 64

EXPORTS = ["mcsd_last_error", "mcsd_version", "mcsd_tree_validate", "mcsd_attn_workspace_bytes",
           "mcsd_tree_attn", "mcsd_tree_attn_static", "mcsd_attn_plan_override", "mcsd_tree_attn_paged", "mcsd_verify_workspace_bytes", "mcsd_verify_sample", "mcsd_verify_step",
           "mcsd_draft_sample", "mcsd_tree_size", "mcsd_tree_build", "mcsd_kv_commit", "mcsd_kv_commit_paged",
           "mcsd_kernel_timing", "mcsd_kernel_count", "mcsd_kernel_name", "mcsd_kernel_timing_read"]


class McsdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libmcsd error {code}: {msg}")
        self.code = code


class AttnDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("B", C.c_int32), ("N", C.c_int32), ("H_q", C.c_int32),
                ("H_kv", C.c_int32), ("d", C.c_int32), ("dtype", C.c_int32), ("L_stride", C.c_int32),
                ("scale", C.c_float), ("parent_per_seq", C.c_int32), ("root_row", C.c_int32)]


class AttnBufs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("q", C.c_void_p), ("k_prefix", C.c_void_p),
                ("v_prefix", C.c_void_p), ("prefix_len", C.c_void_p), ("k_tree", C.c_void_p),
                ("v_tree", C.c_void_p), ("parent", C.c_void_p), ("out", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class VerifyDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("B", C.c_int32), ("N", C.c_int32), ("V", C.c_int32),
                ("P", C.c_int32), ("variant", C.c_int32), ("gamma_max", C.c_int32),
                ("near_tie_eps", C.c_float), ("parent_per_seq", C.c_int32)]


class VerifyBufs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_void_p) for n in (
        "target_logits", "draft_logits", "q_row", "parent", "cand_tok", "u_accept", "u_endpoint",
        "temperature", "n_accepted", "accepted_path", "out_tokens", "acc_child", "endpoint", "ratio",
        "flags", "residual_out", "workspace")] + [("workspace_bytes", C.c_size_t)]


class PagedKV(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("page_size", C.c_int32), ("n_pages", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("block_table", C.c_void_p)]


class DraftDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("B", C.c_int32), ("N", C.c_int32), ("V", C.c_int32),
                ("P", C.c_int32), ("variant", C.c_int32), ("near_tie_eps", C.c_float),
                ("parent_per_seq", C.c_int32)]


class DraftBufs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_void_p) for n in (
        "draft_logits", "q_row", "parent", "u_draw", "temperature", "cand_tok", "flags")]


class CommitDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("B", C.c_int32), ("N", C.c_int32), ("H_kv", C.c_int32),
                ("d", C.c_int32), ("dtype", C.c_int32), ("L_stride", C.c_int32), ("gamma_max", C.c_int32),
                ("n_layers", C.c_int32), ("root_row", C.c_int32)]


class CommitBufs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_void_p) for n in (
        "k_prefix", "v_prefix", "k_tree", "v_tree", "n_accepted", "accepted_path", "out_tokens",
        "prefix_len", "next_root", "flags")]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Loads the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2401_06706_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.mcsd_last_error.restype = C.c_char_p
        L.mcsd_version.restype = C.c_char_p
        L.mcsd_tree_validate.argtypes = [C.c_void_p, C.c_int32]
        L.mcsd_tree_validate.restype = C.c_int32
        L.mcsd_attn_workspace_bytes.argtypes = [C.POINTER(AttnDesc)]
        L.mcsd_attn_workspace_bytes.restype = C.c_size_t
        L.mcsd_verify_workspace_bytes.argtypes = [C.POINTER(VerifyDesc)]
        L.mcsd_verify_workspace_bytes.restype = C.c_size_t
        L.mcsd_tree_attn.argtypes = [C.POINTER(AttnDesc), C.POINTER(AttnBufs), C.c_void_p]
        L.mcsd_tree_attn.restype = C.c_int32
        L.mcsd_tree_attn_static.argtypes = [C.POINTER(AttnDesc), C.POINTER(AttnBufs), C.c_void_p]
        L.mcsd_tree_attn_static.restype = C.c_int32
        L.mcsd_attn_plan_override.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.mcsd_attn_plan_override.restype = C.c_int32
        L.mcsd_tree_attn_paged.argtypes = [C.POINTER(AttnDesc), C.POINTER(AttnBufs), C.POINTER(PagedKV), C.c_void_p]
        L.mcsd_tree_attn_paged.restype = C.c_int32
        L.mcsd_verify_sample.argtypes = [C.POINTER(VerifyDesc), C.POINTER(VerifyBufs), C.c_void_p]
        L.mcsd_verify_sample.restype = C.c_int32
        L.mcsd_verify_step.argtypes = [C.POINTER(AttnDesc), C.POINTER(AttnBufs), C.POINTER(VerifyDesc),
                                       C.POINTER(VerifyBufs), C.c_void_p]
        L.mcsd_verify_step.restype = C.c_int32
        L.mcsd_draft_sample.argtypes = [C.POINTER(DraftDesc), C.POINTER(DraftBufs), C.c_void_p]
        L.mcsd_draft_sample.restype = C.c_int32
        L.mcsd_tree_size.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.mcsd_tree_size.restype = C.c_int32
        L.mcsd_tree_build.argtypes = [C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 5 + [C.c_int32, C.c_void_p]
        L.mcsd_tree_build.restype = C.c_int32
        L.mcsd_kv_commit.argtypes = [C.POINTER(CommitDesc), C.POINTER(CommitBufs), C.c_void_p]
        L.mcsd_kv_commit.restype = C.c_int32
        L.mcsd_kv_commit_paged.argtypes = [C.POINTER(CommitDesc), C.POINTER(CommitBufs), C.POINTER(PagedKV), C.c_void_p]
        L.mcsd_kv_commit_paged.restype = C.c_int32
        L.mcsd_kernel_timing.argtypes = [C.c_int32]
        L.mcsd_kernel_timing.restype = C.c_int32
        L.mcsd_kernel_count.restype = C.c_int32
        L.mcsd_kernel_name.argtypes = [C.c_int32]
        L.mcsd_kernel_name.restype = C.c_char_p
        L.mcsd_kernel_timing_read.argtypes = [C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.mcsd_kernel_timing_read.restype = C.c_int32
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise McsdError(rc, lib().mcsd_last_error().decode())


def _ptr(t: Optional[torch.Tensor], dtype=None, name: str = "tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def version() -> str:
    return lib().mcsd_version().decode()


def mcsd_tree_validate(parent_host) -> None:
    """parent_host: int32 numpy array / CPU tensor [N]."""
    import numpy as np
    a = np.ascontiguousarray(parent_host, dtype=np.int32)
    _check(lib().mcsd_tree_validate(a.ctypes.data_as(C.c_void_p), a.shape[0]))


# ------------------------------------------------------------------ tree attention
@dataclass
class AttnArgs:
    desc: AttnDesc
    bufs: AttnBufs
    keep: tuple       # tensors referenced by the raw pointers


def attn_desc(B, N, H_q, H_kv, d, dtype, L_stride, scale, parent_per_seq=False, root_row=False) -> AttnDesc:
    return AttnDesc(C.sizeof(AttnDesc), B, N, H_q, H_kv, d, dtype, L_stride, float(scale),
                    1 if parent_per_seq else 0, 1 if root_row else 0)


def mcsd_attn_workspace_bytes(desc: AttnDesc) -> int:
    n = lib().mcsd_attn_workspace_bytes(C.byref(desc))
    return int(n)


def attn_args(q, k_prefix, v_prefix, prefix_len, k_tree, v_tree, parent, out, scale,
              workspace: Optional[torch.Tensor] = None) -> AttnArgs:
    """Shapes: q/out [B][N][H_q][d]; k/v_prefix [B][H_kv][L_stride][d]; k/v_tree [B][H_kv][N][d];
    prefix_len int32 [B]; parent int32 [N] or [B][N].  If q, out, k_tree and v_tree have one row
    more than parent has entries, row 0 is the root (root_row = 1 in the descriptor)."""
    B, N, H_q, d = q.shape
    root_row = parent.shape[-1] == N - 1
    H_kv, L_stride = k_prefix.shape[1], k_prefix.shape[2]
    if q.dtype == torch.float32:
        dt = DTYPE_FP32
    elif q.dtype == torch.bfloat16:
        dt = DTYPE_BF16
    else:
        raise ValueError(f"unsupported dtype {q.dtype}")
    if tuple(k_prefix.shape) != (B, H_kv, L_stride, d) or tuple(v_prefix.shape) != (B, H_kv, L_stride, d):
        raise ValueError("k_prefix / v_prefix shape mismatch")
    if tuple(k_tree.shape) != (B, H_kv, N, d) or tuple(v_tree.shape) != (B, H_kv, N, d):
        raise ValueError("k_tree / v_tree shape mismatch")
    if tuple(out.shape) != (B, N, H_q, d) or tuple(prefix_len.shape) != (B,):
        raise ValueError("out / prefix_len shape mismatch")
    Np = N - 1 if root_row else N
    if tuple(parent.shape) not in ((Np,), (B, Np)):
        raise ValueError("parent must be [N] or [B][N]")
    desc = attn_desc(B, Np, H_q, H_kv, d, dt, L_stride, scale, parent.dim() == 2, root_row)
    bufs = AttnBufs(C.sizeof(AttnBufs), _ptr(q, q.dtype, "q"), _ptr(k_prefix, q.dtype, "k_prefix"),
                    _ptr(v_prefix, q.dtype, "v_prefix"), _ptr(prefix_len, torch.int32, "prefix_len"),
                    _ptr(k_tree, q.dtype, "k_tree"), _ptr(v_tree, q.dtype, "v_tree"),
                    _ptr(parent, torch.int32, "parent"), _ptr(out, q.dtype, "out"),
                    _ptr(workspace, None, "workspace"),
                    0 if workspace is None else workspace.numel() * workspace.element_size())
    return AttnArgs(desc, bufs, (q, k_prefix, v_prefix, prefix_len, k_tree, v_tree, parent, out, workspace))


def mcsd_tree_attn(args: AttnArgs, stream=None) -> None:
    _check(lib().mcsd_tree_attn(C.byref(args.desc), C.byref(args.bufs), _stream(stream)))


STATIC_SCRATCH_BYTES = 96 << 20


def mcsd_tree_attn_static(args: AttnArgs, stream=None) -> None:
    """mcsd_tree_attn without a workspace: the library's own static device buffer holds the partials."""
    _check(lib().mcsd_tree_attn_static(C.byref(args.desc), C.byref(args.bufs), _stream(stream)))


def mcsd_attn_plan_override(variant: int = 0, chunk_tiles: int = 0, target_items: int = 0) -> None:
    """Test / tuning aid: force the attention kernel variant (1..3), the segment length in 32-key
    tiles, or the item target of the launch plan, for all later calls (0 = automatic)."""
    _check(lib().mcsd_attn_plan_override(int(variant), int(chunk_tiles), int(target_items)))


def paged_attn_args(q, k_pool, v_pool, block_table, prefix_len, k_tree, v_tree, parent, out, scale, L_stride: int,
                    workspace: Optional[torch.Tensor] = None):
    """Like attn_args, with the prefix in pools [n_pages][H_kv][page_size][d] and block_table
    int32 [B][max_pages_per_seq].  Returns (AttnArgs, PagedKV)."""
    B, N, H_q, d = q.shape
    n_pages, H_kv, page_size, _ = k_pool.shape
    if tuple(v_pool.shape) != tuple(k_pool.shape) or k_pool.shape[3] != d:
        raise ValueError("pool shape mismatch")
    if block_table.dim() != 2 or block_table.shape[0] != B:
        raise ValueError("block_table must be [B][max_pages_per_seq]")
    if q.dtype == torch.float32:
        dt = DTYPE_FP32
    elif q.dtype == torch.bfloat16:
        dt = DTYPE_BF16
    else:
        raise ValueError(f"unsupported dtype {q.dtype}")
    desc = attn_desc(B, N, H_q, H_kv, d, dt, L_stride, scale, parent.dim() == 2)
    bufs = AttnBufs(C.sizeof(AttnBufs), _ptr(q, q.dtype, "q"), _ptr(k_pool, q.dtype, "k_pool"),
                    _ptr(v_pool, q.dtype, "v_pool"), _ptr(prefix_len, torch.int32, "prefix_len"),
                    _ptr(k_tree, q.dtype, "k_tree"), _ptr(v_tree, q.dtype, "v_tree"),
                    _ptr(parent, torch.int32, "parent"), _ptr(out, q.dtype, "out"),
                    _ptr(workspace, None, "workspace"),
                    0 if workspace is None else workspace.numel() * workspace.element_size())
    paged = PagedKV(C.sizeof(PagedKV), page_size, n_pages, block_table.shape[1],
                    _ptr(block_table, torch.int32, "block_table"))
    keep = (q, k_pool, v_pool, block_table, prefix_len, k_tree, v_tree, parent, out, workspace)
    return AttnArgs(desc, bufs, keep), paged


def mcsd_tree_attn_paged(args: AttnArgs, paged: PagedKV, stream=None) -> None:
    _check(lib().mcsd_tree_attn_paged(C.byref(args.desc), C.byref(args.bufs), C.byref(paged), _stream(stream)))


# -------------------------------------------------------------------- verification
@dataclass
class VerifyArgs:
    desc: VerifyDesc
    bufs: VerifyBufs
    keep: tuple


def verify_args(target_logits, draft_logits, q_row, parent, cand_tok, u_accept, u_endpoint, temperature,
                n_accepted, accepted_path, out_tokens, acc_child, endpoint, flags, variant: int,
                ratio=None, residual_out=None, near_tie_eps: float = 1e-6) -> VerifyArgs:
    """Shapes: target_logits [B][1+N][V]; draft_logits [B][P][V]; q_row int32 [1+N] and parent int32 [N]
    (one tree for the batch) or q_row [B][1+N] and parent [B][N] (one tree per sequence);
    cand_tok int32 [B][N]; u_accept [B][N]; u_endpoint [B][1+N]; temperature [B];
    outputs n_accepted [B], accepted_path [B][gamma_max], out_tokens [B][gamma_max+1],
    acc_child / endpoint / flags [B][1+N], ratio [B][N] (optional), residual_out [B][1+N][V] (optional)."""
    B, rows, V = target_logits.shape
    N = rows - 1
    P = draft_logits.shape[1]
    gamma_max = accepted_path.shape[1]
    f32, i32 = torch.float32, torch.int32
    per_seq = parent.dim() == 2
    shapes = [(draft_logits, (B, P, V)), (q_row, (B, 1 + N) if per_seq else (1 + N,)),
              (parent, (B, N) if per_seq else (N,)), (cand_tok, (B, N)),
              (u_accept, (B, N)), (u_endpoint, (B, 1 + N)), (temperature, (B,)), (n_accepted, (B,)),
              (accepted_path, (B, gamma_max)), (out_tokens, (B, gamma_max + 1)), (acc_child, (B, 1 + N)),
              (endpoint, (B, 1 + N)), (flags, (B, 1 + N))]
    if ratio is not None:
        shapes.append((ratio, (B, N)))
    if residual_out is not None:
        shapes.append((residual_out, (B, 1 + N, V)))
    for t, shp in shapes:
        if tuple(t.shape) != shp:
            raise ValueError(f"shape mismatch: got {tuple(t.shape)}, expected {shp}")
    desc = VerifyDesc(C.sizeof(VerifyDesc), B, N, V, P, int(variant), gamma_max, float(near_tie_eps),
                      1 if per_seq else 0)
    bufs = VerifyBufs(C.sizeof(VerifyBufs),
                      _ptr(target_logits, f32, "target_logits"), _ptr(draft_logits, f32, "draft_logits"),
                      _ptr(q_row, i32, "q_row"), _ptr(parent, i32, "parent"), _ptr(cand_tok, i32, "cand_tok"),
                      _ptr(u_accept, f32, "u_accept"), _ptr(u_endpoint, f32, "u_endpoint"),
                      _ptr(temperature, f32, "temperature"), _ptr(n_accepted, i32, "n_accepted"),
                      _ptr(accepted_path, i32, "accepted_path"), _ptr(out_tokens, i32, "out_tokens"),
                      _ptr(acc_child, i32, "acc_child"), _ptr(endpoint, i32, "endpoint"),
                      _ptr(ratio, f32, "ratio"), _ptr(flags, i32, "flags"),
                      _ptr(residual_out, f32, "residual_out"), None, 0)
    return VerifyArgs(desc, bufs, (target_logits, draft_logits, q_row, parent, cand_tok, u_accept,
                                   u_endpoint, temperature, n_accepted, accepted_path, out_tokens,
                                   acc_child, endpoint, ratio, flags, residual_out))


def mcsd_verify_workspace_bytes(desc: VerifyDesc) -> int:
    return int(lib().mcsd_verify_workspace_bytes(C.byref(desc)))


def mcsd_verify_sample(args: VerifyArgs, stream=None) -> None:
    _check(lib().mcsd_verify_sample(C.byref(args.desc), C.byref(args.bufs), _stream(stream)))


def mcsd_verify_step(attn: AttnArgs, verify: VerifyArgs, stream=None) -> None:
    _check(lib().mcsd_verify_step(C.byref(attn.desc), C.byref(attn.bufs), C.byref(verify.desc),
                                  C.byref(verify.bufs), _stream(stream)))


# ----------------------------------------------------------- draft-side candidates
@dataclass
class DraftArgs:
    desc: DraftDesc
    bufs: DraftBufs
    keep: tuple


def draft_args(draft_logits, q_row, parent, u_draw, temperature, cand_tok, flags, variant: int,
               near_tie_eps: float = 1e-6) -> DraftArgs:
    """Shapes: draft_logits [B][P][V]; q_row int32 [1+N] and parent int32 [N], or q_row [B][1+N] and
    parent [B][N] (one tree per sequence); u_draw [B][N]; temperature [B]; outputs cand_tok int32
    [B][N], flags int32 [B][N]."""
    B, P, V = draft_logits.shape
    per_seq = parent.dim() == 2
    N = parent.shape[-1]
    f32, i32 = torch.float32, torch.int32
    for t, shp in [(q_row, (B, 1 + N) if per_seq else (1 + N,)), (parent, (B, N) if per_seq else (N,)), (u_draw, (B, N)), (temperature, (B,)), (cand_tok, (B, N)), (flags, (B, N))]:
        if tuple(t.shape) != shp:
            raise ValueError(f"shape mismatch: got {tuple(t.shape)}, expected {shp}")
    desc = DraftDesc(C.sizeof(DraftDesc), B, N, V, P, int(variant), float(near_tie_eps), 1 if per_seq else 0)
    bufs = DraftBufs(C.sizeof(DraftBufs), _ptr(draft_logits, f32, "draft_logits"), _ptr(q_row, i32, "q_row"),
                     _ptr(parent, i32, "parent"), _ptr(u_draw, f32, "u_draw"),
                     _ptr(temperature, f32, "temperature"), _ptr(cand_tok, i32, "cand_tok"),
                     _ptr(flags, i32, "flags"))
    return DraftArgs(desc, bufs, (draft_logits, q_row, parent, u_draw, temperature, cand_tok, flags))


def mcsd_draft_sample(args: DraftArgs, stream=None) -> None:
    _check(lib().mcsd_draft_sample(C.byref(args.desc), C.byref(args.bufs), _stream(stream)))


# ---------------------------------------------------- candidate tree and KV commit
def mcsd_tree_size(kconfig) -> tuple:
    """(N, P) of the k-ary candidate tree; host only."""
    import numpy as np
    kc = np.ascontiguousarray(kconfig, dtype=np.int32)
    n, pr = C.c_int32(0), C.c_int32(0)
    _check(lib().mcsd_tree_size(kc.ctypes.data_as(C.c_void_p), kc.shape[0], C.byref(n), C.byref(pr)))
    return int(n.value), int(pr.value)


def mcsd_tree_build(kconfig, parent, depth, q_row, prefix_len=None, position_ids=None, stream=None) -> None:
    """kconfig: host sequence; parent/depth int32 [N], q_row int32 [1+N] device tensors;
    position_ids int32 [B][N], or [B][1+N] with the root as entry 0 (optional, needs prefix_len int32 [B])."""
    import numpy as np
    kc = np.ascontiguousarray(kconfig, dtype=np.int32)
    N, _ = mcsd_tree_size(kc)
    i32 = torch.int32
    if tuple(parent.shape) != (N,) or tuple(depth.shape) != (N,) or tuple(q_row.shape) != (N + 1,):
        raise ValueError("parent / depth must be [N], q_row [1+N]")
    B = 1
    root_row = 0
    if position_ids is not None:
        B = position_ids.shape[0]
        root_row = 1 if position_ids.shape[1] == N + 1 else 0
        if tuple(position_ids.shape) != (B, N + root_row) or prefix_len is None or tuple(prefix_len.shape) != (B,):
            raise ValueError("position_ids must be [B][N] (or [B][1+N] with a root row) with prefix_len [B]")
    _check(lib().mcsd_tree_build(kc.ctypes.data_as(C.c_void_p), kc.shape[0], B, _ptr(prefix_len, i32, "prefix_len"),
                                 _ptr(parent, i32, "parent"), _ptr(depth, i32, "depth"), _ptr(q_row, i32, "q_row"),
                                 _ptr(position_ids, i32, "position_ids"), root_row, _stream(stream)))


@dataclass
class CommitArgs:
    desc: CommitDesc
    bufs: CommitBufs
    keep: tuple


def commit_args(k_prefix, v_prefix, k_tree, v_tree, n_accepted, accepted_path, out_tokens, prefix_len,
                next_root, flags, root_row: bool = False) -> CommitArgs:
    """k/v_prefix [n_layers][B][H_kv][L_stride][d] (or 4-D for one layer), k/v_tree [...][N][d]
    ([...][1+N][d] with root_row: row 0 = the root); n_accepted [B], accepted_path [B][gamma_max],
    out_tokens [B][gamma_max+1], prefix_len [B] (in/out), next_root [B], flags [B]."""
    if k_prefix.dim() == 4:
        n_layers, (B, H_kv, L_stride, d) = 1, k_prefix.shape
    else:
        n_layers, B, H_kv, L_stride, d = k_prefix.shape
    N = k_tree.shape[-2] - (1 if root_row else 0)
    lead = () if k_prefix.dim() == 4 else (n_layers,)
    if tuple(v_prefix.shape) != tuple(k_prefix.shape) or tuple(k_tree.shape) != lead + (B, H_kv, N + (1 if root_row else 0), d) or \
            tuple(v_tree.shape) != tuple(k_tree.shape):
        raise ValueError("cache shape mismatch")
    gamma_max = accepted_path.shape[1]
    for t, shp in [(n_accepted, (B,)), (accepted_path, (B, gamma_max)), (out_tokens, (B, gamma_max + 1)),
                   (prefix_len, (B,)), (next_root, (B,)), (flags, (B,))]:
        if tuple(t.shape) != shp:
            raise ValueError(f"shape mismatch: got {tuple(t.shape)}, expected {shp}")
    if k_prefix.dtype == torch.float32:
        dt = DTYPE_FP32
    elif k_prefix.dtype == torch.bfloat16:
        dt = DTYPE_BF16
    else:
        raise ValueError(f"unsupported dtype {k_prefix.dtype}")
    i32 = torch.int32
    desc = CommitDesc(C.sizeof(CommitDesc), B, N, H_kv, d, dt, L_stride, gamma_max, n_layers, 1 if root_row else 0)
    bufs = CommitBufs(C.sizeof(CommitBufs), _ptr(k_prefix, k_prefix.dtype, "k_prefix"),
                      _ptr(v_prefix, k_prefix.dtype, "v_prefix"), _ptr(k_tree, k_prefix.dtype, "k_tree"),
                      _ptr(v_tree, k_prefix.dtype, "v_tree"), _ptr(n_accepted, i32, "n_accepted"),
                      _ptr(accepted_path, i32, "accepted_path"), _ptr(out_tokens, i32, "out_tokens"),
                      _ptr(prefix_len, i32, "prefix_len"), _ptr(next_root, i32, "next_root"),
                      _ptr(flags, i32, "flags"))
    return CommitArgs(desc, bufs, (k_prefix, v_prefix, k_tree, v_tree, n_accepted, accepted_path, out_tokens,
                                   prefix_len, next_root, flags))


def mcsd_kv_commit(args: CommitArgs, stream=None) -> None:
    _check(lib().mcsd_kv_commit(C.byref(args.desc), C.byref(args.bufs), _stream(stream)))


def paged_commit_args(k_pool, v_pool, block_table, k_tree, v_tree, n_accepted, accepted_path, out_tokens, prefix_len,
                      next_root, flags, L_stride: int, root_row: bool = False):
    """Like commit_args with the destination in pools [n_layers][n_pages][H_kv][page_size][d] (or 4-D
    for one layer) and block_table int32 [B][max_pages_per_seq].  Returns (CommitArgs, PagedKV)."""
    if k_pool.dim() == 4:
        n_layers, (n_pages, H_kv, page_size, d) = 1, k_pool.shape
    else:
        n_layers, n_pages, H_kv, page_size, d = k_pool.shape
    B, N = k_tree.shape[-4], k_tree.shape[-2] - (1 if root_row else 0)
    gamma_max = accepted_path.shape[1]
    if k_pool.dtype == torch.float32:
        dt = DTYPE_FP32
    elif k_pool.dtype == torch.bfloat16:
        dt = DTYPE_BF16
    else:
        raise ValueError(f"unsupported dtype {k_pool.dtype}")
    if tuple(v_pool.shape) != tuple(k_pool.shape) or tuple(v_tree.shape) != tuple(k_tree.shape):
        raise ValueError("pool / tree shape mismatch")
    if block_table.dim() != 2 or block_table.shape[0] != B:
        raise ValueError("block_table must be [B][max_pages_per_seq]")
    i32 = torch.int32
    desc = CommitDesc(C.sizeof(CommitDesc), B, N, H_kv, d, dt, L_stride, gamma_max, n_layers, 1 if root_row else 0)
    bufs = CommitBufs(C.sizeof(CommitBufs), _ptr(k_pool, k_pool.dtype, "k_pool"), _ptr(v_pool, k_pool.dtype, "v_pool"),
                      _ptr(k_tree, k_pool.dtype, "k_tree"), _ptr(v_tree, k_pool.dtype, "v_tree"),
                      _ptr(n_accepted, i32, "n_accepted"), _ptr(accepted_path, i32, "accepted_path"),
                      _ptr(out_tokens, i32, "out_tokens"), _ptr(prefix_len, i32, "prefix_len"),
                      _ptr(next_root, i32, "next_root"), _ptr(flags, i32, "flags"))
    paged = PagedKV(C.sizeof(PagedKV), page_size, n_pages, block_table.shape[1], _ptr(block_table, i32, "block_table"))
    keep = (k_pool, v_pool, block_table, k_tree, v_tree, n_accepted, accepted_path, out_tokens, prefix_len, next_root, flags)
    return CommitArgs(desc, bufs, keep), paged


def mcsd_kv_commit_paged(args: CommitArgs, paged: PagedKV, stream=None) -> None:
    _check(lib().mcsd_kv_commit_paged(C.byref(args.desc), C.byref(args.bufs), C.byref(paged), _stream(stream)))


# ------------------------------------------------------------------- profiling aid
def mcsd_kernel_timing(enable: bool) -> None:
    _check(lib().mcsd_kernel_timing(1 if enable else 0))


def mcsd_kernel_timing_read() -> dict:
    """{kernel name: (total ms, launches)} since timing was enabled; waits for the events."""
    out = {}
    L = lib()
    for i in range(L.mcsd_kernel_count()):
        ms, n = C.c_double(0.0), C.c_int64(0)
        _check(L.mcsd_kernel_timing_read(i, C.byref(ms), C.byref(n)))
        out[L.mcsd_kernel_name(i).decode()] = (ms.value, n.value)
    return out
