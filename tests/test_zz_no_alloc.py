"""mcsd_tree_attn_static: the attention entry point that allocates nothing (its split partials go
to a static device buffer inside the library).  Through the C ABI, against mcsd_tree_attn with a
caller workspace (bit for bit: same kernels, same launch plan) and against the oracle, on calls
made one after the other on the same GPU, the later ones with smaller inputs, so that whatever
an earlier call left in the shared buffer must not matter."""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import binding as M
from paper_2401_06706_amd import device as D
from paper_2401_06706_amd import workloads as W
from tests.parity import assert_attn_close

pytestmark = pytest.mark.gpu


def static_call_like(call):
    """The same device tensors with a fresh output and NO workspace."""
    t = call.tensors
    out = torch.full_like(t["out"], 7.0)
    args = M.attn_args(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_len"], t["k_tree"], t["v_tree"], t["parent"],
                       out, call.args.desc.scale, workspace=None)
    assert args.bufs.workspace is None and args.bufs.workspace_bytes == 0
    return args, out


def run_pair(w, label, L_stride=None):
    ai = W.gen_attn_inputs(w, L_stride=L_stride)
    call = D.make_attn_call(ai)
    need = M.mcsd_attn_workspace_bytes(call.args.desc)
    print(f"[no-alloc] {label}: B={ai.B} N={ai.N} H={ai.H_q}/{ai.H_kv} L={ai.prefix_len.tolist()[:6]} partials {need} B", flush=True)
    assert 0 < need <= M.STATIC_SCRATCH_BYTES, "the case must use the scratch buffer"
    M.mcsd_tree_attn(call.args)
    args, out = static_call_like(call)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    M.mcsd_tree_attn_static(args)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out.view(torch.int16), call.out.view(torch.int16)), f"{label}: differs from mcsd_tree_attn"
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, n_threads=16)
    got = out.to(torch.float32).cpu().numpy().astype(np.float64)
    assert_attn_close(got, ref, "bf16", f"no-alloc {label}")
    return args, out, call


def test_static_scratch_two_calls_in_a_row_second_one_smaller():
    big = W.WORKLOADS["c3"]                                           # 40 heads, prefix 2048: 5 segments per head
    small = W.WORKLOADS["c2"].with_(H_q=8, H_kv=4, prefix=(900, 1300), B=2, kconfig=(3, 2))
    a1, o1, c1 = run_pair(big, "first call (c3)")
    a2, o2, c2 = run_pair(small, "second call (smaller)", L_stride=1300)
    # and the first input once more, after the smaller call has left its partials in the buffer
    o1.fill_(7.0)
    M.mcsd_tree_attn_static(a1)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), c1.out.view(torch.int16))


def test_static_scratch_unsplit_shape_and_fp32_path_need_no_scratch():
    """Shapes without partials go through the same entry point (the buffer is simply unused)."""
    for name in ("c1", "c2"):
        w = W.WORKLOADS[name] if name == "c1" else W.WORKLOADS[name].with_(prefix=(64, 64))
        ai = W.gen_attn_inputs(w)
        call = D.make_attn_call(ai)
        M.mcsd_tree_attn(call.args)
        args, out = static_call_like(call)
        M.mcsd_tree_attn_static(args)
        torch.cuda.synchronize()
        assert torch.equal(out, call.out)
