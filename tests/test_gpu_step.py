"""mcsd_verify_step (attention + verification on one stream) and the profiling aid."""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import binding as M
from paper_2401_06706_amd import device as D
from paper_2401_06706_amd import workloads as W
from tests.parity import assert_attn_close, compare_verify, run_oracle

pytestmark = pytest.mark.gpu


def test_verify_step_matches_separate_calls_and_oracle():
    w = W.WORKLOADS["c4"].with_(B=4, H_q=8, H_kv=8, prefix=(100, 700), V=8192, n_greedy=2)
    ai, vi = W.gen_attn_inputs(w), W.gen_verify_inputs(w)
    a1, v1 = D.make_attn_call(ai), D.make_verify_call(vi, want_residual=True)
    M.mcsd_verify_step(a1.args, v1.args)
    torch.cuda.synchronize()
    a2, v2 = D.make_attn_call(ai), D.make_verify_call(vi, want_residual=True)
    M.mcsd_tree_attn(a2.args)
    M.mcsd_verify_sample(v2.args)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a1.out_numpy(), a2.out_numpy())
    r1, r2 = v1.results(), v2.results()
    for k in r1:
        np.testing.assert_array_equal(r1[k], r2[k], err_msg=k)
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, n_threads=8)
    assert_attn_close(a1.out_numpy(), ref, "bf16", "step")
    compare_verify(vi, r1, run_oracle(vi, want_residual=True), check_residual=True, label="step")


@pytest.mark.parametrize("B", [1, 300])
def test_verify_step_with_unsplit_attention_equals_separate_calls(B):
    """Short prefixes: the attention is not split, so the step has no merge launch and the walk
    rides on the attention launch (more than 256 sequences: more than one row of walk blocks)."""
    w = W.WORKLOADS["c2"].with_(B=B, H_q=2, H_kv=2, prefix=(0, 90), V=512, kconfig=(3, 2, 1), n_greedy=B // 3)
    ai, vi = W.gen_attn_inputs(w), W.gen_verify_inputs(w)
    a1, v1 = D.make_attn_call(ai), D.make_verify_call(vi)
    M.mcsd_verify_step(a1.args, v1.args)
    torch.cuda.synchronize()
    a2, v2 = D.make_attn_call(ai), D.make_verify_call(vi)
    M.mcsd_tree_attn(a2.args)
    M.mcsd_verify_sample(v2.args)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a1.out_numpy(), a2.out_numpy())
    r1, r2 = v1.results(), v2.results()
    for k in r1:
        np.testing.assert_array_equal(r1[k], r2[k], err_msg=k)
    assert (r1["n_accepted"] >= 0).all()           # written by the walk (the buffers start at -7)
    compare_verify(vi, r1, run_oracle(vi), label=f"unsplit step B={B}")


def test_verify_step_rejects_bad_half_without_running_the_other():
    w = W.WORKLOADS["c1"]
    ai, vi = W.gen_attn_inputs(w), W.gen_verify_inputs(w)
    a, v = D.make_attn_call(ai), D.make_verify_call(vi)
    a.out.fill_(7.0)
    v.args.desc.variant = 9
    with pytest.raises(M.McsdError) as e:
        M.mcsd_verify_step(a.args, v.args)
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert (a.out == 7.0).all()           # nothing was enqueued


def test_kernel_timing_counts_launches():
    w = W.WORKLOADS["c2"].with_(prefix=(2048, 2048))
    ai, vi = W.gen_attn_inputs(w), W.gen_verify_inputs(w)
    a, v = D.make_attn_call(ai), D.make_verify_call(vi)
    M.mcsd_kernel_timing(True)
    for _ in range(3):
        M.mcsd_verify_step(a.args, v.args)
    t = M.mcsd_kernel_timing_read()
    M.mcsd_kernel_timing(False)
    assert t["tree_attn_mfma"][1] == 3 and t["verify_rows"][1] == 3
    # 65 tiles per head: the attention is split, so the merge of its partials and the walk go out
    # as one launch (the walk has none of its own)
    assert t["tree_attn_combine"][1] == 3 and t["walk"][1] == 0
    assert all(ms > 0 for ms, n in t.values() if n)
    M.mcsd_verify_step(a.args, v.args)             # timing off again: nothing recorded
    assert M.mcsd_kernel_timing_read()["verify_rows"][1] == 3
    # an attention that is not split has no merge launch; the walk then rides on the attention launch
    w1 = W.WORKLOADS["c2"].with_(prefix=(64, 64))
    a1, v1 = D.make_attn_call(W.gen_attn_inputs(w1)), D.make_verify_call(W.gen_verify_inputs(w1))
    M.mcsd_kernel_timing(True)
    M.mcsd_verify_step(a1.args, v1.args)
    t1 = M.mcsd_kernel_timing_read()
    M.mcsd_kernel_timing(False)
    assert t1["walk"][1] == 0 and t1["tree_attn_combine"][1] == 0
    assert t1["tree_attn_mfma"][1] == 1 and t1["verify_rows"][1] == 1
    # the fp32 path (no matrix-core kernel) keeps the walk launch of its own
    w2 = W.WORKLOADS["c1"]
    a2, v2 = D.make_attn_call(W.gen_attn_inputs(w2)), D.make_verify_call(W.gen_verify_inputs(w2))
    M.mcsd_kernel_timing(True)
    M.mcsd_verify_step(a2.args, v2.args)
    t2 = M.mcsd_kernel_timing_read()
    M.mcsd_kernel_timing(False)
    assert t2["walk"][1] == 1 and t2["tree_attn_generic"][1] == 1


def test_long_prefix_sampled_against_oracle():
    """32768-token prefix (more than any bench workload), GQA 16/2: sampled rows."""
    w = W.WORKLOADS["c5"].with_(B=1, H_q=16, H_kv=2, prefix=(32768, 32768), kconfig=(4, 2))
    ai = W.gen_attn_inputs(w)
    call = D.make_attn_call(ai)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    got = call.out_numpy()
    sel = np.array([[0, 0, 0], [0, 11, 15], [0, 5, 7], [0, 3, 8]], np.int32)
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, sel=sel, n_threads=4)
    assert_attn_close(got[sel[:, 0], sel[:, 1], sel[:, 2]], ref, "bf16", "32768-token prefix (sampled rows)")


def test_step_can_be_captured_in_a_hip_graph_and_replayed():
    """The library only enqueues kernels (no allocation, no memset, no synchronisation), so a step
    can be captured; every replay, with eager work and synchronisations in between, reproduces
    the eager results."""
    w = W.WORKLOADS["c3"].with_(B=2, prefix=(1500, 2048))
    ai, vi = W.gen_attn_inputs(w), W.gen_verify_inputs(w)
    a, v = D.make_attn_call(ai), D.make_verify_call(vi)
    M.mcsd_verify_step(a.args, v.args)
    torch.cuda.synchronize()
    ref_out = a.out.clone()
    ref = {k: x.copy() for k, x in v.results().items()}
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        M.mcsd_verify_step(a.args, v.args, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    other = D.make_verify_call(W.gen_verify_inputs(W.WORKLOADS["c2"]))
    for rep in range(4):
        a.out.fill_(7.0)
        for name in ("n_accepted", "accepted_path", "out_tokens", "acc_child", "endpoint", "flags"):
            v.tensors[name].fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        M.mcsd_verify_sample(other.args)            # eager work of the program between replays
        torch.cuda.synchronize()
        assert torch.equal(a.out.view(torch.int16), ref_out.view(torch.int16)), rep
        got = v.results()
        for k in ("n_accepted", "accepted_path", "out_tokens", "acc_child", "endpoint", "flags"):
            np.testing.assert_array_equal(got[k], ref[k], err_msg=f"{k} replay {rep}")


def test_million_token_prefix_sampled_against_oracle():
    """One sequence with a 1,000,003-token prefix (256 MB of K per head): offsets far beyond the
    bench workloads, hundreds of segments per unit, a ragged last prefix tile."""
    w = W.WORKLOADS["c2"].with_(B=1, H_q=2, H_kv=1, prefix=(1000003, 1000003), kconfig=(3, 2))
    ai = W.gen_attn_inputs(w)
    call = D.make_attn_call(ai)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    got = call.out_numpy()
    sel = np.array([[0, 0, 0], [0, 8, 1], [0, 4, 0]], np.int32)
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, sel=sel, n_threads=3)
    assert_attn_close(got[sel[:, 0], sel[:, 1], sel[:, 2]], ref, "bf16", "1000003-token prefix (sampled rows)")
    assert np.isfinite(got).all()
