"""GPU parity of mcsd_tree_attn (through the C ABI) against the CPU oracle.

Every comparison goes through tests.parity.assert_attn_close: the stated absolute tolerance
(2e-2 for bf16 storage, 1e-5 for fp32) AND a bar scaled to the reference (largest error against
max|ref|, RMS error against RMS(ref)), because long-prefix outputs are far smaller than 2e-2.
The five named workloads are compared in full, every row of every sequence and head.
"""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import binding as M
from paper_2401_06706_amd import device as D
from paper_2401_06706_amd import workloads as W
from tests.parity import ATTN_REL, assert_attn_close

pytestmark = pytest.mark.gpu


def oracle_rows(ai, sel=None):
    return O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent,
                       ai.scale, O.FP32 if ai.dtype == "fp32" else O.BF16, sel=sel, n_threads=16)


def run_gpu(ai, parent_per_seq=False):
    call = D.make_attn_call(ai, parent_per_seq=parent_per_seq)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    return call.out_numpy()


def check_full(ai, label, parent_per_seq=False):
    print(f"[attn] {label}: B={ai.B} N={ai.N} H={ai.H_q}/{ai.H_kv} d={ai.d} {ai.dtype} L={ai.prefix_len.tolist()[:8]}",
          flush=True)
    got = run_gpu(ai, parent_per_seq)
    ref = oracle_rows(ai)
    assert_attn_close(got, ref, ai.dtype, label)
    return got, ref


def wl(**kw):
    base = dict(name="t", index=50, B=2, H_q=4, H_kv=4, d=128, dtype="bf16", prefix=(100, 100),
                kconfig=(4, 2, 2), V=8, sigma_q=1.0, variant=0)
    base.update(kw)
    return W.Workload(**base)


def test_c1_tiny_fp32():
    check_full(W.gen_attn_inputs(W.WORKLOADS["c1"]), "c1")


def test_c2_full():
    check_full(W.gen_attn_inputs(W.WORKLOADS["c2"]), "c2")


def test_c3_full():
    check_full(W.gen_attn_inputs(W.WORKLOADS["c3"]), "c3")


def test_c4_full_ragged_batch():
    """All 16 x 60 x 32 rows of the batched workload (the launch configuration the bench times)."""
    ai = W.gen_attn_inputs(W.WORKLOADS["c4"])
    got, _ = check_full(ai, "c4")
    # property that holds at any size: every output is a convex combination of V rows
    vmax = max(np.abs(W.bf16_bits_to_f32(ai.v_prefix)).max(), np.abs(W.bf16_bits_to_f32(ai.v_tree)).max())
    assert np.abs(got).max() <= vmax * 1.01


def test_c5_full_gqa_long_prefix():
    """All 4 x 84 x 64 rows at the 16384-token prefix: every row tile, wave and key segment."""
    check_full(W.gen_attn_inputs(W.WORKLOADS["c5"]), "c5")


@pytest.mark.parametrize("L", [0, 1, 31, 32, 33, 63, 64, 65, 127, 129, 300])
def test_prefix_lengths_around_tile_edges(L):
    ai = W.gen_attn_inputs(wl(prefix=(L, L), B=1, H_q=2, H_kv=2), np.random.default_rng(L), L_stride=max(L, 1))
    check_full(ai, f"L={L}")


@pytest.mark.parametrize("kconfig", [(1,), (2,), (1, 1, 1, 1), (33,), (16, 2, 2), (2, 2, 2, 2, 2, 2), (128,)])
def test_tree_shapes(kconfig):
    """1 node, chains, a level wider than one key tile, 126- and 128-node trees."""
    ai = W.gen_attn_inputs(wl(kconfig=kconfig, prefix=(70, 70), B=1, H_q=2, H_kv=2), np.random.default_rng(7))
    check_full(ai, f"k={kconfig}")


@pytest.mark.parametrize("H_q,H_kv,kconfig", [(8, 2, (4, 2)), (8, 1, (4, 2, 2)), (16, 2, (3, 2)), (6, 2, (5, 2, 1))])
def test_gqa_row_tiles(H_q, H_kv, kconfig):
    """Rows per KV head of 48, 224 (several row tiles, ragged last tile), 72, 45."""
    ai = W.gen_attn_inputs(wl(H_q=H_q, H_kv=H_kv, kconfig=kconfig, prefix=(40, 200), B=2), np.random.default_rng(H_q))
    check_full(ai, f"gqa {H_q}/{H_kv} {kconfig}")


def test_ragged_batch_with_padding_rows_poisoned():
    """Cache rows past prefix_len hold NaN: they must never reach the output."""
    ai = W.gen_attn_inputs(wl(prefix=(1, 260), B=6, H_q=4, H_kv=2), np.random.default_rng(11), L_stride=300)
    nan16 = np.uint16(0x7FC0)
    for b in range(ai.B):
        ai.k_prefix[b, :, ai.prefix_len[b]:] = nan16
        ai.v_prefix[b, :, ai.prefix_len[b]:] = nan16
    check_full(ai, "poisoned padding")


def test_split_factors_agree(plan_override):
    """Different segment lengths give the same result within tolerance; one segment per unit
    (direct write) and many (partials merged by the segment that arrives last)."""
    ai = W.gen_attn_inputs(wl(prefix=(1000, 1500), B=2, H_q=4, H_kv=4), np.random.default_rng(13), L_stride=1500)
    ref = oracle_rows(ai)
    outs = []
    for chunk in (4, 8, 20, 1000):
        plan_override(0, chunk, 0)
        got = run_gpu(ai)
        assert_attn_close(got, ref, "bf16", f"chunk_tiles={chunk}")
        outs.append(got)
    assert_attn_close(outs[0], outs[-1], "bf16", "4-tile segments against one segment")


@pytest.mark.parametrize("variant", [1, 2, 3])
@pytest.mark.parametrize("H_q,H_kv,kconfig", [(2, 2, (3, 2)), (8, 2, (4, 2)), (8, 1, (4, 2, 2)), (32, 4, (4, 2, 2))])
def test_every_kernel_variant_on_every_row_count(plan_override, variant, H_q, H_kv, kconfig):
    """The three matrix-core kernels (32 rows x 4 key streams, 64 x 2, 128 rows sharing one key
    stream) forced in turn on 9, 48, 224 and 224 rows per KV head: fewer rows than one wave's
    share, ragged last row tiles, several row tiles; ragged prefixes with poisoned padding,
    one segment per unit and several; an empty prefix (tree keys only) among them."""
    ai = W.gen_attn_inputs(wl(H_q=H_q, H_kv=H_kv, kconfig=kconfig, prefix=(3, 700), B=3), np.random.default_rng(100 + H_q),
                           L_stride=720)
    ai.prefix_len[:] = [0, 33, 700]         # no prefix at all, one tile and one key, many tiles
    nan16 = np.uint16(0x7FC0)
    for b in range(ai.B):
        ai.k_prefix[b, :, ai.prefix_len[b]:] = nan16
        ai.v_prefix[b, :, ai.prefix_len[b]:] = nan16
    ref = oracle_rows(ai)
    for chunk in (6, 1000):
        plan_override(variant, chunk, 0)
        got = run_gpu(ai)
        assert_attn_close(got, ref, "bf16", f"variant {variant} chunk_tiles={chunk}")


def test_parent_per_sequence_and_determinism():
    ai = W.gen_attn_inputs(wl(prefix=(50, 90), B=3), np.random.default_rng(17))
    a, _ = check_full(ai, "shared parent")
    b, _ = check_full(ai, "per-seq parent", parent_per_seq=True)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a, run_gpu(ai))


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (256, "bf16"), (128, "fp32"), (8, "fp32"), (96, "fp32")])
def test_generic_kernel_shapes(d, dtype):
    ai = W.gen_attn_inputs(wl(d=d, dtype=dtype, prefix=(5, 300), B=2, H_q=4, H_kv=2, kconfig=(3, 2)),
                           np.random.default_rng(d))
    check_full(ai, f"generic d={d} {dtype}")


def test_scale_zero_gives_mean_of_visible_values():
    ai = W.gen_attn_inputs(wl(prefix=(64, 64), B=1, H_q=2, H_kv=2, kconfig=(2, 2)), np.random.default_rng(19))
    ai.scale = 0.0
    got, ref = check_full(ai, "scale 0")


def test_workspace_too_small_is_an_error():
    ai = W.gen_attn_inputs(wl(prefix=(2000, 2000), B=1))
    call = D.make_attn_call(ai)
    assert call.args.bufs.workspace_bytes > 256
    call.args.bufs.workspace_bytes = 256
    with pytest.raises(M.McsdError) as e:
        M.mcsd_tree_attn(call.args)
    assert e.value.code == -5


@pytest.mark.parametrize("name", ["c1", "c2", "c3"])
def test_tree_attention_equals_replicated_candidate_sequences(name):
    """Without tree attention every candidate sequence carries its own copy of the prefix cache
    (Sec. 3.3); the outputs are the same, node by node."""
    w = W.WORKLOADS[name]
    ai = W.gen_attn_inputs(w)
    tree = D.make_attn_call(ai)
    rep = D.make_replicated_attn_call(tree, ai)
    M.mcsd_tree_attn(tree.args)
    M.mcsd_tree_attn(rep.args)
    torch.cuda.synchronize()
    a = tree.out.float().cpu().numpy()                                   # [B][N][H][d]
    r = rep.out.float().cpu().numpy()                                    # [B*leaves][depth][H][d]
    n_leaves = len(rep.paths)
    for b in range(ai.B):
        for li, path in enumerate(rep.paths):
            got = r[b * n_leaves + li]
            want = a[b, path]
            # both sides are rounded outputs of the same kernel: twice the bar against the oracle
            assert np.abs(got - want).max() <= 2 * ATTN_REL[ai.dtype] * np.abs(want).max(), (b, li)


def test_many_short_sequences():
    """300 sequences (more (sequence, segment) pairs than a workgroup ranks: plain dispatch order)."""
    w = W.WORKLOADS["c2"].with_(B=300, H_q=4, H_kv=2, prefix=(0, 700), kconfig=(3, 2))
    ai = W.gen_attn_inputs(w)
    call = D.make_attn_call(ai)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    got = call.out_numpy()
    rng = np.random.default_rng(4)
    sel = np.stack([rng.integers(0, ai.B, 200), rng.integers(0, ai.N, 200), rng.integers(0, ai.H_q, 200)], axis=1).astype(np.int32)
    sel[0, 0] = int(np.argmin(ai.prefix_len)); sel[1, 0] = int(np.argmax(ai.prefix_len))
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, sel=sel, n_threads=16)
    assert_attn_close(got[sel[:, 0], sel[:, 1], sel[:, 2]], ref, "bf16", "300 sequences (sampled rows)")


@pytest.mark.parametrize("H_q,H_kv,kconfig,target", [(16, 8, (4, 2, 2), 4096), (24, 3, (4, 2, 2), 2048), (16, 16, (4, 2), 3000)])
def test_thousands_of_short_segments(plan_override, H_q, H_kv, kconfig, target):
    """Far more workgroups than the chip holds at once, every unit cut into many short segments
    (the minimum run length), an empty prefix and a full one among them; the result is the same
    bits on every run."""
    plan_override(0, 0, target)
    ai = W.gen_attn_inputs(wl(H_q=H_q, H_kv=H_kv, kconfig=kconfig, prefix=(200, 3000), B=7), np.random.default_rng(H_q),
                           L_stride=3000)
    ai.prefix_len[0] = 0
    ai.prefix_len[1] = 3000
    ref = oracle_rows(ai)
    call = D.make_attn_call(ai)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    first = call.out.clone()
    assert_attn_close(call.out_numpy(), ref, "bf16", f"pull {H_q}/{H_kv} target {target}")
    for rep in range(3):
        call.out.fill_(7.0)
        M.mcsd_tree_attn(call.args)
        torch.cuda.synchronize()
        assert torch.equal(call.out.view(torch.int16), first.view(torch.int16)), rep


@pytest.mark.parametrize("H_q,H_kv,kconfig", [(4, 4, (4, 2, 2)), (8, 4, (4, 2, 2)), (32, 4, (4, 2, 2))])
def test_long_unsplit_prefix_is_the_same_bits_on_every_run(plan_override, H_q, H_kv, kconfig):
    """One long segment per sequence: nearly every tile goes through the straight-line step, in
    which the running-maximum update stands close behind the score matrix instructions.  Scores
    that grow along the prefix make that update fire many times; a maximum read before the
    matrix result has landed would move the raises around from run to run (the outputs stay
    within tolerance then, so only the bit comparison sees it).  One case per kernel variant."""
    plan_override(0, 400, 0)
    ai = W.gen_attn_inputs(wl(H_q=H_q, H_kv=H_kv, kconfig=kconfig, prefix=(3000, 4096), B=3), np.random.default_rng(90 + H_q),
                           L_stride=4096)
    # keys later in the prefix score higher: K rows scaled by a ramp (bf16 bits rewritten)
    k = W.bf16_bits_to_f32(ai.k_prefix)
    ramp = np.linspace(0.2, 3.0, k.shape[2], dtype=np.float32)[None, None, :, None]
    ai.k_prefix = W.f32_to_bf16_bits(k * ramp)
    ref = oracle_rows(ai)
    call = D.make_attn_call(ai)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    first = call.out.clone()
    assert_attn_close(call.out_numpy(), ref, "bf16", f"ramp {H_q}/{H_kv}")
    for rep in range(4):
        call.out.fill_(3.0)
        M.mcsd_tree_attn(call.args)
        torch.cuda.synchronize()
        assert torch.equal(call.out.view(torch.int16), first.view(torch.int16)), rep


def test_plan_override_rejects_bad_values():
    with pytest.raises(M.McsdError):
        M.mcsd_attn_plan_override(4, 0, 0)
    with pytest.raises(M.McsdError):
        M.mcsd_attn_plan_override(0, -1, 0)
    M.mcsd_attn_plan_override(0, 0, 0)


def add_root_rows(ai, rng):
    """The same problem with the root as row 0 of the tree block (q, k_tree, v_tree get one more row)."""
    def one_more(a, axis):
        shape = list(a.shape)
        shape[axis] = 1
        if ai.dtype == "bf16":
            extra = W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
        else:
            extra = rng.standard_normal(shape).astype(np.float32)
        return np.ascontiguousarray(np.concatenate([extra, a], axis=axis))
    return one_more(ai.q, 1), one_more(ai.k_tree, 2), one_more(ai.v_tree, 2)


@pytest.mark.parametrize("H_q,H_kv,kconfig,prefix", [(4, 4, (4, 2, 2), (100, 300)), (8, 1, (4, 2, 2), (0, 900)),
                                                     (2, 2, (127,), (40, 40)), (6, 2, (3, 2, 1), (2000, 2100)), (2, 2, (2, 2), (5, 9))])
def test_root_row(H_q, H_kv, kconfig, prefix):
    """root_row = 1: the root is row 0 of the tree block and every candidate's ancestor.  Equal, bit
    for bit, to the same tree written out with the root as an ordinary node 0, and to the oracle
    on that tree; 128 rows (127 candidates) is the largest tree block."""
    rng = np.random.default_rng(H_q * 100 + len(kconfig))
    dtype = "fp32" if kconfig == (2, 2) else "bf16"
    ai = W.gen_attn_inputs(wl(H_q=H_q, H_kv=H_kv, kconfig=kconfig, prefix=prefix, B=3, dtype=dtype, d=128), rng,
                           L_stride=prefix[1])
    q, kt, vt = add_root_rows(ai, rng)
    parent_ext = np.concatenate([[-1], ai.parent.astype(np.int64) + 1]).astype(np.int32)
    ref = O.tree_attn(q, ai.k_prefix, ai.v_prefix, ai.prefix_len, kt, vt, parent_ext, ai.scale,
                      O.FP32 if dtype == "fp32" else O.BF16, n_threads=16)
    base = D.make_attn_call(ai)
    t = base.tensors
    to_dev = lambda a: D._to_device(a, dtype, "cuda:0")
    tq, tkt, tvt = to_dev(q), to_dev(kt), to_dev(vt)
    outs = []
    for parent in (ai.parent.astype(np.int32), parent_ext):           # root row / root as node 0
        out = torch.full_like(tq, 7.0)
        tp = torch.from_numpy(parent).to("cuda:0")
        desc_probe = M.attn_args(tq, t["k_prefix"], t["v_prefix"], t["prefix_len"], tkt, tvt, tp, out, ai.scale).desc
        ws = torch.empty(max(M.mcsd_attn_workspace_bytes(desc_probe), 256), dtype=torch.uint8, device="cuda:0")
        args = M.attn_args(tq, t["k_prefix"], t["v_prefix"], t["prefix_len"], tkt, tvt, tp, out, ai.scale, workspace=ws)
        assert args.desc.root_row == (1 if parent is not parent_ext else 0) and args.desc.N + args.desc.root_row == ai.N + 1
        M.mcsd_tree_attn(args)
        torch.cuda.synchronize()
        outs.append(out)
    assert torch.equal(outs[0].view(torch.int16) if dtype == "bf16" else outs[0], outs[1].view(torch.int16) if dtype == "bf16" else outs[1])
    assert_attn_close(outs[0].float().cpu().numpy().astype(np.float64), ref, dtype, f"root row {kconfig} {H_q}/{H_kv}")
