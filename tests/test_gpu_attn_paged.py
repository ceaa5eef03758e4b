"""mcsd_tree_attn_paged: the prefix cache in a page pool.  Same arithmetic as the contiguous
call (bit-identical outputs), and the oracle on the cache gathered back from the pool."""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import binding as M
from paper_2401_06706_amd import device as D
from paper_2401_06706_amd import workloads as W
from tests.parity import assert_attn_close

pytestmark = pytest.mark.gpu


def run_both(ai, page_size, seed=0):
    tree = D.make_attn_call(ai)
    paged_call, paged, table = D.make_paged_attn_call(tree, ai, page_size, seed=seed)
    M.mcsd_tree_attn(tree.args)
    M.mcsd_tree_attn_paged(paged_call.args, paged)
    torch.cuda.synchronize()
    return tree, paged_call, table


@pytest.mark.parametrize("name,page_size", [("c2", 32), ("c2", 128), ("c3", 64), ("c3", 256), ("c5", 4096), ("c1", 32)])
def test_paged_equals_contiguous_bit_for_bit(name, page_size):
    w = W.WORKLOADS[name]
    if name == "c5":
        w = w.with_(B=2, prefix=(3000, 5000))
    ai = W.gen_attn_inputs(w)
    tree, paged_call, _ = run_both(ai, page_size)
    a, b = tree.out, paged_call.out
    assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                       b.view(torch.int16) if b.dtype == torch.bfloat16 else b)


def test_paged_batched_ragged_against_oracle_on_gathered_cache():
    w = W.WORKLOADS["c4"].with_(B=6, H_q=8, H_kv=4, prefix=(1, 700))
    ai = W.gen_attn_inputs(w, L_stride=704)
    tree, paged_call, table = run_both(ai, 64, seed=5)
    assert torch.equal(tree.out.view(torch.int16), paged_call.out.view(torch.int16))
    # oracle on the cache gathered from the pool by the layout's definition
    kpool = paged_call.tensors["k_pool"].view(torch.int16).cpu().numpy().view(np.uint16)
    vpool = paged_call.tensors["v_pool"].view(torch.int16).cpu().numpy().view(np.uint16)
    kc, vc = O.gather_pages(kpool, table, ai.L_stride), O.gather_pages(vpool, table, ai.L_stride)
    # rows below prefix_len are what the cache held (rows above it are never read)
    for b in range(ai.B):
        L = int(ai.prefix_len[b])
        np.testing.assert_array_equal(kc[b, :, :L], ai.k_prefix[b, :, :L])
    ref = O.tree_attn(ai.q, kc, vc, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale, O.BF16, n_threads=8)
    assert_attn_close(paged_call.out_numpy(), ref, "bf16", "paged")


@pytest.mark.parametrize("page_size", [32, 96, 256])
def test_paged_many_rows_per_kv_head_against_oracle(page_size):
    """224 query rows per KV head (the kernel whose waves share each K/V tile and look the block
    table up one step ahead), ragged prefixes, pages of one tile, three tiles (not a power of two)
    and eight tiles; several segments per sequence and one."""
    w = W.WORKLOADS["c4"].with_(B=3, H_q=16, H_kv=2, kconfig=(4, 2, 2), prefix=(5, 1500))
    ai = W.gen_attn_inputs(w, np.random.default_rng(page_size), L_stride=1536)
    tree, paged_call, table = run_both(ai, page_size, seed=page_size)
    assert torch.equal(tree.out.view(torch.int16), paged_call.out.view(torch.int16))
    kpool = paged_call.tensors["k_pool"].view(torch.int16).cpu().numpy().view(np.uint16)
    vpool = paged_call.tensors["v_pool"].view(torch.int16).cpu().numpy().view(np.uint16)
    kc, vc = O.gather_pages(kpool, table, ai.L_stride), O.gather_pages(vpool, table, ai.L_stride)
    ref = O.tree_attn(ai.q, kc, vc, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale, O.BF16, n_threads=8)
    assert_attn_close(paged_call.out_numpy(), ref, "bf16", "paged")


def test_pages_that_hold_no_valid_rows_are_never_read():
    # prefix 40 of capacity 256 with 32-token pages: only pages 0 and 1 of each sequence matter;
    # the other table entries point far outside the pool
    w = W.WORKLOADS["c2"].with_(B=2, H_q=4, H_kv=4, prefix=(40, 40))
    ai = W.gen_attn_inputs(w, L_stride=256)
    tree = D.make_attn_call(ai)
    paged_call, paged, table = D.make_paged_attn_call(tree, ai, 32)
    bad = table.copy()
    bad[:, 2:] = 2 ** 30
    paged_call.tensors["block_table"].copy_(torch.from_numpy(bad))
    M.mcsd_tree_attn(tree.args)
    M.mcsd_tree_attn_paged(paged_call.args, paged)
    torch.cuda.synchronize()
    assert torch.equal(tree.out.view(torch.int16), paged_call.out.view(torch.int16))


def test_table_entry_outside_the_pool_reads_as_zero_keys():
    # an entry of a page in use that lies outside the pool: handled inside the kernel (zeros), no fault
    w = W.WORKLOADS["c2"].with_(B=1, H_q=4, H_kv=4, prefix=(96, 96))
    ai = W.gen_attn_inputs(w, L_stride=96)
    tree = D.make_attn_call(ai)
    paged_call, paged, table = D.make_paged_attn_call(tree, ai, 32)
    bad = table.copy()
    bad[0, 1] = -5
    paged_call.tensors["block_table"].copy_(torch.from_numpy(bad))
    M.mcsd_tree_attn_paged(paged_call.args, paged)
    torch.cuda.synchronize()
    kz, vz = ai.k_prefix.copy(), ai.v_prefix.copy()
    kz[:, :, 32:64] = 0
    vz[:, :, 32:64] = 0
    ref = O.tree_attn(ai.q, kz, vz, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale, O.BF16, n_threads=4)
    assert_attn_close(paged_call.out_numpy(), ref, "bf16", "paged")
