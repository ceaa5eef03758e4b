"""Randomly drawn (seeded) shapes within the documented limits: tree attention (contiguous and
paged) and verification against the oracle, and the fused step against the separate calls.  The draws cover what the hand-picked cases may
miss: odd head ratios, trees of every size, prefixes around tile and page edges, every kernel
variant the launch plan picks by itself."""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import binding as M
from paper_2401_06706_amd import device as D
from paper_2401_06706_amd import workloads as W
from tests.parity import assert_attn_close, compare_verify, run_oracle

pytestmark = pytest.mark.gpu


def draw_workload(rng):
    depth = int(rng.integers(1, 5))
    kconfig = tuple(int(rng.integers(1, 5)) for _ in range(depth))
    def n_nodes(kc):
        total, level = 0, 1
        for k in kc:
            level *= k
            total += level
        return total
    while n_nodes(kconfig) > 128:
        kconfig = kconfig[:-1]
    H_kv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 1, 2, 3, 4, 8]))
    B = int(rng.integers(1, 6))
    hi = int(rng.choice([40, 130, 700, 2100]))
    lo = int(rng.integers(0, hi + 1))
    V = int(rng.choice([17, 1000, 4096, 5000, 20000]))
    return W.Workload(name="t", index=60, B=B, H_q=H_kv * G, H_kv=H_kv, d=128, dtype="bf16", prefix=(lo, hi),
                      kconfig=kconfig, V=V, sigma_q=float(rng.choice([0.5, 1.0, 2.0])),
                      variant=int(rng.integers(0, 2)), n_greedy=int(rng.integers(0, B + 1)))


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_shape(seed):
    rng = np.random.default_rng(7000 + seed)
    w = draw_workload(rng)
    L_stride = w.prefix[1] + int(rng.integers(0, 40))
    ai = W.gen_attn_inputs(w, np.random.default_rng(seed), L_stride=L_stride)
    print(f"[random] seed {seed}: B={w.B} H={w.H_q}/{w.H_kv} k={w.kconfig} N={ai.N} L={ai.prefix_len.tolist()} "
          f"L_stride={L_stride} V={w.V} variant={w.variant} greedy={w.n_greedy}", flush=True)
    nan16 = np.uint16(0x7FC0)
    for b in range(ai.B):
        ai.k_prefix[b, :, ai.prefix_len[b]:] = nan16
        ai.v_prefix[b, :, ai.prefix_len[b]:] = nan16
    call = D.make_attn_call(ai)
    M.mcsd_tree_attn(call.args)
    torch.cuda.synchronize()
    got = call.out_numpy()
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, n_threads=8)
    assert_attn_close(got, ref, "bf16", f"random {seed}")
    # the same problem over a page pool: bit-identical to the contiguous call
    page_size = int(rng.choice([32, 64, 96, 256]))
    paged_call, paged, _ = D.make_paged_attn_call(call, ai, page_size, seed=seed)
    M.mcsd_tree_attn_paged(paged_call.args, paged)
    torch.cuda.synchronize()
    assert torch.equal(call.out.view(torch.int16), paged_call.out.view(torch.int16)), f"page_size {page_size}"
    # verification on the same tree
    vi = W.gen_verify_inputs(w, np.random.default_rng(100 + seed))
    vcall = D.make_verify_call(vi, want_ratio=True)
    M.mcsd_verify_sample(vcall.args)
    torch.cuda.synchronize()
    compare_verify(vi, vcall.results(), run_oracle(vi), label=f"random {seed}")
    # the fused step (whichever launch carries the walk for this shape) gives the same bits
    a2, v2 = D.make_attn_call(ai), D.make_verify_call(vi, want_ratio=True)
    M.mcsd_verify_step(a2.args, v2.args)
    torch.cuda.synchronize()
    assert torch.equal(call.out.view(torch.int16), a2.out.view(torch.int16))
    r1, r2 = vcall.results(), v2.results()
    for k in r1:
        np.testing.assert_array_equal(r1[k], r2[k], err_msg=f"step vs separate calls: {k}")
