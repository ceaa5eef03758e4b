"""Pins for the tree-attention oracle (Sec. 3.3 of the paper).

The oracle is checked against things that are not itself: textbook causal
attention run separately on every root-to-node candidate sequence (numpy, and
torch's CPU scaled_dot_product_attention as a third opinion), the closed form
at scale 0 (plain mean of the attended values, which exposes the mask), and
the standard grouped-query head mapping.
"""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import workloads as W


def small_inputs(kconfig=(2, 2), B=2, H_q=4, H_kv=2, d=16, prefix=(5, 9), dtype="fp32", seed=0,
                 L_stride=None):
    w = W.Workload("t", 90, B=B, H_q=H_q, H_kv=H_kv, d=d, dtype=dtype, prefix=prefix,
                   kconfig=kconfig, V=8, sigma_q=1.0, variant=0)
    return W.gen_attn_inputs(w, np.random.default_rng(seed), L_stride=L_stride)


def as_f64(a, dtype):
    return (a if dtype == "fp32" else W.bf16_bits_to_f32(a)).astype(np.float64)


def oracle_all(ai):
    return O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree,
                       ai.parent, ai.scale, O.FP32 if ai.dtype == "fp32" else O.BF16)


def path_of(parent, node):
    p = []
    while node >= 0:
        p.append(node); node = int(parent[node])
    return p[::-1]


def causal_attention(Q, K, Vv, scale):
    """Textbook causal attention of one head: Q, K, V [T][d]."""
    T = Q.shape[0]
    S = scale * Q @ K.T
    S = np.where(np.tril(np.ones((T, T), bool)), S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    Pm = np.exp(S)
    Pm /= Pm.sum(axis=1, keepdims=True)
    return Pm @ Vv


@pytest.mark.parametrize("kconfig", [(2, 2), (3, 2, 1), (1, 1, 1, 1), (4,)])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_equals_per_path_causal_attention(kconfig, dtype):
    """Each candidate sequence [prefix ; root-to-node path] run on its own through
    causal attention gives the same rows as the packed tree with the ancestor mask."""
    ai = small_inputs(kconfig=kconfig, dtype=dtype, seed=len(kconfig))
    out = oracle_all(ai)
    q, kp, vp = as_f64(ai.q, dtype), as_f64(ai.k_prefix, dtype), as_f64(ai.v_prefix, dtype)
    kt, vt = as_f64(ai.k_tree, dtype), as_f64(ai.v_tree, dtype)
    G = ai.H_q // ai.H_kv
    for b in range(ai.B):
        L = int(ai.prefix_len[b])
        for node in range(ai.N):
            path = path_of(ai.parent, node)
            for h in range(ai.H_q):
                g = h // G
                K = np.concatenate([kp[b, g, :L], kt[b, g, path]])
                Vv = np.concatenate([vp[b, g, :L], vt[b, g, path]])
                Q = np.concatenate([np.zeros((L, ai.d)), q[b, path, h]])
                ref = causal_attention(Q, K, Vv, ai.scale)
                # every node on the path is reproduced, not only the last one
                for t, a in enumerate(path):
                    np.testing.assert_allclose(out[b, a, h], ref[L + t], atol=1e-12, rtol=0)
                # third opinion: torch CPU SDPA, fp64
                tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (Q, K, Vv))
                tref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True,
                                                                        scale=ai.scale)[0, 0]
                np.testing.assert_allclose(out[b, node, h], tref[-1].numpy(), atol=1e-10, rtol=0)


def test_scale_zero_is_mean_over_visible_keys():
    """With scale 0 every visible key has the same weight, so the output is the
    mean of V over {prefix} U {ancestors} U {self}: a direct read-out of the mask."""
    ai = small_inputs(kconfig=(3, 2, 2), seed=5)
    out = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree,
                      ai.parent, 0.0, O.FP32)
    G = ai.H_q // ai.H_kv
    for b in range(ai.B):
        L = int(ai.prefix_len[b])
        for node in range(ai.N):
            path = path_of(ai.parent, node)
            for h in range(ai.H_q):
                g = h // G
                vis = np.concatenate([ai.v_prefix[b, g, :L], ai.v_tree[b, g, path]]).astype(np.float64)
                np.testing.assert_allclose(out[b, node, h], vis.mean(axis=0), atol=1e-13)


def test_siblings_do_not_see_each_other():
    """Changing the K/V of one candidate must not change rows outside its subtree."""
    ai = small_inputs(kconfig=(2, 2), seed=9)
    base = oracle_all(ai)
    kt = ai.k_tree.copy(); vt = ai.v_tree.copy()
    kt[:, :, 0] += 1.0; vt[:, :, 0] -= 2.0       # node 0: children are nodes 2, 3
    pert = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, kt, vt, ai.parent, ai.scale,
                       O.FP32)
    changed = np.abs(pert - base).max(axis=(0, 2, 3)) > 0
    assert changed.tolist() == [True, False, True, True, False, False]


def test_level1_node_is_single_token_decode_attention():
    """A child of the root sees the prefix and itself: ordinary decode attention
    over L+1 keys."""
    ai = small_inputs(kconfig=(4,), B=1, H_q=2, H_kv=2, seed=3)
    out = oracle_all(ai)
    L = int(ai.prefix_len[0])
    for node in range(4):
        for h in range(2):
            K = np.concatenate([ai.k_prefix[0, h, :L], ai.k_tree[0, h, node:node + 1]]).astype(np.float64)
            Vv = np.concatenate([ai.v_prefix[0, h, :L], ai.v_tree[0, h, node:node + 1]]).astype(np.float64)
            s = ai.scale * K @ ai.q[0, node, h].astype(np.float64)
            wgt = np.exp(s - s.max()); wgt /= wgt.sum()
            np.testing.assert_allclose(out[0, node, h], wgt @ Vv, atol=1e-13)


def test_gqa_head_mapping_and_padding_ignored():
    """Query head h uses KV head h // (H_q/H_kv); cache rows past prefix_len are never read."""
    ai = small_inputs(kconfig=(2, 1), B=2, H_q=6, H_kv=2, prefix=(3, 7), seed=2, L_stride=12)
    base = oracle_all(ai)
    kp, vp = ai.k_prefix.copy(), ai.v_prefix.copy()
    for b in range(ai.B):
        kp[b, :, ai.prefix_len[b]:] = np.nan
        vp[b, :, ai.prefix_len[b]:] = np.nan
    out = O.tree_attn(ai.q, kp, vp, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale, O.FP32)
    assert np.isfinite(out).all()
    np.testing.assert_array_equal(out, base)
    # expanding the KV heads to one per query head (the definition of GQA) changes nothing
    rep = lambda a: np.repeat(a, 3, axis=1)
    mha = O.tree_attn(ai.q, rep(ai.k_prefix), rep(ai.v_prefix), ai.prefix_len, rep(ai.k_tree),
                      rep(ai.v_tree), ai.parent, ai.scale, O.FP32)
    np.testing.assert_array_equal(mha, base)


def test_bf16_storage_is_read_exactly_and_selection_matches_full():
    ai = small_inputs(kconfig=(2, 2), dtype="bf16", seed=4)
    full = oracle_all(ai)
    f32 = lambda a: W.bf16_bits_to_f32(a)
    as32 = O.tree_attn(f32(ai.q), f32(ai.k_prefix), f32(ai.v_prefix), ai.prefix_len, f32(ai.k_tree),
                       f32(ai.v_tree), ai.parent, ai.scale, O.FP32)
    np.testing.assert_array_equal(full, as32)
    sel = np.array([[1, 5, 3], [0, 0, 0], [1, 2, 1]], np.int32)
    part = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree,
                       ai.parent, ai.scale, O.BF16, sel=sel, n_threads=2)
    for i, (b, n, h) in enumerate(sel):
        np.testing.assert_array_equal(part[i], full[b, n, h])


def test_bf16_rounding_helper():
    """Input generator's bf16 rounding is round-to-nearest-even (checked against torch)."""
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    np.testing.assert_array_equal(W.bf16_bits_to_f32(bits),
                                  torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_bad_tree_rejected():
    ai = small_inputs()
    bad = ai.parent.copy(); bad[1] = 3
    with pytest.raises(ValueError):
        O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, bad,
                    ai.scale, O.FP32)
