"""Pins for the oracle's candidate-tree builder (Sec. 3 / 4.3 / 3.3) and KV commit (Sec. 3.3)."""
from collections import deque

import numpy as np
import pytest

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import workloads as W


def _queue_tree(kconfig):
    """Independent construction: breadth-first expansion with a queue of (node, depth)."""
    parent, depth = [], []
    q = deque([(-1, 0)])
    while q:
        node, dep = q.popleft()
        if dep == len(kconfig):
            continue
        for _ in range(kconfig[dep]):
            parent.append(node)
            depth.append(dep + 1)
            q.append((len(parent) - 1, dep + 1))
    return np.array(parent, np.int32), np.array(depth, np.int32)


@pytest.mark.parametrize("kconfig", [(1,), (4,), (2, 2), (4, 2, 2), (8, 2, 1, 1), (4, 2, 2, 1, 1), (4, 4, 2, 1),
                                     (1, 1, 1, 1, 1, 1), (2, 3, 4), (3, 1, 5, 2), (128,)])
def test_tree_build_matches_queue_expansion_and_level_products(kconfig):
    parent, depth, q_row = O.tree_build(kconfig)
    qp, qd = _queue_tree(kconfig)
    np.testing.assert_array_equal(parent, qp)
    np.testing.assert_array_equal(depth, qd)
    sizes = np.cumprod(kconfig)
    assert parent.shape[0] == sizes.sum()
    for lvl, sz in enumerate(sizes, start=1):
        assert (depth == lvl).sum() == sz
    # every node above the last level has exactly k_{depth+1} children, consecutive, parents first
    N = parent.shape[0]
    for row in range(N + 1):
        kids = np.flatnonzero(parent == row - 1)
        dep = 0 if row == 0 else depth[row - 1]
        if dep < len(kconfig):
            assert len(kids) == kconfig[dep] and (np.diff(kids) == 1).all() and (kids > row - 1).all()
        else:
            assert len(kids) == 0
    # draft rows: internal rows numbered in row order, leaves -1
    internal = [r for r in range(N + 1) if (parent == r - 1).any()]
    assert [int(q_row[r]) for r in internal] == list(range(len(internal)))
    assert all(q_row[r] == -1 for r in range(N + 1) if r not in internal)


def test_tree_build_hand_example_and_limits():
    # k-configuration (2, 2): root -> {0, 1}; 0 -> {2, 3}; 1 -> {4, 5}
    parent, depth, q_row = O.tree_build((2, 2))
    assert parent.tolist() == [-1, -1, 0, 0, 1, 1]
    assert depth.tolist() == [1, 1, 2, 2, 2, 2]
    assert q_row.tolist() == [0, 1, 2, -1, -1, -1, -1]
    with pytest.raises(ValueError):
        O.tree_build((4, 4, 4, 2))          # 4 + 16 + 64 + 128 nodes > 128
    with pytest.raises(ValueError):
        O.tree_build((2, 0))


def _attention(q, K, V, scale):
    s = (K.astype(np.float64) @ q.astype(np.float64)) * scale
    w = np.exp(s - s.max())
    return (w / w.sum()) @ V.astype(np.float64)


def test_commit_makes_tree_attention_equal_plain_attention_over_the_cache():
    # the accepted node at depth n attends, in the tree call, to the prefix, its ancestors and itself;
    # after the commit those are exactly rows [0, L + n) of the cache
    rng = np.random.default_rng(31)
    B, H_q, H_kv, d, Ls = 2, 4, 2, 16, 24
    parent, depth, _ = O.tree_build((2, 2, 1))
    N = parent.shape[0]
    L = np.array([7, 13], np.int32)
    q = rng.standard_normal((B, N, H_q, d)).astype(np.float32)
    kp = rng.standard_normal((B, H_kv, Ls, d)).astype(np.float32)
    vp = rng.standard_normal((B, H_kv, Ls, d)).astype(np.float32)
    kt = rng.standard_normal((B, H_kv, N, d)).astype(np.float32)
    vt = rng.standard_normal((B, H_kv, N, d)).astype(np.float32)
    scale = 0.3
    tree_out = O.tree_attn(q, kp, vp, L, kt, vt, parent, scale, O.FP32)
    paths = np.array([[1, 4, 8], [0, 3, -1]], np.int32)       # root->1->4->8 ; root->0->3
    n_acc = np.array([3, 2], np.int32)
    out_tok = np.array([[11, 12, 13, 99], [21, 22, 77, -1]], np.int32)
    for b in range(B):
        for j in range(n_acc[b] - 1):
            assert parent[paths[b, j + 1]] == paths[b, j]
    k2, v2, L2, nxt, full = O.kv_commit(kp[None], vp[None], kt[None], vt[None], n_acc, paths, out_tok, L)
    assert L2.tolist() == [10, 15] and nxt.tolist() == [99, 77] and full.tolist() == [0, 0]
    G = H_q // H_kv
    for b in range(B):
        for j in range(n_acc[b]):
            node = paths[b, j]
            for h in range(H_q):
                g = h // G
                ref = _attention(q[b, node, h], k2[0, b, g, :L[b] + j + 1], v2[0, b, g, :L[b] + j + 1], scale)
                np.testing.assert_allclose(tree_out[b, node, h], ref, rtol=0, atol=1e-12)
    # nothing else moved
    for b in range(B):
        np.testing.assert_array_equal(k2[0, b, :, :L[b]], kp[b, :, :L[b]])
        np.testing.assert_array_equal(k2[0, b, :, L2[b]:], kp[b, :, L2[b]:])
        np.testing.assert_array_equal(v2[0, b, :, L2[b]:], vp[b, :, L2[b]:])


def test_commit_layers_full_cache_and_zero_accepted():
    rng = np.random.default_rng(32)
    nl, B, H_kv, d, Ls, N, G = 3, 3, 2, 8, 10, 6, 2
    kp = rng.integers(0, 60000, (nl, B, H_kv, Ls, d)).astype(np.uint16)
    vp = rng.integers(0, 60000, (nl, B, H_kv, Ls, d)).astype(np.uint16)
    kt = rng.integers(0, 60000, (nl, B, H_kv, N, d)).astype(np.uint16)
    vt = rng.integers(0, 60000, (nl, B, H_kv, N, d)).astype(np.uint16)
    L = np.array([9, 4, 10], np.int32)
    n_acc = np.array([2, 0, 0], np.int32)             # 9 + 2 > 10: full; none accepted; none accepted at a full cache
    paths = np.array([[1, 4], [-1, -1], [-1, -1]], np.int32)
    out_tok = np.array([[5, 6, 7], [8, -1, -1], [9, -1, -1]], np.int32)
    k2, v2, L2, nxt, full = O.kv_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L)
    assert full.tolist() == [1, 0, 0] and L2.tolist() == [9, 4, 10] and nxt.tolist() == [7, 8, 9]
    np.testing.assert_array_equal(k2, kp)
    np.testing.assert_array_equal(v2, vp)
    n_acc = np.array([1, 2, 0], np.int32)
    paths = np.array([[0, -1], [1, 5], [-1, -1]], np.int32)
    k2, v2, L2, nxt, full = O.kv_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L)
    assert full.tolist() == [0, 0, 0] and L2.tolist() == [10, 6, 10]
    for layer in range(nl):
        np.testing.assert_array_equal(k2[layer, 0, :, 9], kt[layer, 0, :, 0])
        np.testing.assert_array_equal(v2[layer, 1, :, 4], vt[layer, 1, :, 1])
        np.testing.assert_array_equal(v2[layer, 1, :, 5], vt[layer, 1, :, 5])
    changed = (k2 != kp)
    assert changed[:, 0, :, 9].any() and not changed[:, 2].any() and not changed[:, 0, :, :9].any()


def test_tree_build_agrees_with_the_input_generator():
    for kc in [(4, 2, 2), (4, 4, 2, 1)]:
        parent, depth, q_row = O.tree_build(kc)
        t = W.build_tree(kc)
        np.testing.assert_array_equal(parent, t.parent)
        np.testing.assert_array_equal(depth, t.depth)
        np.testing.assert_array_equal(q_row, t.q_row)


def with_root(parent):
    """The tree with its root as node 0: what root_row = 1 means for tree attention."""
    return np.concatenate([[-1], np.asarray(parent, np.int64) + 1]).astype(np.int32)


def test_root_row_two_decode_steps_equal_causal_attention_over_the_generated_sequence():
    """Sec. 3.3 / Sec. 3: the root of a step is the endpoint token of the step before and goes
    through the same forward pass as the candidates.  With the root as row 0 of the tree block:
    (1) tree attention of step 1 for the root and every candidate equals textbook causal attention
    over [context ; root ; path]; (2) after the commit the cache holds context, root, accepted
    tokens in sequence order; (3) in step 2 every candidate's attention equals causal attention
    over the whole generated sequence so far: context, root 1, accepted tokens of step 1, root 2
    (the endpoint of step 1), its own path."""
    rng = np.random.default_rng(33)
    B, H_q, H_kv, d, Ls = 2, 4, 2, 16, 40
    parent, depth, _ = O.tree_build((2, 2, 1))
    N = parent.shape[0]
    pr = with_root(parent)
    scale = 0.25
    L0 = np.array([7, 13], np.int32)
    kp = rng.standard_normal((B, H_kv, Ls, d)).astype(np.float32)
    vp = rng.standard_normal((B, H_kv, Ls, d)).astype(np.float32)
    G = H_q // H_kv

    def step_inputs():
        return (rng.standard_normal((B, 1 + N, H_q, d)).astype(np.float32),
                rng.standard_normal((B, H_kv, 1 + N, d)).astype(np.float32),
                rng.standard_normal((B, H_kv, 1 + N, d)).astype(np.float32))

    def check_against_sequences(q, kt, vt, kc, vc, L):
        out = O.tree_attn(q, kc, vc, L, kt, vt, pr, scale, O.FP32)
        for b in range(B):
            for r in range(1 + N):
                # rows of the tree block on the way from the root to r (row 0 = root, row 1 + i = candidate i)
                chain, a = [], r
                while a >= 0:
                    chain.append(a)
                    a = int(pr[a])
                chain = chain[::-1]
                assert chain[0] == 0
                for h in range(H_q):
                    g = h // G
                    K = np.concatenate([kc[b, g, :L[b]], kt[b, g, chain]])
                    V = np.concatenate([vc[b, g, :L[b]], vt[b, g, chain]])
                    np.testing.assert_allclose(out[b, r, h], _attention(q[b, r, h], K, V, scale), rtol=0, atol=1e-12)
        return out

    # step 1
    q1, kt1, vt1 = step_inputs()
    check_against_sequences(q1, kt1, vt1, kp, vp, L0)
    paths = np.array([[1, 4, 8], [0, 3, -1]], np.int32)
    n_acc = np.array([3, 2], np.int32)
    out_tok = np.array([[11, 12, 13, 99], [21, 22, 77, -1]], np.int32)
    k2, v2, L1, nxt, full = O.kv_commit(kp[None], vp[None], kt1[None], vt1[None], n_acc, paths, out_tok, L0, root_row=True)
    assert L1.tolist() == [7 + 1 + 3, 13 + 1 + 2] and nxt.tolist() == [99, 77] and full.tolist() == [0, 0]
    for b in range(B):
        # the cache now holds: context, root, accepted path, in that order; nothing else moved
        np.testing.assert_array_equal(k2[0, b, :, :L0[b]], kp[b, :, :L0[b]])
        np.testing.assert_array_equal(k2[0, b, :, L0[b]], kt1[b, :, 0])
        np.testing.assert_array_equal(v2[0, b, :, L0[b]], vt1[b, :, 0])
        for j in range(n_acc[b]):
            np.testing.assert_array_equal(k2[0, b, :, L0[b] + 1 + j], kt1[b, :, 1 + paths[b, j]])
            np.testing.assert_array_equal(v2[0, b, :, L0[b] + 1 + j], vt1[b, :, 1 + paths[b, j]])
        np.testing.assert_array_equal(k2[0, b, :, L1[b]:], kp[b, :, L1[b]:])
    # step 2: new root (the endpoint of step 1) and new candidates against the grown cache
    q2, kt2, vt2 = step_inputs()
    check_against_sequences(q2, kt2, vt2, k2[0], v2[0], L1)


def test_root_row_commit_full_cache_and_zero_accepted():
    rng = np.random.default_rng(34)
    nl, B, H_kv, d, Ls, N = 2, 3, 2, 8, 10, 6
    kp = rng.integers(0, 60000, (nl, B, H_kv, Ls, d)).astype(np.uint16)
    vp = rng.integers(0, 60000, (nl, B, H_kv, Ls, d)).astype(np.uint16)
    kt = rng.integers(0, 60000, (nl, B, H_kv, 1 + N, d)).astype(np.uint16)
    vt = rng.integers(0, 60000, (nl, B, H_kv, 1 + N, d)).astype(np.uint16)
    L = np.array([8, 4, 10], np.int32)
    n_acc = np.array([2, 0, 0], np.int32)     # 8 + 1 + 2 > 10: full; only the root; a full cache has no room for the root
    paths = np.array([[1, 4], [-1, -1], [-1, -1]], np.int32)
    out_tok = np.array([[5, 6, 7], [8, -1, -1], [9, -1, -1]], np.int32)
    k2, v2, L2, nxt, full = O.kv_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L, root_row=True)
    assert full.tolist() == [1, 0, 1] and L2.tolist() == [8, 5, 10] and nxt.tolist() == [7, 8, 9]
    for layer in range(nl):
        np.testing.assert_array_equal(k2[layer, 1, :, 4], kt[layer, 1, :, 0])
        np.testing.assert_array_equal(v2[layer, 1, :, 4], vt[layer, 1, :, 0])
    changed = (k2 != kp) | (v2 != vp)
    assert not changed[:, 0].any() and not changed[:, 2].any() and not changed[:, 1, :, :4].any() and not changed[:, 1, :, 5:].any()
