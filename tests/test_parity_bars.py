"""The attention parity bars of tests/parity.py have teeth where the outputs are small.

At a 16384-token prefix the outputs of tree attention are of size 0.05 and less, far below the
stated absolute tolerance of 2e-2, so the GPU tests add bars scaled to the reference.  Here
plausible kernel mistakes are planted into a numpy re-computation on the CPU (never on the GPU)
and the bars must catch each of them, while rounding of the size the bf16 kernel legitimately
makes (weights rounded to bf16 before the PV product, output rounded to bf16) must pass.
"""
import numpy as np
import pytest

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import workloads as W
from tests.parity import attn_violations


def round_bf16(x):
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.asarray(x, np.float32))).astype(np.float64)


@pytest.fixture(scope="module")
def long_prefix_case():
    w = W.WORKLOADS["c5"].with_(B=1, H_q=8, H_kv=1, kconfig=(2, 1), prefix=(16384, 16384))
    ai = W.gen_attn_inputs(w, np.random.default_rng(5))
    ref = O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                      O.BF16, n_threads=8)                                   # [1][N][H_q][d]
    f = lambda a: W.bf16_bits_to_f32(a).astype(np.float64)
    q, K, V = f(ai.q)[0], f(ai.k_prefix)[0, 0], f(ai.v_prefix)[0, 0]         # [N][H][d], [L][d]
    kt, vt = f(ai.k_tree)[0, 0], f(ai.v_tree)[0, 0]
    N = ai.N
    anc = np.zeros((N, N), bool)
    for i in range(N):
        a = i
        while a >= 0:
            anc[i, a] = True
            a = int(ai.parent[a])
    keys = np.concatenate([K, kt]); vals = np.concatenate([V, vt])
    S = ai.scale * np.einsum("nhd,kd->nhk", q, keys)
    vis = np.concatenate([np.ones((N, K.shape[0]), bool), anc], axis=1)[:, None, :]
    S = np.where(vis, S, -np.inf)
    return ai, ref[0], S, vals


def softmax_out(S, vals, keep=None, round_weights=False):
    Wt = np.exp(S - S.max(axis=-1, keepdims=True))
    if keep is not None:
        Wt = Wt * keep
    l = Wt.sum(axis=-1, keepdims=True)
    if round_weights:
        Wt = round_bf16(Wt)
    return np.einsum("nhk,kd->nhd", Wt, vals) / l


def test_numpy_recomputation_is_the_oracle(long_prefix_case):
    ai, ref, S, vals = long_prefix_case
    assert np.abs(softmax_out(S, vals) - ref).max() < 1e-12


def test_legitimate_bf16_rounding_passes(long_prefix_case):
    ai, ref, S, vals = long_prefix_case
    got = round_bf16(softmax_out(S, vals, round_weights=True))
    bad, st = attn_violations(got, ref, "bf16")
    assert not bad, bad
    assert st["max_ref"] < 0.1          # the case is one where 2e-2 alone says nothing


def test_all_zero_output_fails(long_prefix_case):
    ai, ref, S, vals = long_prefix_case
    bad, st = attn_violations(np.zeros_like(ref), ref, "bf16")
    assert len(bad) == 3, bad


def test_wrong_normaliser_fails_only_the_scaled_bars(long_prefix_case):
    """Every output 20 % too small (say, a row sum that counted some keys twice): an error of
    at most 9e-3 here, inside the absolute tolerance, caught by the bars scaled to the reference."""
    ai, ref, S, vals = long_prefix_case
    bad, st = attn_violations(round_bf16(0.8 * ref), ref, "bf16")
    assert st["max_err"] < 2e-2 and len(bad) == 2, bad


@pytest.mark.parametrize("tile", [0, 17, 511])
def test_one_dropped_key_tile_fails(long_prefix_case, tile):
    ai, ref, S, vals = long_prefix_case
    keep = np.ones(S.shape[-1])
    keep[32 * tile:32 * tile + 32] = 0.0
    got = round_bf16(softmax_out(S, vals, keep=keep))
    bad, st = attn_violations(got, ref, "bf16")
    assert bad, st


def test_mis_weighted_segment_fails(long_prefix_case):
    """Two key segments merged with the second one's weight off by 3 %."""
    ai, ref, S, vals = long_prefix_case
    keep = np.ones(S.shape[-1])
    keep[8192:] = 1.03
    got = round_bf16(softmax_out(S, vals, keep=keep))
    bad, st = attn_violations(got, ref, "bf16")
    assert bad, st


def test_rows_of_two_heads_swapped_fails(long_prefix_case):
    ai, ref, S, vals = long_prefix_case
    got = round_bf16(softmax_out(S, vals))
    got[:, [0, 1]] = got[:, [1, 0]]
    bad, _ = attn_violations(got, ref, "bf16")
    assert bad
