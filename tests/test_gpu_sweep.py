"""The k-configuration sweep (draft sampling + verification on the GPU over many synthetic
sequences): agrees with the oracle sequence by sequence, and shows the effects the paper reports
for its k-configuration study and ablation (Sec. 4.3 - 4.5) on synthetic distributions."""
import numpy as np
import pytest

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import sweep as S
from paper_2401_06706_amd import workloads as W

pytestmark = pytest.mark.gpu
V, SEQ = 512, 2048


@pytest.mark.parametrize("rule", ["mcss_with", "mcss_without", "mcns"])
def test_sweep_batch_matches_oracle(rule):
    kconfig, B = (3, 2, 2), 64
    r = S.run_config(kconfig, rule, B, V=V, seed=9, batch=B)
    vi, u_draw = S.make_batch(kconfig, rule, B, V, 1.0, 1.0, 9, 0)
    draw_variant, verify_variant = S.RULES[rule]
    cand, dm = O.draft_sample(vi.draft_logits, vi.tree.q_row, vi.tree.parent, u_draw, vi.temperature, draw_variant, n_threads=8)
    ref = O.verify(vi.target_logits, vi.draft_logits, vi.tree.q_row, vi.tree.parent, cand, vi.u_accept, vi.u_endpoint,
                   vi.temperature, verify_variant, gamma_max=vi.tree.gamma, n_threads=8)
    clean = (dm >= 1e-6).all(axis=1) & (ref.margin >= 1e-6).all(axis=1)
    assert clean.sum() >= B // 2
    np.testing.assert_array_equal(r["n_accepted"][clean], ref.n_accepted[clean])


def test_monotonic_rule_and_budget_groups():
    tau = {kc: S.run_config(W.parse_kconfig(kc), "mcss_without", SEQ, V=V, seed=1)["tau"]
           for kc in ["4x2", "2x4", "4x2x2", "2x2x4", "8x1", "1x8"]}
    print("tau:", tau)
    # decreasing beats increasing at the same budget (Sec. 4.4): the next level is only reached through this one
    assert tau["4x2"] > tau["2x4"] + 0.02
    assert tau["4x2x2"] > tau["2x2x4"] + 0.02
    assert tau["8x1"] > tau["1x8"] + 0.02


def test_speculative_rules_beat_naive_sampling_and_more_candidates_help():
    kc = (4, 2, 2)
    t = {rule: S.run_config(kc, rule, SEQ, V=V, seed=2) for rule in S.RULES}
    print({k: (round(v["tau"], 3), [round(a, 3) for a in v["alpha"]]) for k, v in t.items()})
    assert t["mcss_with"]["tau"] > t["mcns"]["tau"] + 0.05           # Sec. 4.5 ablation; Appendix C
    assert t["mcss_without"]["tau"] >= t["mcss_with"]["tau"] - 0.03   # without replacement is at least as good
    sd = S.run_config((1, 1, 1), "mcss_with", SEQ, V=V, seed=2)      # one candidate per step: plain speculative decoding
    assert t["mcss_with"]["tau"] > sd["tau"] + 0.1
    assert t["mcss_with"]["alpha"][0] > sd["alpha"][0] + 0.05        # alpha grows with k (Sec. 4.2)
