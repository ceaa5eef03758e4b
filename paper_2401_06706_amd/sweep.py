"""Acceptance rate and block efficiency of k-configurations on synthetic distributions.

For each k-configuration the draft-side sampler and the verification run on the GPU over many
independent synthetic sequences (target logits z ~ N(0, 3^2), draft logits z + N(0, sigma^2),
one independent row pair per tree row, as in the benchmark workloads) and the accepted path
lengths are averaged:

    tau   = mean(n_accepted) + 1        tokens emitted per verification step (block efficiency)
    alpha = accepted / reached          per tree level: acceptance rate of a parent with k_i candidates

This reproduces the *shape* of the paper's k-configuration study (Sec. 4.3 / 4.4: monotonically
decreasing configurations beat increasing ones of the same budget; equal budgets perform alike)
and of its ablation (Sec. 4.5: speculative sampling with / without replacement against naive
sampling) on synthetic distributions; the paper's own numbers need its models and datasets.

    python -m paper_2401_06706_amd.sweep --kconfigs 4x2 2x4 4x2x2 2x2x4 1x1x1x1 --sequences 512
"""
from __future__ import annotations

import argparse
import json
from typing import Dict, Sequence

import numpy as np
import torch

from . import binding as M
from . import device as D
from . import workloads as W

RULES = {"mcss_with": (W.WITH_REPLACEMENT, W.WITH_REPLACEMENT),
         "mcss_without": (W.WITHOUT_REPLACEMENT, W.WITHOUT_REPLACEMENT),
         "mcns": (W.WITH_REPLACEMENT, W.NAIVE)}       # (how candidates are drawn, how they are verified)


def make_batch(kconfig: Sequence[int], rule: str, B: int, V: int, sigma_q: float, temperature: float, seed: int,
               index: int):
    """Seeded inputs of batch number `index`: (VerifyInputs without candidates, u_draw [B][N])."""
    draw_variant, _ = RULES[rule]
    w = W.WORKLOADS["c2"].with_(kconfig=tuple(kconfig), V=V, sigma_q=sigma_q, n_greedy=0, B=B, variant=draw_variant)
    rng = np.random.default_rng([seed, index])
    vi = W.gen_verify_inputs(w, rng, temperature=[temperature] * B, draw_candidates_on_host=False)
    return vi, W.open_uniform(rng, (B, vi.N))


def run_config(kconfig: Sequence[int], rule: str, sequences: int, V: int = 32000, sigma_q: float = 1.0,
               temperature: float = 1.0, seed: int = 0, batch: int = 64) -> Dict:
    """Returns {"tau", "alpha" (per level), "n_accepted" (int array, one per sequence), ...}."""
    _, verify_variant = RULES[rule]
    gamma = len(kconfig)
    n_acc_all = []
    done = index = 0
    while done < sequences:
        B = min(batch, sequences - done)
        vi, u_draw = make_batch(kconfig, rule, B, V, sigma_q, temperature, seed, index)
        ver = D.make_verify_call(vi, want_ratio=False)
        draft = D.make_draft_call(vi, u_draw, cand_tok=ver.tensors["cand_tok"])
        ver.args.desc.variant = verify_variant
        M.mcsd_draft_sample(draft.args)
        M.mcsd_verify_sample(ver.args)
        torch.cuda.synchronize()
        n_acc_all.append(ver.tensors["n_accepted"].cpu().numpy().copy())
        done += B
        index += 1
    n_acc = np.concatenate(n_acc_all)
    reached = np.array([(n_acc >= lvl).sum() for lvl in range(gamma)], dtype=np.float64)       # parents of level lvl+1
    accepted = np.array([(n_acc >= lvl + 1).sum() for lvl in range(gamma)], dtype=np.float64)
    alpha = np.divide(accepted, reached, out=np.full(gamma, np.nan), where=reached > 0)
    return {"kconfig": "x".join(map(str, kconfig)), "rule": rule, "budget": int(np.cumprod(kconfig).sum()),
            "sequences": int(n_acc.shape[0]), "tau": float(n_acc.mean() + 1.0), "alpha": alpha.tolist(),
            "n_accepted": n_acc}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--kconfigs", nargs="+", default=["4x2", "2x4", "4x2x2", "2x2x4", "8x2x1x1", "1x1x1x1"])
    ap.add_argument("--rules", nargs="+", default=list(RULES), choices=list(RULES))
    ap.add_argument("--sequences", type=int, default=512)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--sigma", type=float, default=1.0)
    ap.add_argument("--temperature", type=float, default=1.0)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("sweep: no GPU visible")
    M.lib()
    for kc in args.kconfigs:
        kconfig = W.parse_kconfig(kc)
        for rule in args.rules:
            r = run_config(kconfig, rule, args.sequences, V=args.vocab, sigma_q=args.sigma, temperature=args.temperature)
            r.pop("n_accepted")
            print(json.dumps(r), flush=True)


if __name__ == "__main__":
    main()
