"""Comparison of libmcsd's verification outputs with the CPU oracle.

Bar: accepted child / endpoint / path / emitted tokens bit-exact, except for rows
where the ORACLE's own decision margin (distance between a uniform and the
threshold it was compared with) is below 1e-6; those are counted, logged and
excluded, together with the walk of the sequence if the differing row lies on
either side's path.  Tested ratios agree to 1e-6 abs, residuals to 1e-6 abs.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from oracle import mcsd_oracle as O

NEAR_TIE = 1e-6


def run_oracle(vi, want_residual=False, n_threads=8):
    return O.verify(vi.target_logits, vi.draft_logits, vi.tree.q_row, vi.tree.parent, vi.cand_tok,
                    vi.u_accept, vi.u_endpoint, vi.temperature, vi.variant, gamma_max=vi.tree.gamma,
                    want_residual=want_residual, n_threads=n_threads)


def compare_verify(vi, gpu: Dict[str, np.ndarray], orc, check_residual=False, label="") -> Dict[str, int]:
    B, N = vi.B, vi.N
    stats = dict(rows=B * (1 + N), near_tie_rows=0, near_tie_mismatch=0, seq_excluded=0, gpu_flagged=0)
    near = orc.margin < NEAR_TIE
    stats["near_tie_rows"] = int(near.sum())
    stats["gpu_flagged"] = int(((gpu["flags"] & 3) != 0).sum())
    row_bad = (gpu["acc_child"] != orc.acc_child) | (gpu["endpoint"] != orc.endpoint)
    hard = row_bad & ~near
    if hard.any():
        b, r = np.argwhere(hard)[0]
        raise AssertionError(
            f"{label}: row (b={b}, row={r}) differs: gpu acc_child={gpu['acc_child'][b, r]} endpoint="
            f"{gpu['endpoint'][b, r]}, oracle acc_child={orc.acc_child[b, r]} endpoint={orc.endpoint[b, r]}, "
            f"oracle margin={orc.margin[b, r]:.3e}; {int(hard.sum())} such rows")
    stats["near_tie_mismatch"] = int((row_bad & near).sum())
    if stats["near_tie_mismatch"]:
        for b, r in np.argwhere(row_bad & near):
            print(f"[near-tie] {label} b={b} row={r} oracle margin={orc.margin[b, r]:.3e} "
                  f"gpu=({gpu['acc_child'][b, r]},{gpu['endpoint'][b, r]}) "
                  f"oracle=({orc.acc_child[b, r]},{orc.endpoint[b, r]})")
    # no data-error flags on well-formed inputs
    assert ((gpu["flags"] & ~np.int32(3 | 8)) == 0).all(), f"{label}: unexpected flag bits"
    # ratios: same tested / not-tested pattern, values to 1e-6 (rows with a mismatch excluded)
    if "ratio" in gpu:
        child_row = vi.tree.parent.astype(np.int64) + 1          # row that owns each node's test
        ok_nodes = ~row_bad[:, child_row]
        g, o = gpu["ratio"].astype(np.float64), orc.ratio
        assert (np.isnan(g) == np.isnan(o))[ok_nodes].all(), f"{label}: tested-candidate pattern differs"
        m = ok_nodes & ~np.isnan(o)
        err = np.abs(g[m] - o[m])
        assert err.size == 0 or err.max() <= 1e-6, f"{label}: ratio error {err.max():.3e}"
        stats["max_ratio_err"] = float(err.max()) if err.size else 0.0
    # walk
    for b in range(B):
        tainted = False
        for res_path, n in ((gpu["accepted_path"][b], int(gpu["n_accepted"][b])),
                            (orc.accepted_path[b], int(orc.n_accepted[b]))):
            rows = [0] + [1 + int(c) for c in res_path[:max(n, 0)] if c >= 0]
            tainted |= any(row_bad[b, r] for r in rows)
        if tainted:
            stats["seq_excluded"] += 1
            continue
        assert gpu["n_accepted"][b] == orc.n_accepted[b], f"{label}: n_accepted differs at b={b}"
        assert (gpu["accepted_path"][b] == orc.accepted_path[b]).all(), f"{label}: path differs at b={b}"
        assert (gpu["out_tokens"][b] == orc.out_tokens[b]).all(), f"{label}: tokens differ at b={b}"
    if check_residual:
        ok = ~row_bad
        err = np.abs(gpu["residual_out"].astype(np.float64) - orc.residual)[ok]
        assert err.max() <= 1e-6, f"{label}: residual error {err.max():.3e}"
        stats["max_residual_err"] = float(err.max())
        s = gpu["residual_out"].astype(np.float64).sum(axis=-1)[ok]
        assert np.abs(s - 1.0).max() < 1e-5, f"{label}: residual does not sum to 1"
    return stats


# ---------------------------------------------------------------- tree attention
# Two bars.  The absolute one is the stated tolerance (2e-2 for bf16 storage, 1e-5 for fp32).
# Outputs are convex combinations of N(0,1) values, so they shrink like 1/sqrt(keys): at a
# 16384-token prefix max|out| is about 0.05 and the absolute bar alone would pass an output of
# zeros.  The second bar therefore scales with the reference itself: the largest error may not
# exceed ATTN_REL x max|ref|, and the RMS error may not exceed ATTN_RMS x RMS(ref).  The sources
# of error are the bf16 rounding of the softmax weights before the PV product (2^-9 relative
# per weight, averaging out over the keys) and of the output (2^-9 of each value): both scale
# with the output, which is why a relative bar holds at every prefix length.
ATTN_ABS = {"fp32": 1e-5, "bf16": 2e-2}
ATTN_REL = {"fp32": 1e-5, "bf16": 2.0 ** -7}
ATTN_RMS = {"fp32": 2e-6, "bf16": 4e-3}


def attn_error_stats(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    err = np.abs(got - ref)
    return dict(max_err=float(err.max()), max_ref=float(np.abs(ref).max()),
                rms_err=float(np.sqrt(np.mean(err * err))), rms_ref=float(np.sqrt(np.mean(ref * ref))),
                argmax=tuple(int(i) for i in np.unravel_index(int(err.argmax()), err.shape)))


def attn_violations(got, ref, dtype):
    """The list of bars `got` fails against the oracle's `ref` (empty: parity)."""
    st = attn_error_stats(got, ref)
    bad = []
    if not np.isfinite(np.asarray(got, np.float64)).all():
        bad.append("non-finite output")
    if st["max_err"] > ATTN_ABS[dtype]:
        bad.append(f"max abs err {st['max_err']:.3e} > {ATTN_ABS[dtype]:.1e}")
    if st["max_err"] > ATTN_REL[dtype] * st["max_ref"]:
        bad.append(f"max abs err {st['max_err']:.3e} > {ATTN_REL[dtype]:.2e} x max|ref| {st['max_ref']:.3e}")
    if st["rms_err"] > ATTN_RMS[dtype] * st["rms_ref"]:
        bad.append(f"rms err {st['rms_err']:.3e} > {ATTN_RMS[dtype]:.1e} x rms(ref) {st['rms_ref']:.3e}")
    return bad, st


def assert_attn_close(got, ref, dtype, label=""):
    bad, st = attn_violations(got, ref, dtype)
    print(f"[attn-parity] {label}: max err {st['max_err']:.3e} (at {st['argmax']}), max|ref| {st['max_ref']:.3e}, "
          f"ratio {st['max_err'] / max(st['max_ref'], 1e-300):.2e}; rms err {st['rms_err']:.3e}, rms(ref) {st['rms_ref']:.3e}, "
          f"ratio {st['rms_err'] / max(st['rms_ref'], 1e-300):.2e}", flush=True)
    assert not bad, f"{label}: " + "; ".join(bad)
    return st
