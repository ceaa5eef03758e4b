"""mcsd_tree_build and mcsd_kv_commit against the oracle (bit-exact), and a short decode loop
(tree build -> draft sampling -> verification step -> KV commit, repeated) run on the GPU
without host round trips and compared with the same loop through the oracle."""
import numpy as np
import pytest
import torch

from oracle import mcsd_oracle as O
from paper_2401_06706_amd import binding as M
from paper_2401_06706_amd import device as D
from paper_2401_06706_amd import workloads as W
from tests.parity import assert_attn_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


@pytest.mark.parametrize("kconfig", [(1,), (2, 2), (4, 2, 2), (8, 2, 1, 1), (4, 2, 2, 1, 1), (4, 4, 2, 1), (128,),
                                     (2, 3, 4), (1,) * 16, (3, 1, 5, 2)])
def test_tree_build(kconfig):
    N, P = M.mcsd_tree_size(kconfig)
    B = 5
    L = np.array([0, 17, 4096, 1, 123456], np.int32)
    parent = torch.full((N,), -9, dtype=torch.int32, device=DEV)
    depth = torch.full((N,), -9, dtype=torch.int32, device=DEV)
    q_row = torch.full((N + 1,), -9, dtype=torch.int32, device=DEV)
    pos = torch.full((B, N), -9, dtype=torch.int32, device=DEV)
    M.mcsd_tree_build(kconfig, parent, depth, q_row, prefix_len=dev_i32(L), position_ids=pos)
    torch.cuda.synchronize()
    rp, rd, rq = O.tree_build(kconfig)
    assert rp.shape[0] == N and (rq >= 0).sum() == P
    np.testing.assert_array_equal(parent.cpu().numpy(), rp)
    np.testing.assert_array_equal(depth.cpu().numpy(), rd)
    np.testing.assert_array_equal(q_row.cpu().numpy(), rq)
    np.testing.assert_array_equal(pos.cpu().numpy(), L[:, None] + rd[None, :] - 1)
    # without position ids
    parent.fill_(-9)
    M.mcsd_tree_build(kconfig, parent, depth, q_row)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(parent.cpu().numpy(), rp)


def make_commit_case(rng, n_layers, B, H_kv, d, Ls, kconfig, dtype, L, n_acc):
    parent, depth, _ = O.tree_build(kconfig)
    N, gamma = parent.shape[0], len(kconfig)
    np_dt = np.float32 if dtype == "fp32" else np.uint16
    def rnd(shape):
        if dtype == "fp32":
            return rng.standard_normal(shape).astype(np.float32)
        return rng.integers(0, 0x7f7f, shape).astype(np.uint16)
    kp, vp = rnd((n_layers, B, H_kv, Ls, d)), rnd((n_layers, B, H_kv, Ls, d))
    kt, vt = rnd((n_layers, B, H_kv, N, d)), rnd((n_layers, B, H_kv, N, d))
    paths = np.full((B, gamma), -1, np.int32)
    for b in range(B):
        node = -1
        for j in range(n_acc[b]):
            kids = np.flatnonzero(parent == node)
            node = int(rng.choice(kids))
            paths[b, j] = node
    out_tok = rng.integers(0, 32000, (B, gamma + 1)).astype(np.int32)
    return kp, vp, kt, vt, paths, out_tok, N, gamma


def run_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L, dtype):
    def up(a):
        t = torch.from_numpy(a.view(np.int16) if dtype == "bf16" else a).to(DEV)
        return t.view(torch.bfloat16) if dtype == "bf16" else t
    t_kp, t_vp, t_kt, t_vt = up(kp), up(vp), up(kt), up(vt)
    B = L.shape[0]
    t_L = dev_i32(L)
    nxt = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    fl = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    args = M.commit_args(t_kp, t_vp, t_kt, t_vt, dev_i32(n_acc), dev_i32(paths), dev_i32(out_tok), t_L, nxt, fl)
    M.mcsd_kv_commit(args)
    torch.cuda.synchronize()
    def down(t):
        a = t.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else t.cpu().numpy()
        return a
    return down(t_kp), down(t_vp), t_L.cpu().numpy(), nxt.cpu().numpy(), fl.cpu().numpy()


@pytest.mark.parametrize("dtype,n_layers,B,H_kv,d,kconfig", [
    ("bf16", 1, 16, 32, 128, (4, 2, 2, 1, 1)), ("bf16", 4, 4, 8, 128, (4, 4, 2, 1)), ("fp32", 2, 3, 1, 64, (2, 2)),
    ("bf16", 3, 2, 2, 8, (3, 1, 2)), ("fp32", 1, 1, 5, 4, (1,))])
def test_kv_commit_matches_oracle(dtype, n_layers, B, H_kv, d, kconfig):
    rng = np.random.default_rng(B * 100 + d)
    Ls, gamma = 40, len(kconfig)
    L = rng.integers(0, Ls - gamma + 1, B).astype(np.int32)
    n_acc = rng.integers(0, gamma + 1, B).astype(np.int32)
    if B >= 3:
        L[1] = Ls - 1; n_acc[1] = min(2, gamma)          # does not fit (when gamma >= 2): nothing committed
        L[2] = Ls - gamma; n_acc[2] = gamma              # fits exactly
    kp, vp, kt, vt, paths, out_tok, N, gamma = make_commit_case(rng, n_layers, B, H_kv, d, Ls, kconfig, dtype, L, n_acc)
    got = run_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L, dtype)
    ref = O.kv_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L)
    np.testing.assert_array_equal(got[0], ref[0])
    np.testing.assert_array_equal(got[1], ref[1])
    np.testing.assert_array_equal(got[2], ref[2])
    np.testing.assert_array_equal(got[3], ref[3])
    np.testing.assert_array_equal(got[4] != 0, ref[4] != 0)
    assert set(np.unique(got[4]).tolist()) <= {0, 256}


def test_kv_commit_flags_bad_path_entries():
    rng = np.random.default_rng(3)
    L = np.array([5, 5], np.int32)
    n_acc = np.array([3, 2], np.int32)
    kp, vp, kt, vt, paths, out_tok, N, gamma = make_commit_case(rng, 1, 2, 2, 8, 20, (2, 2, 2), "fp32", L, n_acc)
    paths[0, 1] = 999                # second entry out of range: only the first row is committed
    got = run_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L, "fp32")
    assert got[2].tolist() == [6, 7] and got[4].tolist() == [64, 0]
    np.testing.assert_array_equal(got[0][0, 0, :, 5], kt[0, 0, :, paths[0, 0]])
    np.testing.assert_array_equal(got[0][0, 0, :, 6:], kp[0, 0, :, 6:])


def test_decode_loop_three_steps_matches_oracle_loop():
    """tree build -> draft sample -> attention + verification -> commit, three times, all on one
    stream with no host reads in between; then the same loop through the oracle.  The root of a
    step (the endpoint token of the step before) goes through the step's forward pass with the
    candidates: it is row 0 of the tree block (root_row = 1), every candidate attends to it, and
    the commit appends it ahead of the accepted path.  From the second step on, the attention of
    every row is also compared with textbook causal attention over the sequence generated so
    far (context, earlier roots and accepted tokens, this step's root, the row's own path)."""
    rng = np.random.default_rng(77)
    kconfig = (3, 2, 2)
    B, H_q, H_kv, d, Ls, V, steps = 3, 4, 2, 128, 64, 2048, 3
    N, P = M.mcsd_tree_size(kconfig)
    gamma = len(kconfig)
    tree = W.build_tree(kconfig)
    L0 = np.array([9, 20, 33], np.int32)
    bf = lambda a: W.f32_to_bf16_bits(a.astype(np.float32))
    kp0, vp0 = bf(rng.standard_normal((B, H_kv, Ls, d))), bf(rng.standard_normal((B, H_kv, Ls, d)))
    temp = np.array([1.0, 0.0, 0.8], np.float32)
    per_step = []
    for s in range(steps):
        zp = (3 * rng.standard_normal((B, 1 + N, V))).astype(np.float32)
        zq = np.empty((B, P, V), np.float32)
        for row in range(1 + N):                      # draft row = its target row plus noise: candidates get accepted
            if tree.q_row[row] >= 0:
                zq[:, tree.q_row[row]] = zp[:, row] + rng.standard_normal((B, V)).astype(np.float32)
        per_step.append(dict(
            q=bf(rng.standard_normal((B, 1 + N, H_q, d))), kt=bf(rng.standard_normal((B, H_kv, 1 + N, d))),
            vt=bf(rng.standard_normal((B, H_kv, 1 + N, d))),
            zp=zp, zq=zq,
            u_draw=W.open_uniform(rng, (B, N)), u_acc=W.open_uniform(rng, (B, N)), u_end=W.open_uniform(rng, (B, 1 + N))))
    variant = W.WITHOUT_REPLACEMENT

    # ---- GPU loop
    def up_bf(a):
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    t_kp, t_vp = up_bf(kp0), up_bf(vp0)
    t_L = dev_i32(L0)
    parent = torch.empty(N, dtype=torch.int32, device=DEV)
    depth = torch.empty(N, dtype=torch.int32, device=DEV)
    q_row = torch.empty(N + 1, dtype=torch.int32, device=DEV)
    pos = torch.empty((B, 1 + N), dtype=torch.int32, device=DEV)
    t_temp = torch.from_numpy(temp).to(DEV)
    i32 = dict(dtype=torch.int32, device=DEV)
    gpu_log = []
    keep = []
    for s in range(steps):
        x = per_step[s]
        M.mcsd_tree_build(kconfig, parent, depth, q_row, prefix_len=t_L, position_ids=pos)
        t_q, t_kt, t_vt = up_bf(x["q"]), up_bf(x["kt"]), up_bf(x["vt"])
        out = torch.empty_like(t_q)
        desc = M.attn_desc(B, N, H_q, H_kv, d, M.DTYPE_BF16, Ls, 1.0 / np.sqrt(d), root_row=True)
        ws = torch.empty(max(M.mcsd_attn_workspace_bytes(desc), 256), dtype=torch.uint8, device=DEV)
        a_args = M.attn_args(t_q, t_kp, t_vp, t_L, t_kt, t_vt, parent, out, 1.0 / np.sqrt(d), workspace=ws)
        assert a_args.desc.root_row == 1 and a_args.desc.N == N
        t_zq = torch.from_numpy(x["zq"]).to(DEV)
        cand = torch.full((B, N), -5, **i32)
        dfl = torch.empty((B, N), **i32)
        d_args = M.draft_args(t_zq, q_row, parent, torch.from_numpy(x["u_draw"]).to(DEV), t_temp, cand, dfl, variant)
        n_acc = torch.empty((B,), **i32); path = torch.empty((B, gamma), **i32); otok = torch.empty((B, gamma + 1), **i32)
        acc = torch.empty((B, 1 + N), **i32); endp = torch.empty((B, 1 + N), **i32); vfl = torch.empty((B, 1 + N), **i32)
        v_args = M.verify_args(torch.from_numpy(x["zp"]).to(DEV), t_zq, q_row, parent, cand,
                               torch.from_numpy(x["u_acc"]).to(DEV), torch.from_numpy(x["u_end"]).to(DEV), t_temp,
                               n_acc, path, otok, acc, endp, vfl, variant)
        nxt = torch.empty((B,), **i32); cfl = torch.empty((B,), **i32)
        c_args = M.commit_args(t_kp, t_vp, t_kt, t_vt, n_acc, path, otok, t_L, nxt, cfl, root_row=True)
        assert c_args.desc.root_row == 1 and c_args.desc.N == N
        M.mcsd_draft_sample(d_args)
        M.mcsd_verify_step(a_args, v_args)
        M.mcsd_kv_commit(c_args)
        keep.append((a_args, d_args, v_args, c_args, ws))
        gpu_log.append((out, cand, n_acc, path, otok, nxt, cfl, pos.clone(), dfl, vfl))
    torch.cuda.synchronize()

    # ---- oracle loop
    kp, vp, L = kp0.copy(), vp0.copy(), L0.copy()
    for s in range(steps):
        x = per_step[s]
        out, cand, n_acc, path, otok, nxt, cfl, pos_s, dfl, vfl = [t.cpu() for t in gpu_log[s]]
        rp, rd, rq = O.tree_build(kconfig)
        np.testing.assert_array_equal(pos_s.numpy()[:, 0], L)                       # the root: first token after the cache
        np.testing.assert_array_equal(pos_s.numpy()[:, 1:], L[:, None] + rd[None, :])
        rp_ext = np.concatenate([[-1], rp.astype(np.int64) + 1]).astype(np.int32)   # the tree with its root as node 0
        r_cand, r_dm = O.draft_sample(x["zq"], rq, rp, x["u_draw"], temp, variant)
        assert (r_dm >= 1e-6).all(), "pick another seed: a draw sits on a CDF edge"
        np.testing.assert_array_equal(cand.numpy(), r_cand)
        ref_attn = O.tree_attn(x["q"], kp, vp, L, x["kt"], x["vt"], rp_ext, 1.0 / np.sqrt(d), O.BF16, n_threads=8)
        got_attn = W.bf16_bits_to_f32(out.view(torch.int16).numpy().view(np.uint16))
        assert_attn_close(got_attn, ref_attn, "bf16", f"decode loop step {s}")
        if s >= 1:
            # causal attention over the generated sequence: cache rows [0, L) hold context, the
            # earlier roots and accepted tokens; then this step's root and the row's path
            f64 = lambda a: W.bf16_bits_to_f32(a).astype(np.float64)
            seq_ref = np.zeros((1 + N, d))
            b0, h0 = 0, 1
            g0 = h0 // (H_q // H_kv)
            for r in range(1 + N):
                chain, a = [], r
                while a >= 0:
                    chain.append(a)
                    a = int(rp_ext[a])
                K = np.concatenate([f64(kp[b0, g0, :L[b0]]), f64(x["kt"][b0, g0, chain[::-1]])])
                Vv = np.concatenate([f64(vp[b0, g0, :L[b0]]), f64(x["vt"][b0, g0, chain[::-1]])])
                sc = (K @ f64(x["q"][b0, r, h0])) / np.sqrt(d)
                wgt = np.exp(sc - sc.max())
                seq_ref[r] = (wgt / wgt.sum()) @ Vv
            assert np.abs(seq_ref - ref_attn[b0, :, h0]).max() < 1e-12
            assert_attn_close(got_attn[b0, :, h0], seq_ref, "bf16", f"step {s}: causal attention over the generated sequence")
        rv = O.verify(x["zp"], x["zq"], rq, rp, r_cand, x["u_acc"], x["u_end"], temp, variant, gamma_max=gamma, n_threads=8)
        on_path_rows = [[0] + [1 + int(c) for c in rv.accepted_path[b] if c >= 0] for b in range(B)]
        for b in range(B):
            assert all(rv.margin[b, r] >= 1e-6 for r in on_path_rows[b]), "pick another seed: near tie on the path"
        np.testing.assert_array_equal(n_acc.numpy(), rv.n_accepted)
        np.testing.assert_array_equal(path.numpy(), rv.accepted_path)
        np.testing.assert_array_equal(otok.numpy(), rv.out_tokens)
        kp1, vp1, L1, r_nxt, r_full = O.kv_commit(kp[None], vp[None], x["kt"][None], x["vt"][None], rv.n_accepted,
                                                  rv.accepted_path, rv.out_tokens, L, root_row=True)
        kp, vp, L = kp1[0], vp1[0], L1
        np.testing.assert_array_equal(nxt.numpy(), r_nxt)
        assert (cfl.numpy() == 0).all() and (r_full == 0).all()
    np.testing.assert_array_equal(t_L.cpu().numpy(), L)
    np.testing.assert_array_equal(t_kp.view(torch.int16).cpu().numpy().view(np.uint16), kp)
    np.testing.assert_array_equal(t_vp.view(torch.int16).cpu().numpy().view(np.uint16), vp)
    assert (L >= L0 + steps).all() and (L - L0).sum() >= 6 + B * steps


@pytest.mark.parametrize("page_size,n_layers", [(32, 1), (64, 3)])
def test_kv_commit_paged_matches_contiguous_commit(page_size, n_layers):
    """Commit into a page pool; gathering the pool back by the layout's definition gives the
    oracle's contiguous commit, layer by layer.  Includes a sequence whose new rows cross a page
    boundary, one without room, and untouched spare pages."""
    rng = np.random.default_rng(11)
    B, H_kv, d, kconfig = 4, 2, 16, (2, 2, 2)
    per_seq = 3
    Ls = per_seq * page_size
    L = np.array([page_size - 1, 5, Ls - 1, 2 * page_size - 2], np.int32)
    n_acc = np.array([3, 2, 2, 3], np.int32)          # seq 0 and 3 cross a page boundary; seq 2 does not fit
    kp, vp, kt, vt, paths, out_tok, N, gamma = make_commit_case(rng, n_layers, B, H_kv, d, Ls, kconfig, "fp32", L, n_acc)
    n_pages = B * per_seq + 2
    table = rng.permutation(n_pages)[: B * per_seq].reshape(B, per_seq).astype(np.int32)
    kpool = rng.standard_normal((n_layers, n_pages, H_kv, page_size, d)).astype(np.float32)
    vpool = rng.standard_normal((n_layers, n_pages, H_kv, page_size, d)).astype(np.float32)
    for layer in range(n_layers):
        for b in range(B):
            for pg in range(per_seq):
                kpool[layer, table[b, pg]] = kp[layer, b, :, pg * page_size:(pg + 1) * page_size]
                vpool[layer, table[b, pg]] = vp[layer, b, :, pg * page_size:(pg + 1) * page_size]
    t = lambda a: torch.from_numpy(a).to(DEV)
    t_kpool, t_vpool, t_L = t(kpool), t(vpool), dev_i32(L)
    nxt = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    fl = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    args, paged = M.paged_commit_args(t_kpool, t_vpool, dev_i32(table), t(kt), t(vt), dev_i32(n_acc), dev_i32(paths),
                                      dev_i32(out_tok), t_L, nxt, fl, Ls)
    M.mcsd_kv_commit_paged(args, paged)
    torch.cuda.synchronize()
    ref_k, ref_v, ref_L, ref_nxt, ref_full = O.kv_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L)
    got_kpool, got_vpool = t_kpool.cpu().numpy(), t_vpool.cpu().numpy()
    for layer in range(n_layers):
        np.testing.assert_array_equal(O.gather_pages(got_kpool[layer], table, Ls), ref_k[layer])
        np.testing.assert_array_equal(O.gather_pages(got_vpool[layer], table, Ls), ref_v[layer])
    np.testing.assert_array_equal(t_L.cpu().numpy(), ref_L)
    np.testing.assert_array_equal(nxt.cpu().numpy(), ref_nxt)
    np.testing.assert_array_equal(fl.cpu().numpy() != 0, ref_full != 0)
    assert ref_full.tolist() == [0, 0, 1, 0]
    spare = [pg for pg in range(n_pages) if pg not in table.reshape(-1).tolist()]
    np.testing.assert_array_equal(got_kpool[:, spare], kpool[:, spare])


def test_kv_commit_paged_stops_at_a_table_entry_outside_the_pool():
    rng = np.random.default_rng(12)
    B, H_kv, d, page_size, per_seq = 2, 2, 8, 32, 2
    Ls = per_seq * page_size
    L = np.array([30, 10], np.int32)
    n_acc = np.array([3, 3], np.int32)                 # sequence 0: rows 30, 31 in page 0, row 32 in page 1
    kp, vp, kt, vt, paths, out_tok, N, gamma = make_commit_case(rng, 1, B, H_kv, d, Ls, (2, 2, 2), "fp32", L, n_acc)
    table = np.array([[0, 99], [1, 2]], np.int32)      # sequence 0's second page is not in the pool
    kpool = np.zeros((1, 3, H_kv, page_size, d), np.float32)
    vpool = np.zeros_like(kpool)
    t = lambda a: torch.from_numpy(a).to(DEV)
    t_kpool, t_vpool, t_L = t(kpool), t(vpool), dev_i32(L)
    nxt = torch.empty((B,), dtype=torch.int32, device=DEV)
    fl = torch.empty((B,), dtype=torch.int32, device=DEV)
    args, paged = M.paged_commit_args(t_kpool, t_vpool, dev_i32(table), t(kt), t(vt), dev_i32(n_acc), dev_i32(paths),
                                      dev_i32(out_tok), t_L, nxt, fl, Ls)
    M.mcsd_kv_commit_paged(args, paged)
    torch.cuda.synchronize()
    assert t_L.cpu().numpy().tolist() == [32, 13] and fl.cpu().numpy().tolist() == [64, 0]
    got = t_kpool.cpu().numpy()
    np.testing.assert_array_equal(got[0, 0, :, 30], kt[0, 0, :, paths[0, 0]])
    np.testing.assert_array_equal(got[0, 0, :, 31], kt[0, 0, :, paths[0, 1]])
    np.testing.assert_array_equal(got[0, 1, :, 10:13], kt[0, 1][:, paths[1]])
    assert not got[0, 2].any()


@pytest.mark.parametrize("dtype,n_layers,B,H_kv,d,kconfig", [("bf16", 2, 5, 4, 128, (4, 2, 2, 1)), ("fp32", 1, 3, 2, 16, (2, 2))])
def test_kv_commit_with_root_row_matches_oracle(dtype, n_layers, B, H_kv, d, kconfig):
    """The tree block carries the root as row 0: the commit appends the root, then the path; a cache
    with room for the path but not for the root as well is left alone; contiguous and paged."""
    rng = np.random.default_rng(B * 7 + d)
    gamma = len(kconfig)
    Ls = 64
    L = rng.integers(0, Ls - gamma - 1, B).astype(np.int32)
    n_acc = rng.integers(0, gamma + 1, B).astype(np.int32)
    L[0], n_acc[0] = Ls - gamma, gamma                 # the path alone would fit, root + path does not
    L[1], n_acc[1] = Ls - 1, 0                          # exactly room for the root
    kp, vp, kt0, vt0, paths, out_tok, N, _ = make_commit_case(rng, n_layers, B, H_kv, d, Ls, kconfig, dtype, L, n_acc)
    def root_first(a):
        extra = rng.standard_normal((n_layers, B, H_kv, 1, d)).astype(np.float32) if dtype == "fp32" else \
            rng.integers(0, 0x7f7f, (n_layers, B, H_kv, 1, d)).astype(np.uint16)
        return np.ascontiguousarray(np.concatenate([extra, a], axis=3))
    kt, vt = root_first(kt0), root_first(vt0)
    ref = O.kv_commit(kp, vp, kt, vt, n_acc, paths, out_tok, L, root_row=True)
    assert ref[4][0] == 1 and ref[4][1] == 0 and ref[2][1] == Ls
    def up(a):
        t = torch.from_numpy(a.view(np.int16) if dtype == "bf16" else a).to(DEV)
        return t.view(torch.bfloat16) if dtype == "bf16" else t
    def down(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else t.cpu().numpy()
    t_kp, t_vp, t_L = up(kp), up(vp), dev_i32(L)
    nxt = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    fl = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    args = M.commit_args(t_kp, t_vp, up(kt), up(vt), dev_i32(n_acc), dev_i32(paths), dev_i32(out_tok), t_L, nxt, fl, root_row=True)
    M.mcsd_kv_commit(args)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(down(t_kp), ref[0])
    np.testing.assert_array_equal(down(t_vp), ref[1])
    np.testing.assert_array_equal(t_L.cpu().numpy(), ref[2])
    np.testing.assert_array_equal(nxt.cpu().numpy(), ref[3])
    np.testing.assert_array_equal(fl.cpu().numpy() != 0, ref[4] != 0)
    # the same into a page pool
    page_size, per_seq = 32, 2
    n_pages = B * per_seq + 1
    table = rng.permutation(n_pages)[: B * per_seq].reshape(B, per_seq).astype(np.int32)
    kpool = np.zeros((n_layers, n_pages, H_kv, page_size, d), kp.dtype)
    vpool = np.zeros_like(kpool)
    for layer in range(n_layers):
        for b in range(B):
            for pg in range(per_seq):
                kpool[layer, table[b, pg]] = kp[layer, b, :, pg * page_size:(pg + 1) * page_size]
                vpool[layer, table[b, pg]] = vp[layer, b, :, pg * page_size:(pg + 1) * page_size]
    t_kpool, t_vpool, t_L2 = up(kpool), up(vpool), dev_i32(L)
    pargs, paged = M.paged_commit_args(t_kpool, t_vpool, dev_i32(table), up(kt), up(vt), dev_i32(n_acc), dev_i32(paths),
                                       dev_i32(out_tok), t_L2, nxt, fl, Ls, root_row=True)
    M.mcsd_kv_commit_paged(pargs, paged)
    torch.cuda.synchronize()
    for layer in range(n_layers):
        np.testing.assert_array_equal(O.gather_pages(down(t_kpool)[layer], table, Ls), ref[0][layer])
        np.testing.assert_array_equal(O.gather_pages(down(t_vpool)[layer], table, Ls), ref[1][layer])
    np.testing.assert_array_equal(t_L2.cpu().numpy(), ref[2])
