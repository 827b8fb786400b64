"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- closed forms, torch's library attention routine, numpy's
stable sort, brute force over tiny cases, exhaustive enumeration, and the one
family of numbers the paper prints (tests/golden/rbar_table.txt).  Each check
is chosen so that a dropped term, a wrong sign or index, or a transposed
operand in the oracle fails it.  CPU only.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2503_14075_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, stream, shape, std=1.0, dtype=torch.float32):
    return W.normal(seed, stream, shape, std, dtype)


# ----------------------------------------------------------------------------
# ttp_score  (Sec. 3.1 Eq. 2-3, head mean)
# ----------------------------------------------------------------------------
def _library_attention_map(q, k, pos0, scale, causal):
    """Attention map through torch's fused attention routine: with V = identity
    the routine's output *is* the map A.  q [n_q][H][d], k [n][H][d] -> [H][n_q][n]."""
    n_q, n = q.shape[0], k.shape[0]
    qq = q.double().permute(1, 0, 2)[None]
    kk = k.double().permute(1, 0, 2)[None]
    eye = torch.eye(n, dtype=torch.float64).expand(1, q.shape[1], n, n)
    mask = None
    if causal:
        pos = pos0 + torch.arange(n_q)[:, None]
        mask = torch.arange(n)[None, :] <= pos
    return F.scaled_dot_product_attention(qq, kk, eye, attn_mask=mask, scale=scale)[0]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("causal", [True, False])
def test_score_matches_library_attention_map(dtype, causal):
    H, d, M, N, n_q, v0 = 3, 16, 37, 9, 5, 2
    n_tot = v0 + M + N
    q = _rand(11, 1, (1, n_q, H, d), 1.0, dtype)
    k = _rand(11, 2, (n_tot, H, d), 1.0, dtype)
    pos0 = n_tot - n_q
    got = oracle.ttp_score(q, k, [n_q], [pos0], [n_tot], [0], v0, M, 0.3, causal)[0]
    A = _library_attention_map(q[0], k, pos0, 0.3, causal)
    want = A[:, :, v0:v0 + M].sum(dim=(0, 1)) / (H * n_q)
    assert torch.allclose(got, want, rtol=0, atol=1e-12)


def test_score_uniform_keys_closed_form():
    # identical keys -> uniform attention: causal row at position p gives 1/(p+1) to each visible key
    H, d, M, N, n_q = 2, 8, 20, 6, 4
    n_tot = M + N
    k = _rand(3, 1, (1, H, d)).expand(n_tot, H, d).contiguous()
    q = _rand(3, 2, (1, n_q, H, d))
    pos0 = n_tot - n_q
    got = oracle.ttp_score(q, k, [n_q], [pos0], [n_tot], [0], 0, M, 0.5, True)[0]
    want = sum(1.0 / (pos0 + i + 1) for i in range(n_q)) / n_q
    assert torch.allclose(got, torch.full((M,), want, dtype=torch.float64), atol=1e-14)
    got = oracle.ttp_score(q, k, [n_q], [pos0], [n_tot], [0], 0, M, 0.5, False)[0]
    assert torch.allclose(got, torch.full((M,), 1.0 / n_tot, dtype=torch.float64), atol=1e-14)


def test_score_mass_and_dominant_key_and_permutation():
    H, d, M, N, n_q = 4, 8, 30, 10, 10
    n_tot = M + N
    q = _rand(5, 1, (1, n_q, H, d))
    k = _rand(5, 2, (n_tot, H, d))
    # whole sequence as the span: every attention row sums to one
    full = oracle.ttp_score(q, k, [n_q], [M], [n_tot], [0], 0, n_tot, 0.35, True)[0]
    assert abs(float(full.sum()) - 1.0) < 1e-13
    vis = oracle.ttp_score(q, k, [n_q], [M], [n_tot], [0], 0, M, 0.35, True)[0]
    assert torch.equal(vis, full[:M])          # span position only selects columns
    # a span that does not start at zero selects the shifted columns
    sh = oracle.ttp_score(q, k, [n_q], [M], [n_tot], [0], 7, 11, 0.35, True)[0]
    assert torch.equal(sh, full[7:18])
    # heads and (non-causal) scoring rows may be permuted freely
    hp = torch.tensor([2, 0, 3, 1])
    rp = torch.randperm(n_q, generator=torch.Generator().manual_seed(1))
    base = oracle.ttp_score(q, k, [n_q], [M], [n_tot], [0], 0, M, 0.35, False)[0]
    perm = oracle.ttp_score(q[:, rp][:, :, hp].contiguous(), k[:, hp].contiguous(), [n_q], [M],
                            [n_tot], [0], 0, M, 0.35, False)[0]
    assert torch.allclose(base, perm, atol=1e-15)
    # one key aligned with every query and a large scale takes all the mass
    k2 = k.clone()
    k2[13] = 0
    qs = torch.ones(1, n_q, H, d)
    k2[13] = 50.0
    dom = oracle.ttp_score(qs, k2, [n_q], [M], [n_tot], [0], 0, M, 1.0, True)[0]
    assert dom[13] > 1 - 1e-9 and float(dom.sum()) <= 1 + 1e-12


def test_score_single_query_textbook_softmax_and_batch_offsets():
    # n_q = 1, H = 1: one softmax over the keys, typed out with numpy
    d, M, N = 8, 12, 3
    n_tot = M + N
    q = _rand(7, 1, (2, 1, 1, d))
    k = _rand(7, 2, (2 * n_tot + 5, 1, d))
    offs = [5, 5 + n_tot]                  # two sequences at different pool offsets
    got = oracle.ttp_score(q, k, [1, 1], [n_tot - 1] * 2, [n_tot] * 2, offs, 0, M, 0.7, True)
    for b in range(2):
        kk = k[offs[b]:offs[b] + n_tot, 0].double().numpy()
        s = 0.7 * kk @ q[b, 0, 0].double().numpy()
        e = np.exp(s - s.max())
        assert np.allclose(got[b].numpy(), (e / e.sum())[:M], atol=1e-14)


def test_score_ragged_rows_use_only_their_own_count():
    H, d, M = 2, 8, 10
    n_tot = [M + 4, M + 7]
    q = _rand(9, 1, (2, 7, H, d))
    k = _rand(9, 2, (sum(n_tot), H, d))
    got = oracle.ttp_score(q, k, [4, 7], [M, M], n_tot, [0, n_tot[0]], 0, M, 0.3, True)
    for b, (nq, off) in enumerate(zip([4, 7], [0, n_tot[0]])):
        A = _library_attention_map(q[b, :nq], k[off:off + n_tot[b]], M, 0.3, True)
        assert torch.allclose(got[b], A[:, :, :M].sum(dim=(0, 1)) / (H * nq), atol=1e-13)


def test_score_rejects_bad_spans():
    q = torch.zeros(1, 2, 1, 4)
    k = torch.zeros(10, 1, 4)
    with pytest.raises(ValueError):
        oracle.ttp_score(q, k, [2], [8], [10], [0], 5, 6, 1.0, True)     # span past the end
    with pytest.raises(ValueError):
        oracle.ttp_score(q, k, [3], [7], [10], [0], 0, 6, 1.0, True)     # more rows than supplied


# ----------------------------------------------------------------------------
# ttp_select  (TopR of Sec. 3.1 Eq. 3; ties toward the lower index)
# ----------------------------------------------------------------------------
def _repeated_max(scores, R):
    s = [float(x) for x in scores]
    taken = []
    for _ in range(R):
        best = None
        for m, x in enumerate(s):
            if m in taken:
                continue
            if best is None or x > s[best]:
                best = m
        taken.append(best)
    return sorted(taken)


@pytest.mark.parametrize("seed", range(6))
def test_select_vs_stable_argsort_and_repeated_max(seed):
    g = torch.Generator().manual_seed(seed)
    M = 97
    # few distinct values -> many ties, including -0.0 / +0.0
    vals = torch.tensor([-1.5, -0.0, 0.0, 0.25, 0.25, 3.0])
    sc = vals[torch.randint(0, len(vals), (4, M), generator=g)].float()
    for R in (0, 1, 13, 50, M - 1, M):
        got = oracle.ttp_select(sc, R)
        for b in range(4):
            x = sc[b].numpy()
            order = np.argsort(-(x + 0.0), kind="stable")      # +0.0 folds -0 into +0
            assert got[b].tolist() == sorted(order[:R].tolist())
            if R <= 13:
                assert got[b].tolist() == _repeated_max(x, R)


def test_select_closed_forms():
    M, R = 40, 7
    assert oracle.ttp_select(torch.zeros(1, M), R)[0].tolist() == list(range(R))
    dec = torch.arange(M, 0, -1).float()[None]
    inc = torch.arange(M).float()[None]
    assert oracle.ttp_select(dec, R)[0].tolist() == list(range(R))
    assert oracle.ttp_select(inc, R)[0].tolist() == list(range(M - R, M))
    assert oracle.ttp_select(inc, M)[0].tolist() == list(range(M))
    assert oracle.ttp_select(inc, 0).shape == (1, 0)
    sc = torch.zeros(1, M)
    sc[0, [5, 9, 31]] = torch.tensor([1e-30, -1e-30, 2.0])     # tiny magnitudes and a negative
    assert oracle.ttp_select(sc, 3)[0].tolist() == [0, 5, 31]
    with pytest.raises(ValueError):
        oracle.ttp_select(inc, M + 1)


# ----------------------------------------------------------------------------
# ttp_compact
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.uint8])
def test_compact_identity_subsequence_and_library_gather(dtype):
    v0, M, N = 3, 25, 6
    n_tot = v0 + M + N
    src = torch.randint(0, 255, (n_tot, 10), generator=torch.Generator().manual_seed(1)).to(dtype)
    assert torch.equal(oracle.ttp_compact(torch.arange(M), v0, M, src), src)      # keep all
    kept = torch.tensor([0, 4, 5, 17, 24])
    dst = oracle.ttp_compact(kept, v0, M, src)
    idx = torch.cat([torch.arange(v0), v0 + kept, torch.arange(v0 + M, n_tot)])
    assert torch.equal(dst, src.index_select(0, idx))
    assert torch.equal(dst[-N:], src[-N:]) and torch.equal(dst[:v0], src[:v0])
    wipe = oracle.ttp_compact(torch.tensor([], dtype=torch.int32), v0, M, src)     # R = 0 drops the span
    assert torch.equal(wipe, torch.cat([src[:v0], src[v0 + M:]]))


def test_compact_composes():
    M, N = 30, 4
    src = _rand(2, 1, (M + N, 6))
    k1 = torch.tensor([1, 3, 4, 8, 20, 21, 29])
    k2 = torch.tensor([0, 2, 5, 6])
    twice = oracle.ttp_compact(k2, 0, len(k1), oracle.ttp_compact(k1, 0, M, src))
    once = oracle.ttp_compact(k1[k2], 0, M, src)
    assert torch.equal(twice, once)
    with pytest.raises(ValueError):
        oracle.ttp_compact(torch.tensor([M]), 0, M, src)


# ----------------------------------------------------------------------------
# tree_ancestors / tree_verify_attn  (Sec. 5.4, App. A)
# ----------------------------------------------------------------------------
def test_ancestors_by_hand():
    #        0
    #      / | \
    #     1  2  3
    #     |     |
    #     4     5
    #     |
    #     6
    par = [-1, 0, 0, 0, 1, 3, 4]
    want = [0b1, 0b11, 0b101, 0b1001, 0b10011, 0b101001, 0b1010011]
    assert oracle.tree_ancestors(par) == want
    assert oracle.tree_ancestors([-1] + list(range(63)))[63] == (1 << 64) - 1
    for bad in ([0, 0], [-1, 1], [-1, -1], [-1, 0, 3]):
        with pytest.raises(ValueError):
            oracle.tree_ancestors(bad)


def _causal_library(q_rows, k_rows, v_rows, scale):
    """Plain causal attention of the last len(q_rows) positions over all rows, via
    torch's routine.  q [t][H][d], k/v [n][H][d] -> [t][H][d] fp64."""
    t, n = q_rows.shape[0], k_rows.shape[0]
    mask = torch.arange(n)[None, :] <= (n - t + torch.arange(t))[:, None]
    o = F.scaled_dot_product_attention(q_rows.double().permute(1, 0, 2)[None],
                                       k_rows.double().permute(1, 0, 2)[None],
                                       v_rows.double().permute(1, 0, 2)[None],
                                       attn_mask=mask, scale=scale)
    return o[0].permute(1, 0, 2)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_verify_chain_equals_causal_decode(dtype):
    H, d, C, T = 3, 16, 21, 7
    q = _rand(21, 1, (1, T, H, d), 1.0, dtype)
    k = _rand(21, 2, (C + T + 4, H, d), 1.0, dtype)
    v = _rand(21, 3, (C + T + 4, H, d), 1.0, dtype)
    par = [-1] + list(range(T - 1))
    got = oracle.tree_verify_attn(q, k, v, [C], [T], [par], 0.25, row_off=[4])[0]
    want = _causal_library(q[0], k[4:], v[4:], 0.25)
    assert torch.allclose(got, want, atol=1e-12)


@pytest.mark.parametrize("seed", range(4))
def test_verify_tree_equals_per_branch_causal_runs(seed):
    H, d, C, T = 2, 8, 13, 12
    par = W.random_parent_tree(W.HostRng(seed, 1), T, 4)
    q = _rand(seed, 1, (1, T, H, d))
    k = _rand(seed, 2, (C + T, H, d))
    v = _rand(seed, 3, (C + T, H, d))
    got = oracle.tree_verify_attn(q, k, v, [C], [T], [par], 0.4, row_off=[0])[0]
    leaves = [i for i in range(T) if i not in par]
    seen = set()
    for leaf in leaves:
        chain = []
        u = leaf
        while u >= 0:
            chain.append(u)
            u = par[u]
        chain.reverse()
        rows = list(range(C)) + [C + u for u in chain]
        want = _causal_library(q[0, chain], k[rows], v[rows], 0.4)
        for pos, u in enumerate(chain):
            assert torch.allclose(got[u], want[pos], atol=1e-12)
            seen.add(u)
    assert seen == set(range(T))


def test_grouped_query_attention_reads_key_head_h_div_g():
    """Grouped-query attention (the Qwen2.5-VL base model among those of Sec. 6): query head h of
    H = g * H_kv reads key/value head h // g.  Checked against the library routines run on the
    key/value heads written out g times each (repeat_interleave; the interleaved order h % H_kv
    would fail, the heads differ)."""
    H, H_kv, d, C, T = 6, 2, 8, 11, 9
    g = H // H_kv
    par = W.random_parent_tree(W.HostRng(5, 1), T, 4)
    q = _rand(21, 1, (1, T, H, d))
    k = _rand(21, 2, (C + T, H_kv, d))
    v = _rand(21, 3, (C + T, H_kv, d))
    got = oracle.tree_verify_attn(q, k, v, [C], [T], [par], 0.4, row_off=[0])[0]
    kx, vx = k.repeat_interleave(g, dim=1), v.repeat_interleave(g, dim=1)
    for leaf in [i for i in range(T) if i not in par]:
        chain = []
        u = leaf
        while u >= 0:
            chain.append(u)
            u = par[u]
        chain.reverse()
        rows = list(range(C)) + [C + u for u in chain]
        want = _causal_library(q[0, chain], kx[rows], vx[rows], 0.4)
        for pos, u in enumerate(chain):
            assert torch.allclose(got[u], want[pos], atol=1e-12)
    wrong = oracle.tree_verify_attn(q, k.repeat(1, g, 1), v.repeat(1, g, 1), [C], [T], [par], 0.4, row_off=[0])[0]
    assert not torch.allclose(got, wrong, atol=1e-3)          # the two head orders are told apart
    # the score: library attention map over the expanded keys
    M, N, n_q, v0 = 21, 7, 4, 1
    n_tot = v0 + M + N
    qs = _rand(22, 1, (1, n_q, H, d))
    ks = _rand(22, 2, (n_tot, H_kv, d))
    pos0 = n_tot - n_q
    sc = oracle.ttp_score(qs, ks, [n_q], [pos0], [n_tot], [0], v0, M, 0.3, True)[0]
    A = _library_attention_map(qs[0], ks.repeat_interleave(g, dim=1), pos0, 0.3, True)
    assert torch.allclose(sc, A[:, :, v0:v0 + M].sum(dim=(0, 1)) / (H * n_q), rtol=0, atol=1e-12)
    with pytest.raises(AssertionError):
        oracle.ttp_score(qs[:, :, :5].contiguous(), ks, [n_q], [pos0], [n_tot], [0], v0, M, 0.3, True)


def test_verify_closed_forms_constant_v_constant_k_star_and_single():
    H, d, C, T = 2, 8, 9, 6
    par = [-1, 0, 0, 1, 1, 2]
    q = _rand(31, 1, (1, T, H, d))
    k = _rand(31, 2, (C + T, H, d))
    v = _rand(31, 3, (C + T, H, d))
    # all value rows equal -> every output equals that row whatever the mask
    vc = v[:1].expand(C + T, H, d).contiguous()
    got = oracle.tree_verify_attn(q, k, vc, [C], [T], [par], 0.3, row_off=[0])[0]
    assert torch.allclose(got, vc[0].double().expand(T, H, d), atol=1e-13)
    # all key rows equal -> uniform weights -> mean of the visible value rows
    kc = k[:1].expand(C + T, H, d).contiguous()
    got = oracle.tree_verify_attn(q, kc, v, [C], [T], [par], 0.3, row_off=[0])[0]
    anc = {0: [0], 1: [0, 1], 2: [0, 2], 3: [0, 1, 3], 4: [0, 1, 4], 5: [0, 2, 5]}
    for t in range(T):
        rows = list(range(C)) + [C + u for u in anc[t]]
        assert torch.allclose(got[t], v[rows].double().mean(0), atol=1e-13)
    # star: each leaf sees context + root + itself only
    star = [-1, 0, 0, 0, 0, 0]
    got = oracle.tree_verify_attn(q, k, v, [C], [T], [star], 0.3, row_off=[0])[0]
    for t in range(1, T):
        rows = list(range(C)) + [C, C + t]
        want = _causal_library(q[0, [t]], k[rows], v[rows], 0.3)
        assert torch.allclose(got[t], want[0], atol=1e-12)
    # T = 1: ordinary one-token decode attention, typed out with numpy for one head
    got = oracle.tree_verify_attn(q[:, :1].contiguous(), k, v, [C], [1], [[-1]], 0.3, row_off=[0])[0]
    s = 0.3 * k[:C + 1, 1].double().numpy() @ q[0, 0, 1].double().numpy()
    e = np.exp(s - s.max())
    assert np.allclose(got[0, 1].numpy(), (e / e.sum()) @ v[:C + 1, 1].double().numpy(), atol=1e-13)
    # empty context: only the tree rows are keys
    got = oracle.tree_verify_attn(q, k, v, [0], [T], [par], 0.3, row_off=[C])[0]
    want = _causal_library(q[0, [0, 1, 3]], k[[C, C + 1, C + 3]], v[[C, C + 1, C + 3]], 0.3)
    assert torch.allclose(got[3], want[2], atol=1e-12)


def test_verify_paged_equals_contiguous_and_ragged_batch():
    H, d, pr = 2, 8, 4
    ctx, nn = [10, 3], [5, 7]
    pars = [[-1, 0, 0, 1, 3, -1, -1], [-1, 0, 1, 1, 0, 4, 5]]     # first tree uses 5 of 7 slots
    pars[0][5:] = [0, 0]                                            # padding entries are ignored
    q = _rand(41, 1, (2, 7, H, d))
    rows = [c + t for c, t in zip(ctx, nn)]
    off = [0, rows[0]]
    k = _rand(41, 2, (sum(rows), H, d))
    v = _rand(41, 3, (sum(rows), H, d))
    cont = oracle.tree_verify_attn(q, k, v, ctx, nn, pars, 0.5, row_off=off)
    # scatter the same rows into shuffled pages
    n_pages = [(r + pr - 1) // pr for r in rows]
    ids = list(range(sum(n_pages)))
    W.HostRng(1, 2).shuffle(ids)
    pt, kk = [], 0
    for n in n_pages:
        pt.append(ids[kk:kk + n] + [0] * (max(n_pages) - n))
        kk += n
    kp = torch.zeros(sum(n_pages) * pr, H, d)
    vp = torch.zeros_like(kp)
    for b in range(2):
        for r in range(rows[b]):
            dst = pt[b][r // pr] * pr + r % pr
            kp[dst], vp[dst] = k[off[b] + r], v[off[b] + r]
    paged = oracle.tree_verify_attn(q, kp, vp, ctx, nn, pars, 0.5, page_table=pt, page_rows=pr)
    assert torch.equal(cont, paged)
    # instance 0 alone gives the same rows; rows past n_nodes stay zero
    solo = oracle.tree_verify_attn(q[:1, :5].contiguous(), k, v, ctx[:1], nn[:1], [pars[0][:5]], 0.5,
                                   row_off=off[:1])
    assert torch.equal(solo[0], cont[0, :5])
    assert float(cont[0, 5:].abs().max()) == 0.0


# ----------------------------------------------------------------------------
# tree_accept  (Sec. 5.4, App. A, Alg. 2; chain = Alg. 1)
# ----------------------------------------------------------------------------
def _enumerate_paths(draft, argmx, par):
    """Every root->node path; keep the fully matched ones; longest wins, then lowest index."""
    best, best_len, best_path = 0, 0, []
    for i in range(len(par)):
        path, u = [], i
        while u > 0:
            path.append(u)
            u = par[u]
        path.reverse()
        if all(draft[u] == argmx[par[u]] for u in path):
            if len(path) > best_len:
                best, best_len, best_path = i, len(path), path
    return best_len, best_path, argmx[best]


def _all_trees(T):
    for tail in itertools.product(*[range(i) for i in range(1, T)]):
        yield [-1] + list(tail)


def _run_accept_cases(cases, T):
    d = [c[0] for c in cases]
    a = [c[1] for c in cases]
    p = [c[2] for c in cases]
    n_acc, path, bonus = oracle.tree_accept(d, a, p, [T] * len(cases))
    for i, (dr, am, pa) in enumerate(cases):
        ln, pth, bo = _enumerate_paths(dr, am, pa)
        assert int(n_acc[i]) == ln, (dr, am, pa)
        assert path[i].tolist() == pth + [-1] * (T - ln), (dr, am, pa)
        assert int(bonus[i]) == bo, (dr, am, pa)


def test_accept_exhaustive_small_trees_binary_alphabet():
    for T in (1, 2, 3, 4, 5):
        cases = []
        for par in _all_trees(T):
            for dr in itertools.product((0, 1), repeat=T):
                for am in itertools.product((0, 1), repeat=T):
                    cases.append((list(dr), list(am), par))
        _run_accept_cases(cases, T)


@pytest.mark.parametrize("T,alpha", [(6, 2), (7, 3), (7, 2), (12, 3)])
def test_accept_sampled_larger_trees(T, alpha):
    rng = W.HostRng(T * 10 + alpha, 0)
    cases = []
    for _ in range(6000):
        par = W.random_parent_tree(rng, T, T)
        dr = [rng.randint(0, alpha - 1) for _ in range(T)]
        am = [rng.randint(0, alpha - 1) for _ in range(T)]
        cases.append((dr, am, par))
    _run_accept_cases(cases, T)


def test_accept_chain_is_longest_matching_prefix_and_special_cases():
    rng = W.HostRng(5, 5)
    T = 9
    par = [-1] + list(range(T - 1))
    for _ in range(500):
        dr = [rng.randint(0, 2) for _ in range(T)]
        am = [rng.randint(0, 2) for _ in range(T)]
        # sequence case: drafts dr[1..], target predictions am[0..]; stop at the first mismatch
        n = 0
        while n + 1 < T and dr[n + 1] == am[n]:
            n += 1
        n_acc, path, bonus = oracle.tree_accept([dr], [am], [par], [T])
        assert int(n_acc[0]) == n and int(bonus[0]) == am[n]
        assert path[0].tolist() == list(range(1, n + 1)) + [-1] * (T - n)
    # nothing matches -> only the bonus token of the root
    par = [-1, 0, 0, 1, 2]
    n_acc, path, bonus = oracle.tree_accept([[9, 1, 2, 3, 4]], [[5, 6, 7, 8, 9]], [par], [5])
    assert (int(n_acc[0]), int(bonus[0]), path[0].tolist()) == (0, 5, [-1] * 5)
    # full match down to leaf 4 (0 -> 2 -> 4)
    n_acc, path, bonus = oracle.tree_accept([[0, 1, 50, 3, 70]], [[50, 6, 70, 8, 99]], [par], [5])
    assert (int(n_acc[0]), int(bonus[0]), path[0].tolist()) == (2, 99, [2, 4, -1, -1, -1])
    # duplicate sibling ids: both children of the root match, only the second continues
    par = [-1, 0, 0, 2]
    n_acc, path, bonus = oracle.tree_accept([[0, 7, 7, 8]], [[7, 1, 8, 3]], [par], [4])
    assert (int(n_acc[0]), int(bonus[0]), path[0].tolist()) == (2, 3, [2, 3, -1, -1])
    # equal depth -> lower node index
    n_acc, path, bonus = oracle.tree_accept([[0, 7, 7, 8]], [[7, 1, 2, 3]], [par], [4])
    assert (int(n_acc[0]), int(bonus[0]), path[0].tolist()) == (1, 1, [1, -1, -1, -1])
    # only the first n_nodes entries count
    n_acc, _, _ = oracle.tree_accept([[0, 7, 7, 8]], [[7, 1, 8, 3]], [par], [3])
    assert int(n_acc[0]) == 1


# ----------------------------------------------------------------------------
# sequence-based self-speculative decoding (Sec. 3.1; App. A, SSD paragraph; Alg. 1)
# ----------------------------------------------------------------------------
def test_chain_draft_length_by_hand():
    th = 0.6
    assert oracle.chain_draft_len([0.9, 0.8, 0.7, 0.65, 0.61], th, 5) == 5      # never below the threshold
    assert oracle.chain_draft_len([0.9, 0.5, 0.9, 0.9, 0.9], th, 5) == 2        # the weak token is the last one kept
    assert oracle.chain_draft_len([0.1, 0.9, 0.9, 0.9, 0.9], th, 5) == 1
    assert oracle.chain_draft_len([0.9, 0.9, 0.9, 0.9, 0.1], th, 5) == 5        # delta reached at the same step
    assert oracle.chain_draft_len([0.6, 0.6, 0.6], 0.6, 3) == 3                 # equal is not below (both fp32)
    assert oracle.chain_draft_len(None, th, 5) == 5
    assert oracle.chain_draft_len([0.0], th, 1) == 1
    with pytest.raises(ValueError):
        oracle.chain_draft_len(None, th, 0)


def test_chain_accept_by_hand_and_against_the_tree_walk():
    x = 77   # the last accepted token: never read
    assert oracle.chain_accept([x, 5, 6, 7], [5, 6, 9, 4], 3) == (2, 9)    # third draft token wrong -> target's 9
    assert oracle.chain_accept([x, 5, 6, 7], [5, 6, 7, 8], 3) == (3, 8)    # all right -> bonus token
    assert oracle.chain_accept([x, 5, 6, 7], [4, 6, 7, 1], 3) == (0, 4)    # later matches do not count after a miss
    assert oracle.chain_accept([x, 5, 6, 7], [5, 6, 7, 8], 2) == (2, 7)    # a shorter draft stops at its end
    assert oracle.chain_accept([x], [3], 0) == (0, 3)
    # the chain is a tree with parent[i] = i - 1: the exhaustively pinned tree walk gives the same
    rng = W.HostRng(11, 3)
    for _ in range(600):
        T = rng.randint(1, 9)
        dr = [rng.randint(0, 2) for _ in range(T)]
        am = [rng.randint(0, 2) for _ in range(T)]
        n_acc, _, bonus = oracle.tree_accept([dr], [am], [[-1] + list(range(T - 1))], [T])
        assert oracle.chain_accept(dr, am, T - 1) == (int(n_acc[0]), int(bonus[0]))
        # and the definition, prefix length by prefix length
        ks = [k for k in range(T) if all(dr[i] == am[i - 1] for i in range(1, k + 1))]
        assert oracle.chain_accept(dr, am, T - 1)[0] == max(ks)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_chain_decoding_reproduces_the_target_model(seed):
    # Sec. 3.1: self-speculative decoding gives the response of the target model alone.  A toy
    # deterministic target (next token = a hash of the last three tokens), a draft model that is
    # the target with mistakes and made-up confidences; draft-then-verify with the two functions
    # must emit exactly the greedy decoding of the target.
    rng = W.HostRng(100 + seed, 1)
    V, delta, theta = 7, 5, 0.6
    target = lambda toks: (3 * toks[-1] + 5 * toks[-2] + toks[-3] * toks[-1] + seed) % V
    prompt = [1, 2, 3]
    want = list(prompt)
    for _ in range(60):
        want.append(target(want))
    got = list(prompt)
    while len(got) < len(want):
        ctx, draft, prob = list(got), [], []
        for _ in range(delta):                       # the draft model runs delta steps; the early exit cuts them
            t = target(ctx) if rng.uniform() < 0.7 else rng.randint(0, V - 1)
            draft.append(t)
            prob.append(rng.uniform())
            ctx.append(t)
        n_draft = oracle.chain_draft_len(prob, theta, delta)
        draft = draft[:n_draft]
        # one pass of the target over [last accepted token] + draft: prediction after every position
        am = [target(got + draft[:i]) for i in range(n_draft + 1)]
        n_acc, nxt = oracle.chain_accept([got[-1]] + draft, am, n_draft)
        got += draft[:n_acc] + [nxt]
    assert got[:len(want)] == want


# ----------------------------------------------------------------------------
# the numbers the paper prints (Sec. 4.2 Eq. 6)
# ----------------------------------------------------------------------------
def test_rbar_matches_printed_settings():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "rbar_table.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 8
    for M, K, R, K_f, L, want in (map(int, r) for r in rows):
        assert oracle.rbar(M, K, R, K_f, L) == want
    assert oracle.rbar(576, 2, 64, 32, 32) == round((576 * 2 + 64 * 30) / 32)   # Eq. 4 form


# ----------------------------------------------------------------------------
# kv_commit (the step after the acceptance walk; KV append of Sec. 3.1)
# ----------------------------------------------------------------------------
def test_kv_commit_gather_identity_and_untouched_rows():
    C, T, width = 5, 8, 6
    pool = torch.arange((C + T + 3) * width, dtype=torch.float32).view(-1, width)
    off = 2
    # accepted nodes 2, 5, 6 -> rows C+1, C+2, C+3 (library gather on a snapshot)
    before = pool.clone()
    new_len = oracle.kv_commit(pool, [C], [T], [[2, 5, 6, -1, -1, -1, -1, -1]], [3], row_off=[off])
    assert new_len == [C + 1 + 3]
    want = before.clone()
    want[off + C + 1:off + C + 4] = before.index_select(0, torch.tensor([off + C + 2, off + C + 5, off + C + 6]))
    assert torch.equal(pool, want)
    assert torch.equal(pool[:off + C + 1], before[:off + C + 1])            # context and root untouched
    assert torch.equal(pool[off + C + 4:], before[off + C + 4:])            # rejected tail left behind
    # a chain prefix is already in place
    pool2 = before.clone()
    assert oracle.kv_commit(pool2, [C], [T], [[1, 2, 3, 4, -1, -1, -1, -1]], [4], row_off=[off]) == [C + 5]
    assert torch.equal(pool2, before)
    # overlapping moves (source of one is the destination of the next) still read the old rows
    pool3 = before.clone()
    oracle.kv_commit(pool3, [C], [T], [[2, 3, 4, 5, 6, 7, -1, -1]], [6], row_off=[off])
    assert torch.equal(pool3[off + C + 1:off + C + 7], before[off + C + 2:off + C + 8])
    # nothing accepted: only the root is committed
    pool4 = before.clone()
    assert oracle.kv_commit(pool4, [C], [T], [[-1] * 8], [0], row_off=[off]) == [C + 1]
    assert torch.equal(pool4, before)
    for bad in ([[0, 1, -1, -1, -1, -1, -1, -1]], [[3, 2, -1, -1, -1, -1, -1, -1]], [[2, 8, -1, -1, -1, -1, -1, -1]]):
        with pytest.raises(ValueError):
            oracle.kv_commit(before.clone(), [C], [T], bad, [2], row_off=[off])


def test_kv_commit_then_decode_equals_attention_over_the_accepted_path():
    # after the commit, one-token decode attention over the committed cache equals attention
    # over [context, root, accepted path] taken from the uncommitted cache
    H, d, C, T = 2, 8, 7, 9
    par = [-1, 0, 0, 1, 1, 2, 4, 4, 6]
    path, n_acc = [1, 4, 6, 8, -1, -1, -1, -1, -1], 4
    k = _rand(51, 1, (C + T, H, d))
    v = _rand(51, 2, (C + T, H, d))
    q = _rand(51, 3, (1, 1, H, d))
    kc, vc = k.clone(), v.clone()
    n1 = oracle.kv_commit(kc, [C], [T], [path], [n_acc], row_off=[0])
    n2 = oracle.kv_commit(vc, [C], [T], [path], [n_acc], row_off=[0])
    assert n1 == n2 == [C + 1 + n_acc]
    # the new token sits at row new_len: give it the K/V of old row C+8's successor slot (any values)
    new_len = n1[0]
    got = oracle.tree_verify_attn(q, kc, vc, [new_len - 1], [1], [[-1]], 0.3, row_off=[0])[0, 0]
    rows = list(range(C + 1)) + [C + p for p in path[:n_acc - 1]] + [C + path[n_acc - 1]]
    want = _causal_library(q[0], k[rows], v[rows], 0.3)[0]
    assert torch.allclose(got, want, atol=1e-12)
    assert W.tree_depths(par)[8] == 4          # the path really is a root-to-node chain of that depth


# ----------------------------------------------------------------------------
# ttp_score_phead  (Sec. 5.1 Eq. 7)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_phead_score_matches_library_softmax_and_sums_to_one(dtype):
    B, H, d, M, v0 = 2, 3, 16, 29, 4
    q = _rand(61, 1, (B, H, d), 1.0, dtype)
    gq = _rand(61, 2, (B, H, d), 1.0, dtype)
    k = _rand(61, 3, (B * (v0 + M) + 3, H, d), 1.0, dtype)
    gk = _rand(61, 4, (B * (v0 + M) + 5, H, d), 1.0, dtype)
    koff = [1 + b * (v0 + M) for b in range(B)]
    goff = [2 + b * (v0 + M) for b in range(B)]
    got = oracle.ttp_score_phead(q, gq, k, gk, koff, goff, v0, M, 0.3)
    for b in range(B):
        kk = (k[koff[b] + v0:koff[b] + v0 + M].double() * gk[goff[b] + v0:goff[b] + v0 + M].double())
        qq = q[b].double() * gq[b].double()
        logits = 0.3 * torch.einsum("mhc,hc->hm", kk, qq)
        want = torch.softmax(logits, dim=1).mean(0)
        assert torch.allclose(got[b], want, atol=1e-13)
        assert abs(float(got[b].sum()) - 1.0) < 1e-13


def test_phead_score_with_unit_gates_is_the_attention_map_form():
    # gates of one, no text keys, a single non-causal query: Eq. 7 reduces to the Eq. 3 form
    H, d, M = 4, 8, 21
    q = _rand(62, 1, (1, H, d))
    k = _rand(62, 2, (M, H, d))
    ones_q, ones_k = torch.ones_like(q), torch.ones_like(k)
    a = oracle.ttp_score_phead(q, ones_q, k, ones_k, [0], [0], 0, M, 0.4)
    b = oracle.ttp_score(q[:, None].contiguous(), k, [1], [M - 1], [M], [0], 0, M, 0.4, False)
    assert torch.allclose(a, b, atol=1e-14)
    # a zero query gate makes every head uniform
    u = oracle.ttp_score_phead(q, torch.zeros_like(q), k, ones_k, [0], [0], 0, M, 0.4)
    assert torch.allclose(u, torch.full((1, M), 1.0 / M, dtype=torch.float64), atol=1e-15)


# ----------------------------------------------------------------------------
# draft-side tree build (Sec. 5.4, App. A)
# ----------------------------------------------------------------------------
def test_draft_topk_vs_stable_argsort():
    g = torch.Generator().manual_seed(3)
    probs = torch.softmax(torch.randn(5, 301, generator=g) * 3, dim=1)
    probs[1, 7:40] = probs[1, 7]                      # a plateau of equal probabilities
    probs[2] = 1.0 / 301                              # all equal
    for E in (1, 10, 64):
        ids, vals = oracle.draft_topk(probs, E)
        for r in range(5):
            order = np.argsort(-probs[r].numpy(), kind="stable")[:E]
            assert ids[r].tolist() == order.tolist()
            assert torch.equal(vals[r], probs[r][order])
    with pytest.raises(ValueError):
        oracle.draft_topk(probs, 302)


def test_draft_topk_logits_closed_forms():
    # (a) logits = log of a known distribution with distinct rational probabilities, at a shift:
    #     the winners are the known largest entries and their probabilities come back
    V, E = 200, 7
    w = np.arange(1, V + 1, dtype=np.float64)
    rng = np.random.default_rng(5)
    perm = rng.permutation(V)
    p0 = (w / w.sum())[perm]                              # p0[i] = (perm[i] + 1) / sum
    logits = torch.tensor(np.log(p0) + 3.25, dtype=torch.float32)[None]
    ids, pr = oracle.draft_topk_logits(logits, E)
    want_ids = [int(np.where(perm == V - 1 - e)[0][0]) for e in range(E)]
    assert ids[0].tolist() == want_ids
    assert np.allclose(pr[0].numpy(), [(V - e) / w.sum() for e in range(E)], rtol=3e-6, atol=0)  # fp32 logits
    # (b) one raised logit among equal ones: p = e^a / (e^a + V - 1) and (V-1) equal shares, ties by index
    a, V = 2.5, 50
    lg = torch.zeros(1, V)
    lg[0, 31] = a
    ids, pr = oracle.draft_topk_logits(lg, 4)
    assert ids[0].tolist() == [31, 0, 1, 2]
    z = np.exp(a) + V - 1
    assert np.allclose(pr[0].numpy(), [np.exp(a) / z, 1 / z, 1 / z, 1 / z], rtol=1e-14, atol=0)
    # (c) E = V: a permutation, descending, summing to one
    g = torch.Generator().manual_seed(9)
    lg = torch.randn(3, 64, generator=g) * 5
    ids, pr = oracle.draft_topk_logits(lg, 64)
    for r in range(3):
        assert sorted(ids[r].tolist()) == list(range(64))
        assert abs(float(pr[r].sum()) - 1.0) < 1e-13
        assert bool((pr[r][1:] <= pr[r][:-1]).all())
        order = np.argsort(-lg[r].numpy(), kind="stable")
        assert ids[r].tolist() == order.tolist()
    # adding a constant changes nothing; checked where the shift is exact, on a grid of 1/8
    grid = torch.round(lg * 8) / 8
    i1, p1 = oracle.draft_topk_logits(grid, 10)
    i2, p2 = oracle.draft_topk_logits(grid + 16.0, 10)
    assert torch.equal(i1, i2) and torch.allclose(p1, p2, rtol=1e-14, atol=0)
    # (d) it agrees with the probability form on a library softmax (fp64), where no two probabilities tie
    sm = torch.softmax(lg.double(), dim=1)
    ia, _ = oracle.draft_topk(sm.float(), 10)
    ib, pb = oracle.draft_topk_logits(lg, 10)
    assert torch.equal(ia, ib)
    assert torch.allclose(pb, torch.gather(sm, 1, ib.long()), rtol=1e-13, atol=0)
    # (e) very large logits do not overflow
    big = torch.tensor([[1e30, -1e30, 1e30, 0.0]])
    ids, pr = oracle.draft_topk_logits(big, 3)
    assert ids[0].tolist() == [0, 2, 3] and np.allclose(pr[0].numpy(), [0.5, 0.5, 0.0])
    with pytest.raises(ValueError):
        oracle.draft_topk_logits(lg, 65)


def _drafted_candidates(rng, E, K, D):
    """Level-wise expansion as in App. A with seeded probabilities: level 1 = E children of the
    root, each later level expands K nodes of the previous level into E children."""
    par, tok, prob, level = [], [], [], []
    prev = []
    for e in range(E):
        par.append(-1), tok.append(rng.randint(0, 31999)), prob.append(rng.uniform()), prev.append(e)
    for _ in range(1, D):
        cur = []
        for u in prev[:K]:
            for _e in range(E):
                par.append(u), tok.append(rng.randint(0, 31999)), prob.append(rng.uniform())
                cur.append(len(par) - 1)
        rng.shuffle(cur)
        prev = cur
    return par, tok, prob


@pytest.mark.parametrize("seed", range(5))
def test_tree_build_keeps_most_confident_ancestor_closed_set(seed):
    rng = W.HostRng(seed, 9)
    par, tok, prob = _drafted_candidates(rng, 4, 3, 4)
    N, T_max = len(par), 17
    n, p_out, t_out, s_out = oracle.tree_build(par, tok, prob, 123, T_max)
    assert n == min(T_max, N + 1) and int(p_out[0]) == -1 and int(t_out[0]) == 123 and int(s_out[0]) == -1
    # brute force: the product of the probabilities along each path in exact rational arithmetic
    # (the fp32 inputs are dyadic rationals), walked from the node upwards; stable order
    # (confidence desc, index asc), first T_max-1
    from fractions import Fraction
    p32 = [Fraction(float(np.float32(x))) for x in prob]
    conf = []
    for i in range(N):
        c, u = Fraction(1), i
        while u >= 0:
            c *= p32[u]
            u = par[u]
        conf.append(c)
    # the oracle's fp64 confidences are the exact products to a few units in the last place
    got = oracle.tree_confidence(par, prob)
    assert all(abs(Fraction(float(g)) - c) <= c * Fraction(1, 2 ** 50) for g, c in zip(got.tolist(), conf))
    order = sorted(range(N), key=lambda i: (-conf[i], i))[:T_max - 1]
    keep = sorted(order)
    assert s_out[1:n].tolist() == keep
    node_of = {c: 1 + r for r, c in enumerate(keep)}
    for r, c in enumerate(keep):
        assert par[c] < 0 or par[c] in node_of                       # closed under taking parents
        assert int(p_out[1 + r]) == (0 if par[c] < 0 else node_of[par[c]])
        assert int(t_out[1 + r]) == tok[c]
        assert 0 <= int(p_out[1 + r]) < 1 + r                        # topological: usable as parent[]
    assert oracle.tree_ancestors(p_out[:n].tolist())                 # accepted by the tree routines
    # every dropped candidate is no more confident than every kept one
    dropped = [i for i in range(N) if i not in node_of]
    if dropped and keep:
        assert max(conf[i] for i in dropped) <= min(conf[i] for i in keep)


def test_tree_build_special_cases():
    # fewer candidates than room: everything is kept in generation order
    n, p, t, s = oracle.tree_build([-1, 0, 1], [5, 6, 7], [0.5, 0.5, 0.5], 9, 8)
    assert n == 4 and p.tolist() == [-1, 0, 1, 2, 0, 0, 0, 0] and t.tolist() == [9, 5, 6, 7, 0, 0, 0, 0]
    assert s.tolist() == [-1, 0, 1, 2, -1, -1, -1, -1]
    # equal confidences: lower index wins, so a parent is never dropped in favour of its child
    n, p, t, s = oracle.tree_build([-1, 0, 1, 2], [1, 2, 3, 4], [1.0, 1.0, 1.0, 1.0], 0, 3)
    assert n == 3 and s.tolist() == [-1, 0, 1]
    # star: the two most probable children of the root
    n, p, t, s = oracle.tree_build([-1, -1, -1, -1], [1, 2, 3, 4], [0.1, 0.4, 0.2, 0.3], 0, 3)
    assert s.tolist() == [-1, 1, 3] and p.tolist() == [-1, 0, 0]
    # no candidates: the root alone
    n, p, t, s = oracle.tree_build([], [], [], 77, 4)
    assert n == 1 and p.tolist() == [-1, 0, 0, 0] and int(t[0]) == 77
    with pytest.raises(ValueError):
        oracle.tree_build([-1, 1], [1, 2], [0.5, 0.5], 0, 4)          # parent not before child


# ----------------------------------------------------------------------------
# level-wise drafting loop (App. A, tree-based SSD)
# ----------------------------------------------------------------------------
def _draft_tree_brute(logits, E, K, D):
    """The same loop from its definition with library routines: fp64 softmax, full sorts."""
    sm = torch.softmax(logits.double(), dim=1)
    top = lambda row: sorted(range(logits.shape[1]), key=lambda t: (-float(logits[row, t]), t))[:E]
    par, tok, prob, conf = [], [], [], []
    for t in top(0):
        par.append(-1), tok.append(t), prob.append(float(sm[0, t])), conf.append(float(sm[0, t]))
    prev, expanded = list(range(E)), []
    for _ in range(2, D + 1):
        chosen = sorted(sorted(prev, key=lambda c: (-conf[c], c))[:K])
        expanded.append(chosen)
        cur = []
        for u in chosen:
            for t in top(1 + u):
                par.append(u), tok.append(t), prob.append(float(sm[1 + u, t])), conf.append(conf[u] * float(sm[1 + u, t]))
                cur.append(len(par) - 1)
        prev = cur
    return par, tok, prob, conf, expanded


@pytest.mark.parametrize("E,K,D,V", [(3, 2, 3, 50), (4, 4, 2, 37), (2, 5, 4, 16), (5, 1, 1, 9)])
def test_draft_tree_against_its_definition(E, K, D, V):
    N = E + (D - 1) * K * E
    g = torch.Generator().manual_seed(100 * E + 10 * K + D)
    logits = torch.randn(1 + N, V, generator=g) * 2.0
    par, tok, prob, conf, exp, margin = oracle.draft_tree(logits, E, K, D)
    bp, bt, bpr, bc, bexp = _draft_tree_brute(logits, E, K, D)
    assert par.tolist() == bp and tok.tolist() == bt
    assert np.allclose(prob.numpy(), bpr, rtol=1e-12, atol=0) and np.allclose(conf.numpy(), bc, rtol=1e-12, atol=0)
    for lvl, chosen in enumerate(bexp):
        assert [c for c in exp[lvl].tolist() if c >= 0] == chosen
    # structure: parents precede children, level sizes, confidence = product along the path
    assert all(p < c for c, p in enumerate(par.tolist()))
    want_conf = oracle.tree_confidence(par.tolist(), prob.float().tolist())
    assert np.allclose(conf.numpy(), want_conf.numpy(), rtol=1e-6)
    assert (margin >= 0).all() and (margin <= 1).all()


def test_draft_tree_by_hand():
    # V = 4, E = 2, K = 1, D = 2 with probabilities chosen through their logarithms:
    # root: p = (0.5, 0.3, 0.15, 0.05) -> candidates 0 (token 0, 0.5), 1 (token 1, 0.3); the more
    # confident one (candidate 0) is expanded with p = (0.1, 0.2, 0.3, 0.4) -> tokens 3 (0.4), 2 (0.3)
    lg = torch.log(torch.tensor([[0.5, 0.3, 0.15, 0.05],
                                 [0.1, 0.2, 0.3, 0.4],     # after candidate 0
                                 [0.7, 0.1, 0.1, 0.1],     # after candidate 1: never read
                                 [0.25, 0.25, 0.25, 0.25],
                                 [0.25, 0.25, 0.25, 0.25]])).float()
    par, tok, prob, conf, exp, margin = oracle.draft_tree(lg, 2, 1, 2)
    assert par.tolist() == [-1, -1, 0, 0] and tok.tolist() == [0, 1, 3, 2]
    assert np.allclose(prob.numpy(), [0.5, 0.3, 0.4, 0.3], rtol=1e-6)
    assert np.allclose(conf.numpy(), [0.5, 0.3, 0.2, 0.15], rtol=1e-6)
    assert exp.tolist() == [[0]] and abs(float(margin[0]) - 0.4) < 1e-6      # (0.5 - 0.3) / 0.5
    with pytest.raises(ValueError):
        oracle.draft_tree(lg[:, :1].contiguous(), 2, 1, 2)      # E > V
