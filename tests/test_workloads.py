"""The seeded input generators: determinism, distributions, and that the
structures they emit (trees, page tables, ragged lengths) have the shape the
configurations state.  CPU only."""
import torch

from paper_2503_14075_amd import workloads as W


def test_normal_is_deterministic_and_counter_based():
    a = W.normal(3, 7, (1000, 33), 0.5, torch.float32)
    b = W.normal(3, 7, (1000, 33), 0.5, torch.float32)
    assert torch.equal(a, b)
    assert abs(float(a.mean())) < 5e-3 and abs(float(a.std()) - 0.5) < 5e-3
    c = W.normal(3, 8, (1000, 33), 0.5, torch.float32)
    assert not torch.equal(a, c)
    # a prefix of a longer stream is the same stream
    d = W.normal(3, 7, (2000, 33), 0.5, torch.float32)
    assert torch.equal(d[:1000], a)


def test_trees_respect_caps():
    for seed in range(5):
        par = W.random_parent_tree(W.HostRng(seed, 1), 64, 6)
        assert par[0] == -1 and all(0 <= p < i for i, p in enumerate(par) if i)
        assert max(W.tree_depths(par)) <= 6
    par = W.fanout_tree(W.HostRng(1, 1), 26, (4, 3, 2, 1, 1))
    assert len(par) == 26 and par[0] == -1 and all(0 <= p < i for i, p in enumerate(par) if i)
    dep = W.tree_depths(par)
    assert max(dep) <= 5 and dep == sorted(dep)
    kids = [par.count(u) for u in range(26)]
    assert all(k <= (4, 3, 2, 1, 1, 0)[d] for k, d in zip(kids, dep))


def test_config_shapes():
    w = W.make_workload(W.CONFIGS["cfg0"])
    assert w.k_score.shape == (608, 4, 64) and w.q_sel.shape == (1, 8, 4, 64)
    assert w.ctx_len == [96] and w.k_pool.shape == (104, 4, 64) and w.k_pool.dtype == torch.float32
    assert len(w.compact_src) == 3 and w.compact_src[0].shape == (608, 256)
    w = W.make_workload(W.CONFIGS["cfg1"], with_compact=False)
    assert w.ctx_len == [256] and w.n_q == [64] and w.k_pool.shape == (282, 32, 128)
    assert w.k_pool.dtype == torch.bfloat16
    w = W.make_workload(W.replicate(W.CONFIGS["cfg3"], 4), with_compact=False, with_score=False)
    assert w.page_table is not None and len(w.page_table) == 4
    flat = [p for b in range(4) for p in w.page_table[b][:(w.ctx_len[b] + 32 + 15) // 16]]
    assert len(set(flat)) == len(flat)                       # pages are not shared
    for b in range(4):
        assert 32 <= w.n_text[b] <= 128 and 64 + w.n_text[b] <= w.ctx_len[b] <= 64 + w.n_text[b] + 512
        rows = W.instance_rows(w, b)
        assert rows.numel() == w.ctx_len[b] + 32 and int(rows.max()) < w.k_pool.shape[0]


def test_planted_tokens_give_nontrivial_paths():
    rng = W.HostRng(9, 9)
    par = W.random_parent_tree(rng, 32, 5)
    hits = 0
    for s in range(50):
        d, a = W.plant_tokens(W.HostRng(s, 3), par)
        hits += sum(d[c] == a[par[c]] for c in range(1, 32))
        assert all(0 <= x < 32000 for x in d + a)
    assert hits > 50
