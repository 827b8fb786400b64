"""tw_tree_verify_attn_static (the entry point that allocates nothing: its scratch is a device array
inside the library) against tw_tree_verify_attn on the same inputs, through the C ABI, on two calls
in a row -- the second with a smaller input, so that it meets the scratch as the first left it."""
import math
import os

import pytest
import torch

from paper_2503_14075_amd import workloads as W

DEV = "cuda:0"
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tw():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_14075_amd import binding
    return binding


def _i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def _case(seed, B, H, d_h, ctx, T):
    trees = [W.random_parent_tree(W.HostRng(seed, b), T, 6) for b in range(B)]
    rows = [c + T for c in ctx]
    off, acc = [], 0
    for r in rows:
        off.append(acc)
        acc += r
    q = W.normal(seed, 1, (B, T, H, d_h), 1.0 / math.sqrt(d_h), torch.bfloat16).to(DEV)
    k = W.normal(seed, 2, (acc, H, d_h), 0.5, torch.bfloat16).to(DEV)
    v = W.normal(seed, 3, (acc, H, d_h), 0.5, torch.bfloat16).to(DEV)
    return q, k, v, _i32(off), _i32(ctx), _i32(trees), _i32([T] * B)


def test_static_scratch_entry_point_matches_the_workspace_one(tw):
    H, d_h = 32, 128
    scale = 1 / math.sqrt(d_h)
    # both launches cut their sequences into pieces (scratch in use); the first has sequences of one and of
    # several pieces side by side, the second is smaller in every dimension
    for seed, B, ctx, T in ((5, 3, [2600, 300, 1500], 40), (6, 1, [900], 26)):
        q, k, v, off, ctx_d, par, n_nodes = _case(seed, B, H, d_h, ctx, T)
        kv, vv = tw.kv_view(k, off), tw.kv_view(v, off)
        nbytes = tw.workspace_bytes(tw.TW_CALL_TREE_VERIFY_ATTN, B, T, H, d_h, max(ctx) + T)
        assert 0 < nbytes <= tw.TW_STATIC_SCRATCH_BYTES
        ws = torch.zeros(nbytes // 4, dtype=torch.float32, device=DEV)
        want = torch.full((B, T, H, d_h), float("nan"), dtype=torch.float32, device=DEV)
        tw.tree_verify_attn(q, kv, vv, ctx_d, max(ctx), par, n_nodes, scale, want, ws)
        got = torch.full_like(want, float("nan"))
        tw.tree_verify_attn_static(q, kv, vv, ctx_d, max(ctx), par, n_nodes, scale, got)
        torch.cuda.synchronize()
        assert torch.isfinite(want).all()
        # the same kernels on the same inputs with a fixed summation order: bit-identical
        assert torch.equal(got, want)


@pytest.mark.parametrize("seed", range(int(os.environ.get("TW_RANDOM_SHAPES", "8"))))
def test_static_scratch_random_shapes(tw, seed):
    # launch after launch of random shapes through the one scratch array (with and without pieces, one or
    # several per sequence): bit-identical to the entry point that takes a workspace
    rng = W.HostRng(23000 + seed)
    B, H, d_h, T = rng.randint(1, 4), (rng.randint(1, 16), rng.randint(1, 63))[rng.randint(0, 1)], (64, 128)[seed & 1], rng.randint(1, 64)
    ctx = [rng.randint(0, (300, 3000)[rng.randint(0, 1)]) for _ in range(B)]
    nbytes = tw.workspace_bytes(tw.TW_CALL_TREE_VERIFY_ATTN, B, T, H, d_h, max(ctx) + T)
    if nbytes > tw.TW_STATIC_SCRATCH_BYTES:
        pytest.skip("needs more scratch than the library holds")
    q, k, v, off, ctx_d, par, n_nodes = _case(23000 + seed, B, H, d_h, ctx, T)
    kv, vv = tw.kv_view(k, off), tw.kv_view(v, off)
    ws = torch.zeros(max(nbytes // 4, 1), dtype=torch.float32, device=DEV)
    want = torch.full((B, T, H, d_h), float("nan"), dtype=torch.float32, device=DEV)
    scale = 1 / math.sqrt(d_h)
    tw.tree_verify_attn(q, kv, vv, ctx_d, max(ctx), par, n_nodes, scale, want, ws if nbytes else None)
    got = torch.full_like(want, float("nan"))
    tw.tree_verify_attn_static(q, kv, vv, ctx_d, max(ctx), par, n_nodes, scale, got)
    torch.cuda.synchronize()
    assert torch.isfinite(want).all()
    if not torch.equal(got, want):
        # say which of the two stands alone: both calls once more
        want2, got2 = torch.full_like(want, float("nan")), torch.full_like(want, float("nan"))
        ws.zero_()
        tw.tree_verify_attn(q, kv, vv, ctx_d, max(ctx), par, n_nodes, scale, want2, ws if nbytes else None)
        tw.tree_verify_attn_static(q, kv, vv, ctx_d, max(ctx), par, n_nodes, scale, got2)
        torch.cuda.synchronize()
        d = (got != want).nonzero()
        raise AssertionError(
            f"B={B} H={H} d_h={d_h} T={T} ctx={ctx} scratch={nbytes}: {d.shape[0]} elements differ, max "
            f"{float((got - want).abs().max()):.3e}, sequences {sorted(set(d[:, 0].tolist()))} heads "
            f"{sorted(set(d[:, 2].tolist()))}; second run of the workspace call equals the first: "
            f"{torch.equal(want2, want)}, equals the static call: {torch.equal(want2, got)}; second static run "
            f"equals the first: {torch.equal(got2, got)}, equals the workspace call: {torch.equal(got2, want)}")


def test_static_scratch_serves_more_units_after_fewer(tw):
    # a launch with few (sequence, head) units, then one with many: the second one's arrival counters lie
    # where the first one must not have left anything behind
    for seed, B, H, ctx, T in ((31, 1, 2, [2000], 64), (32, 3, 80, [700, 40, 900], 8), (33, 2, 120, [600, 600], 3)):
        d_h = 64
        q, k, v, off, ctx_d, par, n_nodes = _case(seed, B, H, d_h, ctx, T)
        kv, vv = tw.kv_view(k, off), tw.kv_view(v, off)
        nbytes = tw.workspace_bytes(tw.TW_CALL_TREE_VERIFY_ATTN, B, T, H, d_h, max(ctx) + T)
        assert 0 < nbytes <= tw.TW_STATIC_SCRATCH_BYTES
        ws = torch.zeros(nbytes // 4, dtype=torch.float32, device=DEV)
        want = torch.full((B, T, H, d_h), float("nan"), dtype=torch.float32, device=DEV)
        tw.tree_verify_attn(q, kv, vv, ctx_d, max(ctx), par, n_nodes, 0.125, want, ws)
        got = torch.full_like(want, float("nan"))
        tw.tree_verify_attn_static(q, kv, vv, ctx_d, max(ctx), par, n_nodes, 0.125, got)
        torch.cuda.synchronize()
        assert torch.isfinite(want).all() and torch.equal(got, want)


def test_static_scratch_rejects_what_does_not_fit(tw):
    # 255 (sequence, head) units of 64 tree rows in two pieces each: 17 MB of partial results
    B, H, d_h, T = 85, 3, 128, 64
    ctx = [600] * B
    assert tw.workspace_bytes(tw.TW_CALL_TREE_VERIFY_ATTN, B, T, H, d_h, ctx[0] + T) > tw.TW_STATIC_SCRATCH_BYTES
    q, k, v, off, ctx_d, par, n_nodes = _case(7, B, H, d_h, ctx, T)
    out = torch.zeros((B, T, H, d_h), dtype=torch.float32, device=DEV)
    with pytest.raises(tw.TwigError) as e:
        tw.tree_verify_attn_static(q, tw.kv_view(k, off), tw.kv_view(v, off), ctx_d, ctx[0], par, n_nodes,
                                   1 / math.sqrt(d_h), out)
    assert e.value.status == tw.TW_ERR_WORKSPACE
