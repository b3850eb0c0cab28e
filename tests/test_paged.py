"""Paged KV cache (Section 4.2 of the paper: tokens of a node scattered over pages of one pool, nothing
materialised): oracle pins and planner parity on the CPU, GPU parity against the oracle."""

from collections import Counter

import numpy as np
import pytest
import torch

import oracle
from oracle.plan import PlanError, flatten_plan, flatten_plan_paged
from paper_2404_00242_amd import binding, workloads as wl

ARRAYS = ("q_order", "node_q_lo", "node_q_hi", "chunk_seg_ptr", "seg_tok_begin", "seg_len", "seg_qlo", "seg_qhi",
          "seg_node", "chunk_qlo", "chunk_qhi", "chunk_slot_base", "seg_mask_ptr", "seg_mask", "q_part_ptr",
          "q_part_chunk", "q_part_slot")


def paged_case(seed, page_size, **kw):
    t = wl.random_tree(seed, **kw)
    Q, K, V = wl.make_qkv(t)
    pp, pg, npool, row_of = wl.to_paged(t, page_size, seed=seed)
    Kp = wl.scatter_to_pool(K, row_of, npool * page_size, 1)
    Vp = wl.scatter_to_pool(V, row_of, npool * page_size, 2)
    return t, (Q, K, V), (pp, pg, npool), (Kp, Vp), row_of


@pytest.mark.parametrize("seed,page_size", [(0, 16), (1, 1), (2, 4), (3, 32), (4, 7)])
def test_oracle_moving_tokens_into_pages_leaves_outputs_unchanged(seed, page_size):
    t, (Q, K, V), (pp, pg, npool), (Kp, Vp), _ = paged_case(seed, page_size, n_nodes=9, max_len=40, nq=7, Hq=4,
                                                               Hkv=2, d=16)
    ref = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    got = oracle.tree_attention_paged(Q, Kp, Vp, pp, pg, page_size, t.node_tok_len, t.node_parent, t.query_node)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


def test_oracle_pages_in_pool_order_are_a_contiguous_cache():
    # nodes whose lengths are whole pages, pages handed out in order: the pool *is* the contiguous cache
    lens = [32, 16, 48, 16]
    t = wl._finish("aligned", lens, [-1, 0, 0, 2], [1, 3, 3], 4, 2, 8, 9)
    Q, K, V = wl.make_qkv(t)
    pp, pg, npool, row_of = wl.to_paged(t, 16, shuffle=False, spare_pages=0)
    assert np.array_equal(row_of, np.arange(t.ntok))
    a = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    b = oracle.tree_attention_paged(Q, K, V, pp, pg, 16, t.node_tok_len, t.node_parent, t.query_node)
    assert np.array_equal(a, b)
    # and its plan is the contiguous plan: consecutive pages are joined into one run per node
    p1 = flatten_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 32)
    p2 = flatten_plan_paged(pp, pg, 16, npool, t.node_tok_len, t.node_parent, t.query_node, 32)
    for a_ in ARRAYS:
        assert np.array_equal(p1[a_], p2[a_]), a_


@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("mode", ["flatten", "node", "node_chunk", "query", "balanced"])
def test_paged_plan_covers_every_pair_once_and_matches_the_planner(seed, mode):
    page_size = [1, 4, 16, 16, 5][seed % 5]
    t = wl.random_tree(600 + seed, n_nodes=2 + seed, max_len=60, nq=1 + 2 * seed, n_roots=1 + seed % 2)
    pp, pg, npool, row_of = wl.to_paged(t, page_size, seed=seed)
    B = 32
    G = 4 if mode == "balanced" else 1
    ref = flatten_plan_paged(pp, pg, page_size, npool, t.node_tok_len, t.node_parent, t.query_node, B, mode, G)
    # coverage against an independent walk: (query, pool row) pairs, each once
    want = Counter()
    for j, u in enumerate(t.query_node):
        u = int(u)
        while u >= 0:
            for r in range(int(t.node_tok_begin[u]), int(t.node_tok_begin[u] + t.node_tok_len[u])):
                want[(j, int(row_of[r]))] += 1
            u = int(t.node_parent[u])
    got = Counter()
    for s in range(ref["n_segs"]):
        for pos in range(int(ref["seg_qlo"][s]), int(ref["seg_qhi"][s])):
            for r in range(int(ref["seg_tok_begin"][s]), int(ref["seg_tok_begin"][s] + ref["seg_len"][s])):
                got[(int(ref["q_order"][pos]), r)] += 1
    assert got == want
    # no segment crosses a page boundary unless the pages are neighbours in the pool
    if mode == "flatten":
        assert ref["n_chunks"] == -(-ref["n_flat"] // B)
    # the C++ planner gives the same arrays
    view = binding.deft_plan_paged(pp, pg, page_size, npool, t.node_tok_len, t.node_parent, t.query_node, B,
                                   binding.SPLIT_MODES[mode] | (binding.rows_per_query(G) if G > 1 else 0)).view()
    for a in ARRAYS:
        assert np.array_equal(view[a], ref[a]), a


def test_a_node_too_long_for_one_chunk_and_scattered_over_pages_is_refused_at_plan_time():
    """DeFT-Node makes one chunk per node whatever its length.  A chunk of several pieces is expanded by the
    kernels into a table of at most DEFT_MAX_CHUNK = 4096 entries, so a longer node whose pages are not one run
    cannot be decoded: the planner says so (DEFT_EINVAL) instead of handing out a plan that fails at launch.
    The same node in one run of pages, or cut by any other split, is fine."""
    P, n = 16, 5000
    pages = -(-n // P)
    ptr = [0, pages, pages + 1]
    scattered = list(range(pages - 1, -1, -1)) + [pages]     # the node's pages in reverse pool order
    in_order = list(range(pages + 1))
    args = dict(page_size=P, n_pool_pages=pages + 1, node_tok_len=[n, 3], node_parent=[-1, 0], query_node=[1, 1])
    with pytest.raises(binding.DeftError) as e:
        binding.deft_plan_paged(ptr, scattered, chunk_size=128, flags=binding.DEFT_SPLIT_NODE, **args)
    assert e.value.status == -1
    v = binding.deft_plan_paged(ptr, in_order, chunk_size=128, flags=binding.DEFT_SPLIT_NODE, **args).view()
    assert v["n_chunks"] == 2 and int(v["seg_len"].max()) == n
    for mode in ("flatten", "node_chunk", "balanced", "query"):
        v = binding.deft_plan_paged(ptr, scattered, chunk_size=4096, flags=binding.SPLIT_MODES[mode], **args).view()
        lens = [int(v["seg_len"][v["chunk_seg_ptr"][c]:v["chunk_seg_ptr"][c + 1]].sum()) for c in range(v["n_chunks"])]
        assert max(lens) <= 4096


def test_paged_planner_rejects_bad_page_tables():
    ok = dict(node_page_ptr=[0, 2, 3], page_ids=[5, 1, 0], page_size=4, n_pool_pages=8, node_tok_len=[7, 3],
              node_parent=[-1, 0], query_node=[1], chunk_size=32)
    binding.deft_plan_paged(**ok)
    flatten_plan_paged(**ok)
    for bad in (dict(page_ids=[5, 1, 5]), dict(page_ids=[5, 1, 9]), dict(node_tok_len=[9, 3]), dict(page_size=0),
                dict(node_page_ptr=[1, 2, 3]), dict(page_ids=[5, -1, 0])):
        args = dict(ok)
        args.update(bad)
        with pytest.raises(binding.DeftError):
            binding.deft_plan_paged(**args)
        with pytest.raises(PlanError):
            flatten_plan_paged(**args)


@pytest.mark.gpu
@pytest.mark.parametrize("seed,page_size", [(0, 16), (1, 1), (2, 4), (3, 32), (4, 7), (5, 16)])
def test_gpu_paged_random_trees(seed, page_size):
    t, (Q, K, V), (pp, pg, npool), (Kp, Vp), _ = paged_case(700 + seed, page_size, n_nodes=4 + 3 * seed, max_len=150,
                                                               nq=3 + 5 * seed, Hq=8, Hkv=2, d=128, n_roots=1 + seed % 2)
    ref = oracle.tree_attention_paged(Q, Kp, Vp, pp, pg, page_size, t.node_tok_len, t.node_parent, t.query_node)
    dev = torch.device("cuda:0")
    for chunk in (64, 256):
        plan = binding.deft_plan_paged(pp, pg, page_size, npool, t.node_tok_len, t.node_parent, t.query_node, chunk)
        got = binding.deft_tree_attn_decode(plan, Q.to(dev), Kp.to(dev), Vp.to(dev), out_dtype=torch.float32)
        torch.cuda.synchronize()
        got = got.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        num, den = np.sqrt((err ** 2).sum(-1)), np.sqrt((ref ** 2).sum(-1))
        print(f"    chunk {chunk}: max|err|={err.max():.3e} max row-rel={(num / np.maximum(den, 1e-300)).max():.3e}", flush=True)
        # the stated tolerance, element-wise and per (query, head) row
        assert np.isfinite(got).all() and (err <= 2e-3 + 1e-2 * np.abs(ref)).all(), err.max()
        assert (num <= 1e-2 * den).all()


@pytest.mark.gpu
@pytest.mark.parametrize("cfg,page_size", [(2, 16), (3, 16), (2, 1)])
def test_gpu_paged_benchmark_trees(cfg, page_size):
    t = wl.make_config(cfg)
    Q, K, V = wl.make_qkv(t)
    pp, pg, npool, row_of = wl.to_paged(t, page_size, seed=cfg)
    Kp = wl.scatter_to_pool(K, row_of, npool * page_size, 1)
    Vp = wl.scatter_to_pool(V, row_of, npool * page_size, 2)
    ref = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    dev = torch.device("cuda:0")
    chunk = binding.deft_suggest_chunk_size(t.node_tok_len, t.node_parent, t.query_node, t.Hq, t.Hkv)
    plan = binding.deft_plan_paged(pp, pg, page_size, npool, t.node_tok_len, t.node_parent, t.query_node, chunk)
    got = binding.deft_tree_attn_decode(plan, Q.to(dev), Kp.to(dev), Vp.to(dev))
    torch.cuda.synchronize()
    got = got.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    print(f"\n  config {cfg} page {page_size}: max|err|={err.max():.3e} segments={plan.view()['n_segs']}", flush=True)
    assert err.max() <= 2e-3
