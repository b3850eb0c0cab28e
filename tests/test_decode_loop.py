"""The tree changes every decode iteration (a token per live leaf, forks, pruned branches whose pages are
reused): the plan is rebuilt from the page tables each time and must stay the oracle's plan, and the
attention computed on it must stay the oracle's attention (Section 2 / Appendix A.1: the branch controller
and the KV manager change the tree between calls of the attention kernel)."""

import numpy as np
import pytest
import torch

import oracle
from oracle.plan import flatten_plan, flatten_plan_paged
from paper_2404_00242_amd import binding, workloads as wl

ARRAYS = ("q_order", "chunk_seg_ptr", "seg_tok_begin", "seg_len", "seg_qlo", "seg_qhi", "seg_node", "chunk_qlo",
          "chunk_qhi", "chunk_slot_base", "seg_mask_ptr", "seg_mask", "q_part_ptr", "q_part_chunk", "q_part_slot")


def script(sim, it):
    sim.step()
    if it % 3 == 1:
        sim.branch(2 + it % 2)
    if it % 4 == 3:
        sim.prune(2)


@pytest.mark.parametrize("seed,page_size,chunk", [(0, 16, 64), (1, 4, 32), (2, 1, 128)])
def test_replanned_tables_stay_the_oracles_plan(seed, page_size, chunk):
    sim = wl.DecodeLoopSim(seed, prompt_len=150, width=5, page_size=page_size, n_pool_pages=4000 // page_size)
    for it in range(14):
        script(sim, it)
        pp, pg, nl, par, qn = sim.tables()
        want = flatten_plan_paged(pp, pg, page_size, sim.n_pool, nl, par, qn, chunk)
        got = binding.deft_plan_paged(pp, pg, page_size, sim.n_pool, nl, par, qn, chunk).view()
        for a in ARRAYS:
            assert np.array_equal(got[a], want[a]), (it, a)
    # pruned branches gave pages back and new nodes took them
    assert len(sim.free) + sum(len(p) for p in sim.pages) == sim.n_pool


ALL_ARRAYS = ARRAYS + ("node_q_lo", "node_q_hi")


def same_plan(got, want, what):
    for key in ("n_flat", "n_chunks", "n_segs", "n_slots", "nq", "n_nodes", "chunk_size"):
        assert got[key] == want[key], (what, key)
    for a in ALL_ARRAYS:
        assert np.array_equal(got[a], want[a]), (what, a)


@pytest.mark.parametrize("mode", ["flatten", "balanced", "node", "node_chunk", "query"])
@pytest.mark.parametrize("seed,page_size,chunk", [(0, 16, 64), (1, 4, 32), (2, 1, 128), (3, 16, 256)])
def test_plans_updated_from_the_previous_iteration_are_the_oracles_plans(seed, page_size, chunk, mode):
    """deft_plan_paged_update, fed the plan of the iteration before: bit for bit the plan of a full re-plan (the
    oracle's), whatever changed in between: a token per leaf (pages filling up and new pages), forks that add
    nodes and move queries, prunes that empty nodes and hand their pages to later nodes."""
    G = 4
    flags = binding.SPLIT_MODES[mode] | (binding.rows_per_query(G) if mode == "balanced" else 0)
    sim = wl.DecodeLoopSim(10 + seed, prompt_len=300, width=6, page_size=page_size, n_pool_pages=6000 // page_size)
    prev = None
    for it in range(16):
        script(sim, it)
        pp, pg, nl, par, qn = sim.tables()
        want = flatten_plan_paged(pp, pg, page_size, sim.n_pool, nl, par, qn, chunk, mode, G)
        plan = binding.deft_plan_paged(pp, pg, page_size, sim.n_pool, nl, par, qn, chunk, flags, prev=prev)
        same_plan(plan.view(), want, (it, mode))
        prev = plan


@pytest.mark.parametrize("mode", ["flatten", "balanced", "node_chunk"])
def test_updates_of_a_contiguous_cache_under_random_changes(mode):
    """deft_plan_update on node-contiguous trees: lengths of random nodes grow or shrink (the cache has room
    behind every node), queries move, nodes are re-parented, chunk size or split change; after every change the
    updated plan equals the oracle's plan of the new tree, and a refused tree is refused with the old plan too."""
    rng = np.random.default_rng(77)
    G = 2
    for trial in range(12):
        n = int(rng.integers(2, 20))
        cap = 200                                      # every node owns a slot of `cap` rows, so lengths may change freely
        par = np.full(n, -1, dtype=np.int64)
        for u in range(1, n):
            par[u] = rng.integers(0, u) if rng.random() < 0.9 else -1
        lens = rng.integers(0, cap, size=n)
        begins = np.arange(n) * cap
        qn = rng.integers(0, n, size=int(rng.integers(1, 30)))
        chunk, cur_mode = 64, mode
        prev = None
        for step in range(14):
            kind = int(rng.integers(0, 7)) if step else -1
            if kind in (0, 1, 2):                      # the usual case: some nodes (leaves, mostly) gain a token or a few
                for u in rng.choice(n, size=int(rng.integers(1, n + 1)), replace=False):
                    lens[u] = min(cap, lens[u] + int(rng.integers(1, 4)))
            elif kind == 3:                            # a node is emptied (pruned) or shortened
                lens[int(rng.integers(n))] = int(rng.integers(0, 5))
            elif kind == 4:                            # queries move
                qn = rng.integers(0, n, size=int(rng.integers(1, 30)))
            elif kind == 5 and n > 2:                  # a node is hung somewhere else (never under a descendant: under a smaller id)
                u = int(rng.integers(1, n))
                par[u] = int(rng.integers(0, u))
            elif kind == 6:
                chunk = int(rng.choice([32, 64, 128]))
            flags = binding.SPLIT_MODES[cur_mode] | (binding.rows_per_query(G) if cur_mode == "balanced" else 0)
            want = flatten_plan(begins, lens, par, qn, n * cap, chunk, cur_mode, G)
            plan = binding.deft_plan(begins, lens, par, qn, n * cap, chunk, flags, prev=prev)
            same_plan(plan.view(), want, (trial, step, kind))
            # an invalid tree is refused with a previous plan exactly as without one, and the previous plan survives
            bad = lens.copy()
            victims = [u for u in range(n - 1) if lens[u + 1] > 5]
            if victims:
                bad[victims[int(rng.integers(len(victims)))]] = cap + 5   # runs into the rows of the node behind it
                with pytest.raises(binding.DeftError):
                    binding.deft_plan(begins, bad, par, qn, n * cap, chunk, flags, prev=plan)
                same_plan(plan.view(), want, "after a refused update")
            prev = plan


@pytest.mark.gpu
@pytest.mark.parametrize("seed,page_size", [(0, 16), (1, 1)])
def test_decode_iterations_on_a_changing_tree_match_the_oracle(seed, page_size):
    Hq, Hkv, d = 8, 2, 128
    sim = wl.DecodeLoopSim(seed, prompt_len=700, width=6, page_size=page_size, n_pool_pages=6000 // page_size)
    g = torch.Generator().manual_seed(100 + seed)
    rows = sim.n_pool * page_size
    K = torch.randn((rows, Hkv, d), generator=g).to(torch.bfloat16)
    V = torch.randn((rows, Hkv, d), generator=g).to(torch.bfloat16)
    Kd, Vd = K.cuda(), V.cuda()
    plan = None  # every iteration's plan is an update of the one before
    for it in range(12):
        script(sim, it)
        pp, pg, nl, par, qn = sim.tables()
        Q = torch.randn((len(qn), Hq, d), generator=g).to(torch.bfloat16)
        chunk = binding.deft_suggest_chunk_size(nl, par, qn, Hq, Hkv)
        plan = binding.deft_plan_paged(pp, pg, page_size, sim.n_pool, nl, par, qn, chunk, prev=plan)
        got = binding.deft_tree_attn_decode(plan, Q.cuda(), Kd, Vd, out_dtype=torch.float32)
        torch.cuda.synchronize()
        ref = oracle.tree_attention_paged(Q, K, V, pp, pg, page_size, nl, par, qn)
        got = got.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        print(f"    iteration {it}: nodes={len(nl)} queries={len(qn)} chunk={chunk} max|err|={err.max():.3e}", flush=True)
        # the stated tolerance, element-wise and per (query, head) row
        assert (err <= 2e-3 + 1e-2 * np.abs(ref)).all()
        assert (np.sqrt((err ** 2).sum(-1)) <= 1e-2 * np.sqrt((ref ** 2).sum(-1))).all()
