"""The tree changes every decode iteration (a token per live leaf, forks, pruned branches whose pages are
reused): the plan is rebuilt from the page tables each time and must stay the oracle's plan, and the
attention computed on it must stay the oracle's attention (Section 2 / Appendix A.1: the branch controller
and the KV manager change the tree between calls of the attention kernel)."""

import numpy as np
import pytest
import torch

import oracle
from oracle.plan import flatten_plan_paged
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
    for it in range(12):
        script(sim, it)
        pp, pg, nl, par, qn = sim.tables()
        Q = torch.randn((len(qn), Hq, d), generator=g).to(torch.bfloat16)
        chunk = binding.deft_suggest_chunk_size(nl, par, qn, Hq, Hkv)
        plan = binding.deft_plan_paged(pp, pg, page_size, sim.n_pool, nl, par, qn, chunk)
        got = binding.deft_tree_attn_decode(plan, Q.cuda(), Kd, Vd, out_dtype=torch.float32)
        torch.cuda.synchronize()
        ref = oracle.tree_attention_paged(Q, K, V, pp, pg, page_size, nl, par, qn)
        got = got.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref)
        print(f"    iteration {it}: nodes={len(nl)} queries={len(qn)} chunk={chunk} max|err|={err.max():.3e}", flush=True)
        # the stated tolerance, element-wise and per (query, head) row
        assert (err <= 2e-3 + 1e-2 * np.abs(ref)).all()
        assert (np.sqrt((err ** 2).sum(-1)) <= 1e-2 * np.sqrt((ref ** 2).sum(-1))).all()
