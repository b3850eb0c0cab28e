"""deft_tree_attn_decode_static, the entry point for callers that cannot allocate: its partial results live in
a fixed array inside the library's device code instead of a caller workspace.  It runs the same kernels as
deft_tree_attn_decode, so its output must be that call's output bit for bit, also on a second call with a
smaller tree that leaves the first call's partial results behind in the array."""

import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2404_00242_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

STATIC_BYTES = 64 << 20  # DEFT_STATIC_SCRATCH_BYTES of include/deft.h


def both_ways(t, chunk, out_dtype):
    """(output of the static-workspace call, output of the ordinary call, plan) for one tree"""
    dev = torch.device("cuda:0")
    lib = binding.load_library()
    Q, K, V = wl.make_qkv(t)
    q, k, v = Q.to(dev), K.to(dev), V.to(dev)
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, chunk)
    want = binding.deft_tree_attn_decode(plan, q, k, v, out_dtype=out_dtype)
    got = torch.full_like(want, float("nan"))
    img = plan.image(t.Hq, t.Hkv, dev)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    flags = binding.DEFT_OUT_F32 if out_dtype == torch.float32 else binding.DEFT_OUT_BF16
    rc = lib.deft_tree_attn_decode_static(plan.handle, img.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                          got.data_ptr(), t.Hq, t.Hkv, t.d, 0.0, flags, st)
    assert rc == 0, (rc, lib.deft_last_hip_error())
    torch.cuda.synchronize()
    return got, want, plan, (Q, K, V)


def test_static_workspace_call_equals_the_ordinary_call_twice_in_a_row():
    # first a tree with wide groups and many slots, then a much smaller one: the array still holds the first
    # call's partial results when the second call runs
    big = wl._finish("star", [700] + [40] * 90, [-1] + [0] * 90, list(range(1, 91)), 8, 2, 128, 31)
    small = wl.random_tree(12, n_nodes=7, max_len=90, nq=5, Hq=8, Hkv=2, d=128)
    for t, chunk, dt in ((big, 128, torch.float32), (small, 64, torch.bfloat16)):
        got, want, plan, (Q, K, V) = both_ways(t, chunk, dt)
        print(f"\n  {t.name}: nq={t.nq} ntok={t.ntok} slots={plan.view()['n_slots']} "
              f"workspace={plan.workspace_bytes(t.Hq, t.Hkv, t.d)} B", flush=True)
        assert torch.equal(got, want)
        # and both are the attention: the five benchmark configurations' bound
        ref = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
        err = np.abs(got.float().cpu().numpy().astype(np.float64) - ref)
        assert (err <= 2e-3 + 1e-2 * np.abs(ref)).all(), err.max()


def test_plans_that_need_more_than_the_array_are_refused_before_any_launch():
    dev = torch.device("cuda:0")
    lib = binding.load_library()
    # 400 queries on one 1600-token node in chunks of 32: 20000 slots x 32 heads x 130 floats = 333 MB
    t = wl._finish("too_wide", [1600], [-1], [0] * 400, 32, 8, 128, 5)
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 32)
    assert plan.workspace_bytes(t.Hq, t.Hkv, t.d) > STATIC_BYTES
    img = plan.image(t.Hq, t.Hkv, dev)
    q = torch.zeros((t.nq, t.Hq, t.d), dtype=torch.bfloat16, device=dev)
    k = torch.zeros((t.ntok, t.Hkv, t.d), dtype=torch.bfloat16, device=dev)
    o = torch.full((t.nq, t.Hq, t.d), 7.0, dtype=torch.bfloat16, device=dev)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.deft_tree_attn_decode_static(plan.handle, img.data_ptr(), q.data_ptr(), k.data_ptr(), k.data_ptr(),
                                          o.data_ptr(), t.Hq, t.Hkv, t.d, 0.0, 0, st)
    assert rc == -3
    torch.cuda.synchronize()
    assert bool((o == 7.0).all())  # nothing ran
    # bad head shape: refused as by the ordinary call
    rc = lib.deft_tree_attn_decode_static(plan.handle, img.data_ptr(), q.data_ptr(), k.data_ptr(), k.data_ptr(),
                                          o.data_ptr(), t.Hq, t.Hkv, 96, 0.0, 0, st)
    assert rc == -1
