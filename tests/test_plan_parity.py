"""deft_plan (C++ host code behind the C ABI) against the oracle's plan: bit-exact, CPU only."""

import ctypes
import glob
import json
import os

import numpy as np
import pytest

from oracle.plan import PlanError, flatten_plan
from paper_2404_00242_amd import binding, workloads as wl

ARRAYS = ("q_order", "node_q_lo", "node_q_hi", "chunk_seg_ptr", "seg_tok_begin", "seg_len", "seg_qlo", "seg_qhi",
          "seg_node", "chunk_qlo", "chunk_qhi", "chunk_slot_base", "seg_mask_ptr", "seg_mask", "q_part_ptr",
          "q_part_chunk", "q_part_slot")
SCALARS = ("chunk_size", "n_nodes", "nq", "n_flat", "n_chunks", "n_segs", "n_slots")


def assert_same_plan(t, B, mode="flatten", G=1):
    ref = flatten_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, B, mode, G)
    got = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, B,
                            binding.SPLIT_MODES[mode] | (binding.rows_per_query(G) if G > 1 else 0)).view()
    for s in SCALARS:
        assert got[s] == ref[s], s
    assert got["n_mask_words"] == len(ref["seg_mask"])
    for a in ARRAYS:
        assert got[a].dtype == ref[a].dtype, a
        assert np.array_equal(got[a], ref[a]), a


def test_library_exports_every_declared_symbol(repo_root):
    lib = binding.load_library()
    header = open(os.path.join(repo_root, "include", "deft.h")).read()
    import re

    declared = set(re.findall(r"\b(deft_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.deft_strerror(0) == b"ok" and lib.deft_strerror(-3) != lib.deft_strerror(-1)


def test_public_header_is_plain_c(repo_root, tmp_path):
    """The boundary is a C ABI: its header must compile as C99 (and as C++) with nothing but itself."""
    import shutil
    import subprocess

    src = tmp_path / "use_header.c"
    src.write_text('#include "deft.h"\nint main(void) { deft_plan_view_t v; (void)v; return DEFT_OK; }\n')
    inc = os.path.join(repo_root, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)],
                   check=True)
    if shutil.which("g++"):
        subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c++",
                        "-I", inc, str(src)], check=True)


@pytest.mark.parametrize("cfg,B", [(1, 128), (1, 32), (2, 128), (2, 256), (3, 128), (3, 32), (4, 128), (5, 128),
                                   (5, 1024)])
def test_benchmark_configs(cfg, B):
    assert_same_plan(wl.make_config(cfg), B)


def test_tiny_variant_with_320_tokens():
    assert_same_plan(wl.config1_tiny(leaf_len=16), 128)


@pytest.mark.parametrize("seed", range(60))
def test_random_forests(seed):
    t = wl.random_tree(seed, n_nodes=1 + seed % 23, max_len=150, nq=(seed * 5) % 31, n_roots=1 + seed % 4,
                       zero_len_prob=0.15)
    for B in (32, 96, 128):
        assert_same_plan(t, B)


def test_wide_group_masks():
    t = wl._finish("star", [100] + [3] * 150, [-1] + [0] * 150, list(range(1, 151)), 2, 1, 8, 1)
    assert_same_plan(t, 32)
    t = wl._finish("star64", [70] + [1] * 64, [-1] + [0] * 64, list(range(1, 65)), 2, 1, 8, 1)
    assert_same_plan(t, 64)


@pytest.mark.parametrize("path", sorted(glob.glob(os.path.join(os.path.dirname(__file__), "golden", "plan_*.json"))))
def test_hand_derived_fixtures(path):
    g = json.load(open(path))
    i = g["input"]
    flags = binding.SPLIT_MODES[i.get("mode", "flatten")] | binding.rows_per_query(i.get("rows_per_query", 0))
    got = binding.deft_plan(i["node_tok_begin"], i["node_tok_len"], i["node_parent"], i["query_node"], i["ntok"],
                            i["chunk_size"], flags).view()
    for key, want in g["expect"].items():
        assert (got[key].tolist() if isinstance(want, list) else got[key]) == want, key


@pytest.mark.parametrize("bad", [
    dict(node_parent=[0, 0]), dict(node_parent=[1, 0]), dict(node_parent=[-1, 5]), dict(node_parent=[-2, 0]),
    dict(node_tok_begin=[0, 2]), dict(node_tok_len=[4, 9]), dict(node_tok_len=[4, -1]), dict(node_tok_begin=[-1, 4]),
    dict(query_node=[2]), dict(query_node=[-1]), dict(chunk_size=48), dict(chunk_size=-32), dict(chunk_size=8192),
    dict(ntok=-1),
])
def test_invalid_inputs_return_einval_like_the_oracle(bad):
    args = dict(node_tok_begin=[0, 4], node_tok_len=[4, 4], node_parent=[-1, 0], query_node=[1], ntok=8, chunk_size=32)
    args.update(bad)
    with pytest.raises(binding.DeftError) as e:
        binding.deft_plan(**args)
    assert e.value.status == -1
    if bad.get("chunk_size") != 8192:   # the size cap is a property of the kernels, not of the method
        with pytest.raises(PlanError):
            flatten_plan(**args)


def test_null_pointers_and_degenerate_trees():
    lib = binding.load_library()
    out = ctypes.c_void_p(1234)
    assert lib.deft_plan(None, None, None, 1, None, 0, 0, 0, 0, ctypes.byref(out)) == -1
    assert out.value is None
    assert lib.deft_plan_view(None, None) == -1
    assert lib.deft_plan_device_bytes(None, 4, 2) == 0
    assert lib.deft_workspace_bytes(None, 4, 2, 128) == 0
    lib.deft_plan_destroy(None)
    # no queries / no tokens: empty plans, like the oracle's
    for args in (([0], [10], [-1], [], 10), ([0, 0], [0, 0], [-1, 0], [1], 0)):
        ref = flatten_plan(*args, 32)
        got = binding.deft_plan(*args, 32).view()
        for a in ARRAYS:
            assert np.array_equal(got[a], ref[a]), a
    p = binding.deft_plan([0], [10], [-1], [0], 10, 0)
    assert p.view()["chunk_size"] == 128
    assert p.device_bytes(4, 3) == 0 and p.device_bytes(4, 2) > 0
    assert p.workspace_bytes(4, 2, 96) == 0 and p.workspace_bytes(4, 2, 128) >= 1 * 4 * 130 * 4


def test_large_chain_is_planned_quickly():
    # 50k nodes in one path: linear-time preorder and cycle check, no recursion
    n = 50_000
    lens = np.full(n, 3, np.int32)
    par = np.arange(-1, n - 1, dtype=np.int32)
    beg = (np.arange(n, dtype=np.int64) * 3).astype(np.int32)
    v = binding.deft_plan(beg, lens, par, [n - 1, n // 2], 3 * n, 128).view()
    assert v["n_flat"] == 3 * n and v["n_chunks"] == -(-3 * n // 128)


def test_suggested_chunk_size():
    for cfg in range(1, 6):
        t = wl.make_config(cfg)
        c = binding.deft_suggest_chunk_size(t.node_tok_len, t.node_parent, t.query_node, t.Hq, t.Hkv)
        assert 128 <= c <= 1024 and c % 128 == 0
        assert_same_plan(t, c)     # whatever it suggests, the plan is still the oracle's plan
    # few-shot: about 512 tasks of (chunk, KV head)
    t = wl.make_config(2)
    c = binding.deft_suggest_chunk_size(t.node_tok_len, t.node_parent, t.query_node, t.Hq, t.Hkv)
    assert 400 <= -(-t.ntok // c) * t.Hkv <= 512
    with pytest.raises(binding.DeftError):
        binding.deft_suggest_chunk_size([4, 4], [1, 0], [1], 4, 2)      # cycle
    with pytest.raises(binding.DeftError):
        binding.deft_suggest_chunk_size([4, 4], [-1, 0], [1], 4, 3)     # Hq % Hkv != 0
    with pytest.raises(binding.DeftError):
        binding.deft_suggest_chunk_size([4, 4], [-1, 0], [7], 4, 2)     # query node out of range


@pytest.mark.parametrize("mode", ["node", "node_chunk", "query"])
def test_other_partitioning_strategies(mode):
    for seed in range(30):
        t = wl.random_tree(400 + seed, n_nodes=1 + seed % 17, max_len=120, nq=(seed * 3) % 19, n_roots=1 + seed % 3,
                           zero_len_prob=0.15)
        for B in (32, 128):
            assert_same_plan(t, B, mode)
    for cfg in (1, 2, 3):
        assert_same_plan(wl.make_config(cfg), 128, mode)
    with pytest.raises(binding.DeftError):
        binding.deft_plan([0], [4], [-1], [0], 4, 32, 7)       # unknown strategy
    with pytest.raises(binding.DeftError):
        binding.deft_suggest_chunk_size([4], [-1], [0], 4, 2, 7)


def test_balanced_split_matches_the_oracle():
    # the tokens x rows split needs the number of query heads per KV head; wide and narrow groups, several sizes
    for seed in range(60):
        G = [1, 2, 4, 8, 5][seed % 5]
        t = wl.random_tree(900 + seed, n_nodes=1 + seed % 23, max_len=150, nq=(seed * 3) % 41, n_roots=1 + seed % 3,
                           zero_len_prob=0.1)
        for B in (32, 64, 256):
            assert_same_plan(t, B, "balanced", G)
    for cfg in (1, 2, 3, 4, 5):
        t = wl.make_config(cfg)
        for B in (128, 768):
            assert_same_plan(t, B, "balanced", t.Hq // t.Hkv)
    # a very wide, very long node: chunks stop at DEFT_MAX_CHUNK tokens whatever the stretch
    t = wl._finish("wide", [20000, 8], [-1, 0], [1] * 200, 8, 2, 128, 3)
    assert_same_plan(t, 2048, "balanced", 4)
    v = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 2048,
                          binding.DEFT_SPLIT_BALANCED | binding.rows_per_query(4)).view()
    assert int(v["seg_len"].max()) == 4096
    with pytest.raises(binding.DeftError):   # bits outside the mode, the weights flag and the rows field
        binding.deft_plan([0], [4], [-1], [0], 4, 32, binding.DEFT_SPLIT_BALANCED | 0x200)


def test_corrupted_trees_are_accepted_or_refused_exactly_as_by_the_oracle():
    """400 valid random forests with one to three random corruptions each (parent, length, position, query,
    chunk size, cache size): the planner returns an error exactly when the oracle's validation raises, and when
    both accept, the plans are equal."""
    rng = np.random.default_rng(77)
    refused = accepted = 0
    for it in range(400):
        t = wl.random_tree(9000 + it, n_nodes=int(rng.integers(1, 12)), max_len=int(rng.integers(1, 50)),
                           nq=int(rng.integers(0, 9)), n_roots=int(rng.integers(1, 3)))
        nb, nl, par, qn = (np.array(x, dtype=np.int64) for x in
                           (t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node))
        ntok, chunk = int(t.ntok), 32
        for _ in range(int(rng.integers(1, 4))):
            kind = int(rng.integers(6))
            u = int(rng.integers(len(nb)))
            if kind == 0:
                par[u] = int(rng.integers(-3, len(nb) + 2))
            elif kind == 1:
                nl[u] = int(rng.integers(-2, 80))
            elif kind == 2:
                nb[u] = int(rng.integers(-2, ntok + 5))
            elif kind == 3 and len(qn):
                qn[int(rng.integers(len(qn)))] = int(rng.integers(-2, len(nb) + 2))
            elif kind == 4:
                chunk = int(rng.choice([0, -32, 16, 48, 64, 4096]))  # the 4096 cap is the kernels', tested above
            else:
                ntok = int(rng.integers(-1, ntok + 3))
        try:
            want = flatten_plan(nb, nl, par, qn, ntok, chunk if chunk else 128)
        except PlanError:
            want = None
        try:
            got = binding.deft_plan(nb.astype(np.int32), nl.astype(np.int32), par.astype(np.int32),
                                    qn.astype(np.int32), ntok, chunk).view()
        except binding.DeftError:
            got = None
        assert (want is None) == (got is None), (it, nb, nl, par, qn, ntok, chunk)
        if want is None:
            refused += 1
        else:
            accepted += 1
            for key in ("seg_tok_begin", "seg_len", "seg_qlo", "seg_qhi", "chunk_qlo", "chunk_qhi", "q_part_slot", "q_order"):
                assert np.array_equal(got[key], want[key]), (it, key)
    assert refused > 100 and accepted > 50
