"""Pins for the fp64 attention oracle (CPU only).

The oracle is checked against things other than itself:
  * a single-branch tree must equal ordinary decode attention -> library SDPA in fp64;
  * a dense-mask formulation softmax(QK^T/sqrt(d) + M)V (the vanilla tree attention of
    Section 3.3 / Appendix A.4) whose mask comes from the transitive closure of the
    adjacency matrix, not from walking parent pointers;
  * closed forms (two-token path with weights 1/3, 2/3; equal keys -> mean of V;
    value tagged by KV head -> GQA head mapping);
  * invariances (sibling order / node relabelling, moving nodes in the physical cache);
  * eq. 1: splitting a path into segments and merging (A_i, LSE_i) is an identity.
"""

import numpy as np
import pytest
import torch

import oracle
from oracle import deft_flatten
from paper_2404_00242_amd import workloads as wl


def dense_mask_attention(Q, K, V, nb, nl, par, qn, scale):
    """softmax(scale*QK^T + M)V with M from the reflexive-transitive closure of the tree's adjacency."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    n = len(nb)
    A = np.eye(n, dtype=np.int64)
    for u in range(n):
        if par[u] >= 0:
            A[par[u], u] = 1  # edge parent -> child
    R = A.copy()
    for _ in range(max(1, int(np.ceil(np.log2(max(n, 2)))) + 1)):
        R = ((R @ R) > 0).astype(np.int64)
    # R[a, u] = 1 iff a is an ancestor of u or u itself
    ntok = K.shape[0]
    owner = np.full(ntok, -1)
    for u in range(n):
        owner[nb[u]:nb[u] + nl[u]] = u
    nq, Hq, d = Q.shape
    G = Hq // K.shape[1]
    M = np.full((nq, ntok), -np.inf)
    for j in range(nq):
        ok = (owner >= 0) & (R[np.clip(owner, 0, n - 1), qn[j]] > 0)
        M[j, ok] = 0.0
    O = np.zeros((nq, Hq, d))
    for h in range(Hq):
        S = scale * (Q[:, h, :] @ K[:, h // G, :].T) + M
        for j in range(nq):
            if not np.isfinite(S[j]).any():
                continue
            e = np.exp(S[j] - S[j][np.isfinite(S[j])].max())
            O[j, h] = (e / e.sum()) @ V[:, h // G, :]
    return O


def _f32(t):
    return t.float().numpy()


def test_single_branch_equals_library_sdpa():
    # a chain of nodes is ordinary causal decode: the last token's query sees every token
    rng = np.random.default_rng(7)
    lens = [5, 17, 1, 40]
    Hq, Hkv, d = 6, 2, 32
    ntok = sum(lens)
    nb = np.cumsum([0] + lens[:-1])
    par = [-1, 0, 1, 2]
    Q = rng.standard_normal((1, Hq, d)).astype(np.float32)
    K = rng.standard_normal((ntok, Hkv, d)).astype(np.float32)
    V = rng.standard_normal((ntok, Hkv, d)).astype(np.float32)
    got = oracle.tree_attention(Q, K, V, nb, lens, par, [3])
    q = torch.from_numpy(Q).double().permute(1, 0, 2).unsqueeze(0)            # [1,Hq,1,d]
    k = torch.from_numpy(K).double().permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0).unsqueeze(0)
    v = torch.from_numpy(V).double().permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0).unsqueeze(0)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v)[0, :, 0, :].numpy()
    np.testing.assert_allclose(got[0], ref, rtol=0, atol=1e-12)
    # a query on an inner node of the chain sees only the prefix up to that node
    got2 = oracle.tree_attention(Q, K, V, nb, lens, par, [1])
    n2 = lens[0] + lens[1]
    ref2 = torch.nn.functional.scaled_dot_product_attention(q, k[:, :, :n2], v[:, :, :n2])[0, :, 0, :].numpy()
    np.testing.assert_allclose(got2[0], ref2, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", range(8))
def test_matches_dense_mask_formulation(seed):
    t = wl.random_tree(seed, n_nodes=3 + seed, max_len=9, nq=5, Hq=4, Hkv=2, d=8, n_roots=1 + seed % 2)
    Q, K, V = wl.make_qkv(t)
    scale = 1.0 / np.sqrt(t.d)
    got = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    ref = dense_mask_attention(_f32(Q), _f32(K), _f32(V), t.node_tok_begin, t.node_tok_len, t.node_parent,
                               t.query_node, scale)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_closed_form_two_tokens():
    # scores 0 and ln 2  ->  weights 1/3 and 2/3, whatever d is (catches a missing 1/sqrt(d))
    d = 16
    Q = np.zeros((1, 1, d), np.float32)
    Q[0, 0, 0] = 1.0
    K = np.zeros((2, 1, d), np.float32)
    K[1, 0, 0] = np.float32(np.sqrt(d) * np.log(2.0))
    V = np.zeros((2, 1, d), np.float32)
    V[0, 0, :] = 3.0
    V[1, 0, :] = -6.0
    got = oracle.tree_attention(Q, K, V, [0, 1], [1, 1], [-1, 0], [1])
    k1 = float(K[1, 0, 0]) / np.sqrt(d)
    w1 = np.exp(k1) / (1 + np.exp(k1))
    assert abs(w1 - 2 / 3) < 1e-7
    np.testing.assert_allclose(got[0, 0], np.full(d, (1 - w1) * 3.0 + w1 * -6.0), atol=1e-13)
    # explicit scale overrides 1/sqrt(d)
    got2 = oracle.tree_attention(Q, K, V, [0, 1], [1, 1], [-1, 0], [1], scale=0.0)
    np.testing.assert_allclose(got2[0, 0], np.full(d, -1.5), atol=1e-13)


def test_equal_keys_give_path_mean_and_gqa_head_mapping():
    t = wl.config1_tiny()
    rng = np.random.default_rng(3)
    Hq, Hkv, d = 6, 3, 8
    Q = rng.standard_normal((t.nq, Hq, d)).astype(np.float32)
    K = np.ones((t.ntok, Hkv, d), np.float32)             # every score equal -> uniform softmax
    V = rng.standard_normal((t.ntok, Hkv, d)).astype(np.float32)
    got = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    for j, leaf in enumerate(t.query_node):
        rows = list(range(0, 256)) + list(range(t.node_tok_begin[leaf], t.node_tok_begin[leaf] + 32))
        for h in range(Hq):
            np.testing.assert_allclose(got[j, h], V[rows, h // 2, :].astype(np.float64).mean(0), atol=1e-13)
    # value = index of the KV head: the output names the KV head each query head read
    V2 = np.broadcast_to(np.arange(Hkv, dtype=np.float32)[None, :, None], (t.ntok, Hkv, d)).copy()
    Kr = rng.standard_normal((t.ntok, Hkv, d)).astype(np.float32)
    got2 = oracle.tree_attention(Q, Kr, V2, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    for h in range(Hq):
        np.testing.assert_allclose(got2[:, h, :], h // 2, atol=1e-13)


def test_dominant_key_selects_its_value():
    # one key aligned with the query and scaled up takes (numerically) all the weight
    t = wl.config1_tiny()
    rng = np.random.default_rng(5)
    d = 8
    Q = np.zeros((t.nq, 1, d), np.float32)
    Q[:, 0, 0] = 1.0
    K = np.zeros((t.ntok, 1, d), np.float32)
    V = rng.standard_normal((t.ntok, 1, d)).astype(np.float32)
    for r in (100, 300, 330, 383):   # 100 is in the root; 300, 330, 383 are in the leaves of queries 1, 2, 3
        K[r, 0, 0] = 400.0
    got = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    # every query sees root token 100; queries 1, 2, 3 also see the hot token of their own leaf only
    np.testing.assert_allclose(got[0, 0], V[100, 0], atol=1e-12)
    np.testing.assert_allclose(got[1, 0], 0.5 * (V[100, 0].astype(np.float64) + V[300, 0]), atol=1e-12)
    np.testing.assert_allclose(got[2, 0], 0.5 * (V[100, 0].astype(np.float64) + V[330, 0]), atol=1e-12)
    np.testing.assert_allclose(got[3, 0], 0.5 * (V[100, 0].astype(np.float64) + V[383, 0]), atol=1e-12)


@pytest.mark.parametrize("seed", range(4))
def test_relabelling_and_cache_moves_leave_outputs_unchanged(seed):
    t = wl.random_tree(100 + seed, n_nodes=9, max_len=12, nq=6, Hq=2, Hkv=2, d=8, zero_len_prob=0.0)
    Q, K, V = (_f32(x) for x in wl.make_qkv(t))
    base = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node)
    rng = np.random.default_rng(seed)
    # relabel nodes (changes sibling order under the ascending-id rule)
    perm = rng.permutation(t.n_nodes)          # old id -> new id
    nb2 = np.empty_like(t.node_tok_begin)
    nl2 = np.empty_like(t.node_tok_len)
    par2 = np.empty_like(t.node_parent)
    for u in range(t.n_nodes):
        nb2[perm[u]] = t.node_tok_begin[u]
        nl2[perm[u]] = t.node_tok_len[u]
        par2[perm[u]] = -1 if t.node_parent[u] < 0 else perm[t.node_parent[u]]
    qn2 = perm[t.query_node]
    got = oracle.tree_attention(Q, K, V, nb2, nl2, par2, qn2)
    np.testing.assert_allclose(got, base, rtol=0, atol=1e-13)
    # move every node to a new place in a bigger cache
    order = rng.permutation(t.n_nodes)
    nb3 = np.zeros_like(t.node_tok_begin)
    cur = 2
    for u in order:
        nb3[u] = cur
        cur += int(t.node_tok_len[u]) + 1
    K3 = rng.standard_normal((cur, 2, 8)).astype(np.float32)
    V3 = rng.standard_normal((cur, 2, 8)).astype(np.float32)
    for u in range(t.n_nodes):
        a, n, b = t.node_tok_begin[u], t.node_tok_len[u], nb3[u]
        K3[b:b + n] = K[a:a + n]
        V3[b:b + n] = V[a:a + n]
    got3 = oracle.tree_attention(Q, K3, V3, nb3, t.node_tok_len, t.node_parent, t.query_node)
    np.testing.assert_allclose(got3, base, rtol=0, atol=1e-13)
    # permuting the queries permutes the outputs
    qp = rng.permutation(t.nq)
    got4 = oracle.tree_attention(Q[qp], K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node[qp])
    np.testing.assert_allclose(got4, base[qp], rtol=0, atol=1e-13)


def test_eq1_segment_merge_is_an_identity():
    rng = np.random.default_rng(11)
    d, n = 16, 97
    q = rng.standard_normal(d)
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    s = K @ q / np.sqrt(d)
    full = (np.exp(s - s.max()) / np.exp(s - s.max()).sum()) @ V
    for cuts in ([40], [1, 2, 50], [10, 20, 30, 40, 96]):
        parts, lses = [], []
        for a, b in zip([0] + cuts, cuts + [n]):
            e = np.exp(s[a:b] - s[a:b].max())
            parts.append((e / e.sum()) @ V[a:b])
            lses.append(s[a:b].max() + np.log(e.sum()))
        np.testing.assert_allclose(deft_flatten.seg_attn(parts, lses), full, rtol=0, atol=1e-13)
    # an empty segment (LSE = -inf) carries no weight
    e = np.exp(s - s.max())
    np.testing.assert_allclose(
        deft_flatten.seg_attn([np.zeros(d), full], [-np.inf, s.max() + np.log(e.sum())]), full, atol=1e-13)


def test_empty_path_and_errors():
    # a query whose whole path has no tokens gets zeros
    Q = np.ones((1, 1, 4), np.float32)
    K = np.ones((3, 1, 4), np.float32)
    got = oracle.tree_attention(Q, K, K, [0, 0], [0, 0], [-1, 0], [1])
    assert np.all(got == 0)
    with pytest.raises(ValueError):
        oracle.tree_attention(Q, K, K, [0, 0], [1, 1], [1, 0], [1])   # cycle
    with pytest.raises(ValueError):
        oracle.tree_attention(Q, K, K, [0, 2], [1, 5], [-1, 0], [1])  # range outside cache


def test_thread_count_does_not_change_results():
    t = wl.random_tree(42, n_nodes=10, max_len=30, nq=7, Hq=4, Hkv=2, d=16)
    Q, K, V = wl.make_qkv(t)
    a = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, nthreads=1)
    b, used = oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node,
                                    nthreads=4, return_threads=True)
    assert used >= 1
    assert np.array_equal(a, b)
