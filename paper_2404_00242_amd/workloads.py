"""Seeded synthetic decoding trees and Q/K/V values.

This module only *generates inputs*: tree topologies (node table + query map)
shaped like the paper's few-shot, multi-step-reasoning and speculative-decoding
workloads (Section 4.1, Table 4; Appendix A.6, Table 13), and N(0,1) values
rounded to bf16.  It holds none of the method's arithmetic, so both the CPU
oracle's tests and the HIP path's tests may draw their inputs from it.

A tree is a node table over a node-contiguous KV cache:
  node_tok_begin[u], node_tok_len[u]  physical token rows [begin, begin+len) of node u
  node_parent[u]                      parent node id, -1 for a root
  query_node[j]                       node whose tip query j sits on; the query
                                      attends over every token of every node on
                                      the root -> query_node[j] path, inclusive.
Physical cache order is node-id order (creation order), which is breadth-first
for the multi-level configs and therefore differs from depth-first order.
"""

from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Tree:
    name: str
    node_tok_begin: np.ndarray  # int32 [n_nodes]
    node_tok_len: np.ndarray  # int32 [n_nodes]
    node_parent: np.ndarray  # int32 [n_nodes]
    query_node: np.ndarray  # int32 [nq]
    ntok: int
    Hq: int
    Hkv: int
    d: int
    value_seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def n_nodes(self) -> int:
        return int(self.node_tok_len.shape[0])

    @property
    def nq(self) -> int:
        return int(self.query_node.shape[0])


def _finish(name, lens, parents, query_node, Hq, Hkv, d, value_seed, begins=None, ntok=None, **meta):
    lens = np.asarray(lens, dtype=np.int32)
    parents = np.asarray(parents, dtype=np.int32)
    if begins is None:
        begins = np.zeros_like(lens)
        if lens.size:
            begins[1:] = np.cumsum(lens[:-1], dtype=np.int64).astype(np.int32)
    begins = np.asarray(begins, dtype=np.int32)
    if ntok is None:
        ntok = int(lens.sum())
    return Tree(name, begins, lens, parents, np.asarray(query_node, dtype=np.int32), int(ntok),
                Hq, Hkv, d, value_seed, dict(meta))


def config1_tiny(leaf_len: int = 32) -> Tree:
    """Tiny tree: root of 256 tokens, four leaves of `leaf_len` tokens, a query at each leaf."""
    lens = [256] + [leaf_len] * 4
    parents = [-1, 0, 0, 0, 0]
    return _finish("cfg1_tiny" if leaf_len == 32 else f"cfg1_tiny_leaf{leaf_len}",
                   lens, parents, [1, 2, 3, 4], 4, 4, 64, 1001)


def config2_fewshot(prefix: int = 4000, branches: int = 20, gen: int = 256) -> Tree:
    """Few-shot prompting: one shared prompt, `branches` generations, a query per branch tip."""
    lens = [prefix] + [gen] * branches
    parents = [-1] + [0] * branches
    return _finish("cfg2_fewshot", lens, parents, list(range(1, branches + 1)), 32, 32, 128, 1002)


def config3_speculative(prefix: int = 4000, fanouts=(10, 3, 1, 1), keep: int = 64,
                        Hq: int = 32, Hkv: int = 32) -> Tree:
    """Speculative decoding: committed prefix plus a token tree of one-token nodes.

    The token tree is grown level by level with the given top-k fanouts, numbered
    in breadth-first order and truncated to the first `keep` nodes; every kept
    tree token carries a query.
    """
    parents = [-1]
    level = [0]
    for f in fanouts:
        nxt = []
        for u in level:
            for _ in range(f):
                parents.append(u)
                nxt.append(len(parents) - 1)
        level = nxt
    parents = parents[: keep + 1]
    lens = [prefix] + [1] * keep
    return _finish("cfg3_speculative", lens, parents, list(range(1, keep + 1)), Hq, Hkv, 128, 1003)


def config4_reasoning(root: int = 1000, depth: int = 4, branching: int = 4, lo: int = 128, hi: int = 512,
                      struct_seed: int = 2004) -> Tree:
    """Multi-step reasoning: a `branching`-ary tree of `depth` levels under a prompt; queries at the leaves."""
    rng = np.random.default_rng(struct_seed)
    parents = [-1]
    level = [0]
    for _ in range(depth):
        nxt = []
        for u in level:
            for _ in range(branching):
                parents.append(u)
                nxt.append(len(parents) - 1)
        level = nxt
    n = len(parents)
    lens = np.empty(n, dtype=np.int64)
    lens[0] = root
    lens[1:] = rng.integers(lo, hi + 1, size=n - 1)
    return _finish("cfg4_reasoning_gqa", lens, parents, level, 32, 8, 128, 1004)


def config5_longcontext(root: int = 32768, branches: int = 64, lo: int = 64, hi: int = 2048,
                        sub_parents: int = 8, sub_children: int = 8, sub_len: int = 128,
                        struct_seed: int = 2005) -> Tree:
    """Long-context stress: a very long shared prefix, ragged branches, a second level under a few of them."""
    rng = np.random.default_rng(struct_seed)
    blens = rng.integers(lo, hi + 1, size=branches)
    lens = [root] + [int(x) for x in blens]
    parents = [-1] + [0] * branches
    for b in range(1, sub_parents + 1):
        for _ in range(sub_children):
            parents.append(b)
            lens.append(sub_len)
    n = len(parents)
    has_child = np.zeros(n, dtype=bool)
    for u in range(1, n):
        has_child[parents[u]] = True
    leaves = [u for u in range(n) if not has_child[u]]
    return _finish("cfg5_longcontext_gqa", lens, parents, leaves, 32, 8, 128, 1005)


def make_config(i: int) -> Tree:
    """The five benchmark configurations, numbered 1..5."""
    return {1: config1_tiny, 2: config2_fewshot, 3: config3_speculative,
            4: config4_reasoning, 5: config5_longcontext}[i]()


def random_tree(seed: int, n_nodes: int = 12, max_len: int = 70, nq: int = 9, Hq: int = 4, Hkv: int = 2,
                d: int = 64, n_roots: int = 1, zero_len_prob: float = 0.1, shuffle_cache: bool = True,
                gap: int = 3) -> Tree:
    """A random forest with random node lengths, queries on arbitrary nodes (internal ones and repeats
    included), node ids that are not in topological order, and a shuffled, gapped physical cache."""
    rng = np.random.default_rng(seed)
    n_roots = max(1, min(n_roots, n_nodes))
    # topology on canonical ids 0..n-1 (parent < child), then relabel with a random permutation
    par = np.full(n_nodes, -1, dtype=np.int64)
    for u in range(n_roots, n_nodes):
        par[u] = rng.integers(0, u)
    perm = rng.permutation(n_nodes)  # canonical id -> public id
    parents = np.full(n_nodes, -1, dtype=np.int64)
    for u in range(n_nodes):
        parents[perm[u]] = -1 if par[u] < 0 else perm[par[u]]
    lens = rng.integers(1, max_len + 1, size=n_nodes)
    lens[rng.random(n_nodes) < zero_len_prob] = 0
    # physical placement: random order, random gaps
    order = rng.permutation(n_nodes) if shuffle_cache else np.arange(n_nodes)
    begins = np.zeros(n_nodes, dtype=np.int64)
    cur = int(rng.integers(0, gap + 1)) if gap else 0
    for u in order:
        begins[u] = cur
        cur += int(lens[u]) + (int(rng.integers(0, gap + 1)) if gap else 0)
    ntok = max(cur, 1)
    query_node = rng.integers(0, n_nodes, size=nq)
    return _finish(f"random_{seed}", lens, parents, query_node, Hq, Hkv, d, 5000 + seed, begins=begins, ntok=ntok)


def to_paged(tree: Tree, page_size: int, seed: int = 0, shuffle: bool = True, spare_pages: int = 3):
    """Scatters a tree's tokens over a paged pool: every node gets ceil(len / page_size) pages of its own,
    drawn from the pool in random order (or in node order when shuffle is false), the last one partly filled.
    Returns (node_page_ptr, page_ids, n_pool_pages, row_of) where row_of[r] is the pool row of row r of the
    tree's node-contiguous cache (-1 for rows no node owns)."""
    rng = np.random.default_rng(seed)
    need = [-(-int(n) // page_size) for n in tree.node_tok_len]
    total = int(sum(need))
    n_pool = total + spare_pages
    order = rng.permutation(n_pool)[:total] if shuffle else np.arange(total)
    node_page_ptr = np.zeros(tree.n_nodes + 1, dtype=np.int32)
    node_page_ptr[1:] = np.cumsum(need)
    page_ids = np.asarray(order, dtype=np.int32)
    row_of = np.full(tree.ntok, -1, dtype=np.int64)
    for u in range(tree.n_nodes):
        b, n = int(tree.node_tok_begin[u]), int(tree.node_tok_len[u])
        for t in range(n):
            row_of[b + t] = int(page_ids[node_page_ptr[u] + t // page_size]) * page_size + t % page_size
    return node_page_ptr, page_ids, n_pool, row_of


def scatter_to_pool(x, row_of, n_pool_rows: int, fill_seed: int = 7):
    """Moves a [ntok, H, d] tensor of a node-contiguous cache into a [n_pool_rows, H, d] pool; rows of the pool
    that no token owns are filled with other random values (they must never be read)."""
    import torch

    g = torch.Generator().manual_seed(fill_seed)
    pool = torch.randn((n_pool_rows,) + tuple(x.shape[1:]), generator=g).to(x.dtype)
    owned = torch.from_numpy(np.nonzero(row_of >= 0)[0])
    pool[torch.from_numpy(row_of[row_of >= 0])] = x[owned]
    return pool


def _to_bf16(x: np.ndarray):
    import torch

    return torch.from_numpy(x).to(torch.bfloat16)


def make_qkv(tree: Tree, seed: int | None = None):
    """Q [nq,Hq,d], K and V [ntok,Hkv,d] as CPU bf16 tensors: i.i.d. N(0,1) drawn in float32
    (Q first, then K, then V, from one generator) and rounded to nearest-even bf16."""
    rng = np.random.default_rng(tree.value_seed if seed is None else seed)
    q = rng.standard_normal((tree.nq, tree.Hq, tree.d), dtype=np.float32)
    k = rng.standard_normal((tree.ntok, tree.Hkv, tree.d), dtype=np.float32)
    v = rng.standard_normal((tree.ntok, tree.Hkv, tree.d), dtype=np.float32)
    return _to_bf16(q), _to_bf16(k), _to_bf16(v)


def path_token_count(tree: Tree) -> int:
    """Sum over queries of the token length of their root-to-node path (the paper's sum of N_i)."""
    total = 0
    for u in tree.query_node:
        u = int(u)
        while u >= 0:
            total += int(tree.node_tok_len[u])
            u = int(tree.node_parent[u])
    return total


class DecodeLoopSim:
    """A decoding tree that changes every iteration, over a paged pool, as in tree-based decoding
    (Section 2 and Appendix A.1 of the paper: every live leaf generates a token per iteration, the branch
    controller now and then forks a leaf into several children or prunes branches).

    Only structure is simulated (no values, no arithmetic of the method): nodes own pages of a pool handed out
    from a shuffled free list; a pruned branch gives its pages back, so later nodes reuse them.  `tables()`
    returns the current (node_page_ptr, page_ids, node_tok_len, node_parent, query_node) in the form
    deft_plan_paged takes; nodes are never renumbered, pruned ones just keep no query below them.
    """

    def __init__(self, seed: int, prompt_len: int, width: int, page_size: int, n_pool_pages: int):
        self.rng = np.random.default_rng(seed)
        self.P = page_size
        self.n_pool = n_pool_pages
        self.free = list(self.rng.permutation(n_pool_pages))
        self.pages, self.lens, self.parent = [], [], []
        self.leaves = []  # live leaves, each carries one query
        root = self._new_node(-1, prompt_len)
        for _ in range(width):
            self.leaves.append(self._new_node(root, 1))

    def _grow(self, u: int, n: int):
        need = -(-(self.lens[u] + n) // self.P) - len(self.pages[u])
        if need > len(self.free):
            raise RuntimeError("pool exhausted")
        for _ in range(need):
            self.pages[u].append(int(self.free.pop()))
        self.lens[u] += n

    def _new_node(self, parent: int, n: int) -> int:
        self.pages.append([])
        self.lens.append(0)
        self.parent.append(parent)
        u = len(self.lens) - 1
        self._grow(u, n)
        return u

    def step(self):
        """Every live leaf appends the token it generated."""
        for u in self.leaves:
            self._grow(u, 1)

    def branch(self, fanout: int = 2):
        """A random live leaf forks: `fanout` children of one token each take over its query."""
        i = int(self.rng.integers(len(self.leaves)))
        u = self.leaves.pop(i)
        for _ in range(fanout):
            self.leaves.append(self._new_node(u, 1))

    def prune(self, n: int = 1):
        """Drops n random live leaves; nodes that no live leaf descends from give their pages back."""
        for _ in range(min(n, len(self.leaves) - 1)):
            self.leaves.pop(int(self.rng.integers(len(self.leaves))))
        alive = set()
        for u in self.leaves:
            while u >= 0 and u not in alive:
                alive.add(u)
                u = self.parent[u]
        for u in range(len(self.lens)):
            if u not in alive and self.pages[u]:
                self.free.extend(self.pages[u])
                self.pages[u] = []
                self.lens[u] = 0

    def tables(self):
        ptr = np.zeros(len(self.lens) + 1, dtype=np.int32)
        ptr[1:] = np.cumsum([len(p) for p in self.pages])
        ids = np.asarray([x for p in self.pages for x in p], dtype=np.int32)
        return (ptr, ids, np.asarray(self.lens, dtype=np.int32), np.asarray(self.parent, dtype=np.int32),
                np.asarray(self.leaves, dtype=np.int32))
