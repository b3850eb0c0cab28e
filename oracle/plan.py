"""TEST INFRASTRUCTURE ONLY -- the DeFT-Flatten QKV-preparation plan in plain Python.

Follows Algorithm 3 (QKV Preparation of DeFT-Flatten) and Remark 3.1 of the
paper: flatten the tree's KV depth-first, cut the flattened token sequence into
even chunks of at most S_t tokens, group every chunk with all queries that share
any of its tokens (KV-guided grouping), and give each node-piece inside a chunk a
bit causal mask over that group.  Where the paper leaves the encoding open the
following readings are used (each is also listed in the design notes):

  * children are visited in ascending node id, roots in ascending node id;
  * queries are renumbered in depth-first order (ties by caller index) so that
    the queries whose path contains node u form one interval [q_lo[u], q_hi[u]);
  * nodes that no query reaches, and nodes without tokens, are left out of the
    flattened sequence;
  * mask bit j of a segment is 1 when the j-th query of the chunk's group
    attends to the segment (1 = valid); groups wider than 64 queries use
    ceil(w/64) little-endian 64-bit words per segment;
  * a query attends to its own node's tokens (paths are inclusive).

Besides DeFT-Flatten (mode "flatten") the same encoding expresses the paper's
other partitioning strategies (Table 2): DeFT-Node ("node", Algorithm 1: one
group per tree node), DeFT-Node-Chunk ("node_chunk": nodes cut into blocks) and
Q-guided grouping with the Flash-Decoding split ("query": each query with its own
path, shared prefixes repeated), which the ablations and the IO comparison need.

Mode "balanced" is not in the paper.  Remark 3.1 cuts the flattened sequence into
chunks of equal token count because, with decoding bound by the KV read, equal
tokens mean equal cost (Section 3.3).  Where the cost of a chunk also grows with
the number of query rows that share it, "balanced" keeps the depth-first order
but weighs a chunk by tokens x rows: a node piece joins the open chunk only if
the joint chunk is not dearer than the two apart (a chunk pays every one of its
tokens for every row of its whole group), and a chunk shared by many rows may
be up to four times longer (fewer partial results per row).  The cost model is
stated in _balanced_weight; it is this build's, not the paper's.

Everything is integer work; the output arrays are the canonical encoding that
the C++ planner must reproduce bit for bit.
"""

from __future__ import annotations

import numpy as np


class PlanError(ValueError):
    pass


def _validate(nb, nl, par, qn, ntok, chunk_size):
    n = len(nb)
    if n < 1 or len(nl) != n or len(par) != n:
        raise PlanError("node table must have n_nodes >= 1 equal-length columns")
    if chunk_size <= 0 or chunk_size % 32 != 0:
        raise PlanError("chunk_size must be a positive multiple of 32")
    if ntok < 0:
        raise PlanError("ntok < 0")
    for u in range(n):
        if par[u] < -1 or par[u] >= n or par[u] == u:
            raise PlanError("parent out of range")
        if nl[u] < 0 or nb[u] < 0 or nb[u] + nl[u] > ntok:
            raise PlanError("token range outside the cache")
    # cycles: every node must reach a root within n steps
    for u in range(n):
        v, steps = u, 0
        while v != -1:
            v = par[v]
            steps += 1
            if steps > n:
                raise PlanError("parent pointers contain a cycle")
    # overlap of non-empty ranges
    spans = sorted((nb[u], nb[u] + nl[u]) for u in range(n) if nl[u] > 0)
    for a, b in zip(spans, spans[1:]):
        if b[0] < a[1]:
            raise PlanError("node token ranges overlap")
    for x in qn:
        if x < 0 or x >= n:
            raise PlanError("query node out of range")


BALANCED_ROWS_PER_TILE = 16    # rows handled together (one matrix tile)
BALANCED_TILES_PER_TASK = 8    # a chunk whose group has more tiles is worked on by several tasks
BALANCED_OPEN_COST = 192       # fixed cost of opening a chunk: 64 tokens of a one-tile group
BALANCED_MAX_STRETCH = 4       # a chunk of t tasks may hold min(t, 4) * chunk_size tokens,
BALANCED_MAX_TOKENS = 4096     # but never more than this


def _balanced_weight(width, rows_per_query):
    """(cost of one token of a chunk shared by `width` queries, number of tasks that work on the chunk).

    The group's rows (queries x query heads per KV head) are tiled BALANCED_ROWS_PER_TILE at a time; up to
    BALANCED_TILES_PER_TASK tiles make one task, wider groups are split into equal tasks; a task spends 2 units
    per token on fetching it and 1 per tile on the arithmetic."""
    rows = width * rows_per_query
    tiles = -(-rows // BALANCED_ROWS_PER_TILE)
    tasks = max(1, -(-tiles // BALANCED_TILES_PER_TASK))
    per_task = -(-tiles // tasks)
    return tasks * (2 + per_task), tasks


def flatten_plan(node_tok_begin, node_tok_len, node_parent, query_node, ntok, chunk_size=128, mode="flatten",
                 rows_per_query=1):
    """The plan for a node-contiguous cache: node u owns rows [node_tok_begin[u], +node_tok_len[u]).
    rows_per_query (query heads per KV head) only matters to mode "balanced"."""
    nb = [int(x) for x in node_tok_begin]
    nl = [int(x) for x in node_tok_len]
    par = [int(x) for x in node_parent]
    qn = [int(x) for x in query_node]
    _validate(nb, nl, par, qn, int(ntok), int(chunk_size))
    ext = [[(nb[u], nl[u])] if nl[u] > 0 else [] for u in range(len(nb))]
    return _plan(ext, nl, par, qn, int(chunk_size), mode, int(rows_per_query))


def flatten_plan_paged(node_page_ptr, page_ids, page_size, n_pool_pages, node_tok_len, node_parent, query_node,
                       chunk_size=128, mode="flatten", rows_per_query=1):
    """The plan for a paged cache (Section 4.2): token t of node u is row
    page_ids[node_page_ptr[u] + t // page_size] * page_size + t % page_size.  Pages that follow each other in
    the pool are joined into one run; segments are cut where a node's storage is not contiguous."""
    pp = [int(x) for x in node_page_ptr]
    pg = [int(x) for x in page_ids]
    nl = [int(x) for x in node_tok_len]
    par = [int(x) for x in node_parent]
    qn = [int(x) for x in query_node]
    P, npool = int(page_size), int(n_pool_pages)
    n = len(nl)
    if P < 1 or npool < 0 or len(pp) != n + 1 or pp[0] != 0:
        raise PlanError("bad page table")
    ext, seen = [], set()
    for u in range(n):
        if nl[u] < 0 or pp[u + 1] < pp[u]:
            raise PlanError("bad page table")
        need = -(-nl[u] // P)
        if pp[u + 1] - pp[u] < need:
            raise PlanError("node has too few pages")
        runs = []
        for i in range(need):
            page = pg[pp[u] + i]
            if page < 0 or page >= npool or page in seen:
                raise PlanError("page out of range or owned twice")
            seen.add(page)
            begin, cnt = page * P, min(P, nl[u] - i * P)
            if runs and runs[-1][0] + runs[-1][1] == begin:
                runs[-1] = (runs[-1][0], runs[-1][1] + cnt)
            else:
                runs.append((begin, cnt))
        ext.append(runs)
    _validate([0] * n, [0] * n, par, qn, npool * P, int(chunk_size))   # tree shape, query map, chunk size
    return _plan(ext, nl, par, qn, int(chunk_size), mode, int(rows_per_query))


def _plan(ext, nl, par, qn, B, mode, G=1):
    n, nq = len(nl), len(qn)
    if G < 1:
        raise PlanError("rows_per_query must be positive")

    # 1. children lists, ascending node id
    children = [[] for _ in range(n)]
    roots = []
    for u in range(n):
        if par[u] == -1:
            roots.append(u)
        else:
            children[par[u]].append(u)

    # 2./3. depth-first preorder with the running query counter
    cnt = [0] * n
    for x in qn:
        cnt[x] += 1
    pre, q_lo, q_hi = [], [0] * n, [0] * n
    ctr = 0
    for r in roots:
        stack = [(r, 0)]
        q_lo[r] = ctr
        ctr += cnt[r]
        pre.append(r)
        while stack:
            u, i = stack.pop()
            if i < len(children[u]):
                stack.append((u, i + 1))
                c = children[u][i]
                q_lo[c] = ctr
                ctr += cnt[c]
                pre.append(c)
                stack.append((c, 0))
            else:
                q_hi[u] = ctr
    assert ctr == nq and len(pre) == n
    rank = [0] * n
    for i, u in enumerate(pre):
        rank[u] = i
    q_order = sorted(range(nq), key=lambda j: (rank[qn[j]], j))

    # 4. flattened sequence: reached, non-empty nodes in preorder
    flat_nodes = [u for u in pre if q_hi[u] > q_lo[u] and nl[u] > 0]

    def node_range(u, off, take):
        """Physical runs (begin, length) of tokens [off, off+take) of node u."""
        out, skip = [], off
        for (b, ln) in ext[u]:
            if take == 0:
                break
            if skip >= ln:
                skip -= ln
                continue
            here = min(take, ln - skip)
            out.append((b + skip, here))
            take -= here
            skip = 0
        return out

    # 5./6. the split: chunks as lists of node pieces (physical begin, length, query interval, node)
    chunks = []
    if mode == "flatten":
        # DeFT-Flatten (Remark 3.1): cut the flattened sequence every B tokens, whatever node the cut falls in
        cur, room = [], B
        for u in flat_nodes:
            off = 0
            while off < nl[u]:
                if room == 0:
                    chunks.append(cur)
                    cur, room = [], B
                take = min(room, nl[u] - off)
                cur.extend((b, ln, q_lo[u], q_hi[u], u) for (b, ln) in node_range(u, off, take))
                off += take
                room -= take
        if cur:
            chunks.append(cur)
    elif mode == "node":
        # DeFT-Node (Algorithm 1): one QKV group per tree node, however long
        for u in flat_nodes:
            chunks.append([(b, ln, q_lo[u], q_hi[u], u) for (b, ln) in node_range(u, 0, nl[u])])
    elif mode == "node_chunk":
        # DeFT-Node-Chunk (Section 3.3): node-wise grouping, each node cut into blocks of B tokens
        for u in flat_nodes:
            for off in range(0, nl[u], B):
                chunks.append([(b, ln, q_lo[u], q_hi[u], u) for (b, ln) in node_range(u, off, min(B, nl[u] - off))])
    elif mode == "query":
        # Q-guided grouping with the Flash-Decoding split (Section 3.1; Table 2): every query is grouped with
        # its own root-to-node KV, cut into blocks of B tokens; shared prefixes are repeated per query
        for pos in range(nq):
            path = []
            u = qn[q_order[pos]]
            while u != -1:
                path.append(u)
                u = par[u]
            cur, room = [], B
            for u in reversed(path):
                off = 0
                while off < nl[u]:
                    if room == 0:
                        chunks.append(cur)
                        cur, room = [], B
                    take = min(room, nl[u] - off)
                    cur.extend((b, ln, pos, pos + 1, u) for (b, ln) in node_range(u, off, take))
                    off += take
                    room -= take
            if cur:
                chunks.append(cur)
    elif mode == "balanced":
        # depth-first order as in "flatten"; a piece joins the open chunk only if that is not dearer than a
        # chunk of its own, and the length limit grows with the number of tasks the chunk's group needs
        cur, cur_tokens, cur_lo, cur_hi = [], 0, 0, 0
        for u in flat_nodes:
            off = 0
            while off < nl[u]:
                left = nl[u] - off
                if cur:
                    lo, hi = min(cur_lo, q_lo[u]), max(cur_hi, q_hi[u])
                    w_joint, tasks = _balanced_weight(hi - lo, G)
                    take = min(left, min(B * min(tasks, BALANCED_MAX_STRETCH), BALANCED_MAX_TOKENS) - cur_tokens)
                    w_cur, _ = _balanced_weight(cur_hi - cur_lo, G)
                    w_own, _ = _balanced_weight(q_hi[u] - q_lo[u], G)
                    if take <= 0 or (cur_tokens + take) * w_joint > cur_tokens * w_cur + take * w_own + BALANCED_OPEN_COST:
                        chunks.append(cur)
                        cur, cur_tokens = [], 0
                        continue
                else:
                    lo, hi = q_lo[u], q_hi[u]
                    _, tasks = _balanced_weight(hi - lo, G)
                    take = min(left, min(B * min(tasks, BALANCED_MAX_STRETCH), BALANCED_MAX_TOKENS))
                cur.extend((b, ln, q_lo[u], q_hi[u], u) for (b, ln) in node_range(u, off, take))
                cur_tokens += take
                cur_lo, cur_hi = lo, hi
                off += take
        if cur:
            chunks.append(cur)
    else:
        raise PlanError("unknown split mode")

    m = len(chunks)
    n_flat = sum(piece[1] for ch in chunks for piece in ch)
    chunk_seg_ptr = [0]
    seg_tok_begin, seg_len, seg_qlo, seg_qhi, seg_node = [], [], [], [], []
    for ch in chunks:
        for (b, ln, lo, hi, u) in ch:
            seg_tok_begin.append(b)
            seg_len.append(ln)
            seg_qlo.append(lo)
            seg_qhi.append(hi)
            seg_node.append(u)
        chunk_seg_ptr.append(len(seg_len))
    nseg = len(seg_len)

    # 7. KV-guided grouping: the chunk's query interval and its partial-result slots
    chunk_qlo, chunk_qhi, chunk_slot_base = [], [], [0]
    for c in range(m):
        segs = range(chunk_seg_ptr[c], chunk_seg_ptr[c + 1])
        lo = min(seg_qlo[s] for s in segs)
        hi = max(seg_qhi[s] for s in segs)
        chunk_qlo.append(lo)
        chunk_qhi.append(hi)
        chunk_slot_base.append(chunk_slot_base[-1] + (hi - lo))
    n_slots = chunk_slot_base[-1]

    # 8. bit causal masks, one run of 64-bit words per segment
    seg_mask_ptr, seg_mask = [0], []
    for c in range(m):
        w = chunk_qhi[c] - chunk_qlo[c]
        words = (w + 63) // 64
        for s in range(chunk_seg_ptr[c], chunk_seg_ptr[c + 1]):
            for k in range(words):
                word = 0
                for j in range(64):
                    p = chunk_qlo[c] + 64 * k + j
                    if p < chunk_qhi[c] and seg_qlo[s] <= p < seg_qhi[s]:
                        word |= 1 << j
                seg_mask.append(word)
            seg_mask_ptr.append(len(seg_mask))

    # 9. per query: the chunks it takes part in and where its partial results live
    q_part_ptr, q_part_chunk, q_part_slot = [0], [], []
    for p in range(nq):
        for c in range(m):
            if chunk_qlo[c] <= p < chunk_qhi[c]:
                q_part_chunk.append(c)
                q_part_slot.append(chunk_slot_base[c] + (p - chunk_qlo[c]))
        q_part_ptr.append(len(q_part_chunk))

    i32 = lambda a: np.asarray(a, dtype=np.int32).reshape(-1)  # noqa: E731
    return {
        "chunk_size": B, "n_nodes": n, "nq": nq, "n_flat": n_flat,
        "n_chunks": m, "n_segs": nseg, "n_slots": n_slots,
        "q_order": i32(q_order), "node_q_lo": i32(q_lo), "node_q_hi": i32(q_hi),
        "chunk_seg_ptr": i32(chunk_seg_ptr),
        "seg_tok_begin": i32(seg_tok_begin), "seg_len": i32(seg_len),
        "seg_qlo": i32(seg_qlo), "seg_qhi": i32(seg_qhi), "seg_node": i32(seg_node),
        "chunk_qlo": i32(chunk_qlo), "chunk_qhi": i32(chunk_qhi), "chunk_slot_base": i32(chunk_slot_base),
        "seg_mask_ptr": i32(seg_mask_ptr), "seg_mask": np.asarray(seg_mask, dtype=np.uint64).reshape(-1),
        "q_part_ptr": i32(q_part_ptr), "q_part_chunk": i32(q_part_chunk), "q_part_slot": i32(q_part_slot),
    }
