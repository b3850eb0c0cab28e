"""TEST INFRASTRUCTURE ONLY -- DeFT-Flatten's attention phase, step by step, in fp64 numpy.

Takes the steps of Algorithm 4 (Attention Calculation of DeFT-Flatten) in the
paper's order: per QKV group rebuild the [b_i x b_kv] mask from the bit causal
masks and the node offsets, compute the masked partial attention o_i and its
LogSumExp lse_i, hand both to every query of the group; then per query the
global reduction of eq. 1 with the maximum LSE subtracted.  It exists to check
that a plan (oracle.plan.flatten_plan, or the product's plan viewed through the
same keys) together with the merge reproduces the plain definition; it is slow
and meant for small trees.
"""

from __future__ import annotations

import numpy as np


def seg_attn(partials, lses):
    """Eq. 1: sum_i A_i e^{LSE_i} / sum_i e^{LSE_i}, evaluated with the largest LSE subtracted.

    partials: list of [d] arrays (A_i); lses: list of scalars (LSE_i, natural log).  Segments with
    LSE = -inf (no token) carry zero weight; if every segment is empty the result is zero.
    """
    lses = np.asarray(lses, dtype=np.float64)
    d = np.asarray(partials[0]).shape[-1] if len(partials) else 0
    out = np.zeros(d, dtype=np.float64)
    if len(partials) == 0 or not np.isfinite(lses.max()):
        return out
    lse_max = lses.max()
    mid_l = 0.0
    for lse in lses:
        mid_l += np.exp(lse - lse_max)
    for a, lse in zip(partials, lses):
        out += np.exp(lse - lse_max) * np.asarray(a, dtype=np.float64) / mid_l
    return out


def reconstruct_mask(plan, c):
    """[b_i x b_kv] boolean mask of chunk c from its bit causal masks and segment offsets."""
    lo, hi = int(plan["chunk_qlo"][c]), int(plan["chunk_qhi"][c])
    w = hi - lo
    words = (w + 63) // 64
    s0, s1 = int(plan["chunk_seg_ptr"][c]), int(plan["chunk_seg_ptr"][c + 1])
    b_kv = int(plan["seg_len"][s0:s1].sum())
    mask = np.zeros((w, b_kv), dtype=bool)
    ofs = 0
    for s in range(s0, s1):
        mp = int(plan["seg_mask_ptr"][s])
        n = int(plan["seg_len"][s])
        for j in range(w):
            bit = (int(plan["seg_mask"][mp + j // 64]) >> (j % 64)) & 1
            if bit:
                mask[j, ofs:ofs + n] = True
        ofs += n
        assert int(plan["seg_mask_ptr"][s + 1]) - mp == words
    return mask


def chunk_tokens(plan, c):
    """Physical token rows of chunk c in flattened order."""
    s0, s1 = int(plan["chunk_seg_ptr"][c]), int(plan["chunk_seg_ptr"][c + 1])
    rows = []
    for s in range(s0, s1):
        b, n = int(plan["seg_tok_begin"][s]), int(plan["seg_len"][s])
        rows.extend(range(b, b + n))
    return np.asarray(rows, dtype=np.int64)


def partials_by_plan(plan, Q, K, V, scale=None):
    """Stage 1 of Algorithm 4: per QKV group the masked partial attention o_i and LogSumExp lse_i.

    Returns (part_o [n_slots,Hq,d], part_lse [n_slots,Hq]); a (slot, head) whose query sees no token of
    the chunk keeps lse = -inf and o = 0.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    nq, Hq, d = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    q_order = plan["q_order"]
    n_slots = int(plan["n_slots"])
    part_o = np.zeros((n_slots, Hq, d))
    part_lse = np.full((n_slots, Hq), -np.inf)
    for c in range(int(plan["n_chunks"])):
        lo, hi = int(plan["chunk_qlo"][c]), int(plan["chunk_qhi"][c])
        rows = chunk_tokens(plan, c)
        mask = reconstruct_mask(plan, c)
        base = int(plan["chunk_slot_base"][c])
        for h in range(Hq):
            Qi = Q[q_order[lo:hi], h, :]                    # [b_i, d]
            Kb, Vb = K[rows, h // G, :], V[rows, h // G, :]  # [b_kv, d]
            S = scale * (Qi @ Kb.T)
            S = np.where(mask, S, -np.inf)
            for j in range(hi - lo):
                if not mask[j].any():
                    continue
                smax = S[j].max()
                e = np.exp(S[j] - smax)
                part_lse[base + j, h] = smax + np.log(e.sum())
                part_o[base + j, h] = (e / e.sum()) @ Vb
    return part_o, part_lse


def attention_by_plan(plan, Q, K, V, scale=None):
    """Two-stage DeFT-Flatten attention; Q [nq,Hq,d], K/V [ntok,Hkv,d] -> O [nq,Hq,d] (fp64)."""
    Q = np.asarray(Q, dtype=np.float64)
    nq, Hq, d = Q.shape
    q_order = plan["q_order"]
    # stage 1: one partial attention per QKV group
    part_o, part_lse = partials_by_plan(plan, Q, K, V, scale)
    # stage 2: tree-topology-aware global reduction, per query
    O = np.zeros((nq, Hq, d))
    for p in range(nq):
        slots = plan["q_part_slot"][int(plan["q_part_ptr"][p]):int(plan["q_part_ptr"][p + 1])]
        if len(slots) == 0:
            continue  # a query no chunk is grouped with (its path holds no token): zeros
        for h in range(Hq):
            O[q_order[p], h] = seg_attn([part_o[s, h] for s in slots], [part_lse[s, h] for s in slots])
    return O
