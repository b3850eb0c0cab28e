// Host side of libdeft: the QKV Preparation Phase of DeFT-Flatten (Algorithm 3, Remark 3.1)
// and the launch schedule derived from it.  Pure integer work, no device calls.
#include <algorithm>
#include <cstring>
#include <memory>
#include <new>
#include <numeric>

#include "deft_internal.h"

namespace {

struct Range {
    int64_t begin, end;
};

// Depth-first preorder over a forest given as parent pointers.  Children are visited in
// ascending id, roots in ascending id.  Returns false when some node is not reachable from a
// root, i.e. the parent pointers contain a cycle.
bool preorder(const int32_t *parent, int32_t n, std::vector<int32_t> &order, std::vector<int32_t> &first_child,
              std::vector<int32_t> &next_sibling) {
    // sibling lists in ascending id: walk ids downwards and push to the front
    first_child.assign(n, -1);
    next_sibling.assign(n, -1);
    int32_t first_root = -1;
    for (int32_t u = n - 1; u >= 0; --u) {
        int32_t p = parent[u];
        if (p < 0) {
            next_sibling[u] = first_root;
            first_root = u;
        } else {
            next_sibling[u] = first_child[p];
            first_child[p] = u;
        }
    }
    order.clear();
    order.reserve(n);
    std::vector<int32_t> stack;
    for (int32_t r = first_root; r >= 0; r = next_sibling[r]) {
        stack.push_back(r);
        while (!stack.empty()) {
            int32_t u = stack.back();
            stack.pop_back();
            order.push_back(u);
            // push children so that the smallest id is popped first
            size_t mark = stack.size();
            for (int32_t c = first_child[u]; c >= 0; c = next_sibling[c]) stack.push_back(c);
            std::reverse(stack.begin() + (ptrdiff_t)mark, stack.end());
        }
    }
    return (int32_t)order.size() == n;
}

}  // namespace

namespace {

// Where a node's tokens live: node u owns extents ext_ptr[u] .. ext_ptr[u+1]-1, each a run of physical rows
// [begin, begin+len); its tokens are the concatenation of its extents.  A contiguous cache gives one extent
// per node, a paged cache one per run of consecutive pages.
struct NodeExtents {
    std::vector<int32_t> ptr, begin, len;
};

// prev: a plan of an earlier version of the tree, or null.  Whatever the new tree shares with it is taken over
// instead of being recomputed: the depth-first order and the renumbering of the queries when parents and the
// query map are the same, and every chunk in front of the first node whose tokens differ when the split and
// the chunk size are the same too.  The result is the plan a call without prev gives.
int plan_impl(const NodeExtents &ext, const int32_t *node_tok_len, const int32_t *node_parent, int32_t n_nodes,
              const int32_t *query_node, int32_t nq, int32_t ntok, int32_t chunk_size, uint32_t flags,
              deft_plan_t **out_plan, const deft_plan_t *prev = nullptr) {
    if (n_nodes < 1 || nq < 0 || ntok < 0) return DEFT_EINVAL;
    const uint32_t mode = flags & 0xffu;
    const int32_t rows_per_query = (int32_t)((flags >> 16) & 0xfffu);  // DEFT_ROWS_PER_QUERY(g), 0 = not given
    if ((flags & ~(0xffu | (uint32_t)DEFT_PRECISE_WEIGHTS | (0xfffu << 16))) != 0) return DEFT_EINVAL;
    if (mode > DEFT_SPLIT_BALANCED) return DEFT_EINVAL;
    if (nq > 0 && !query_node) return DEFT_EINVAL;
    if (chunk_size == 0) chunk_size = DEFT_DEFAULT_CHUNK;
    if (chunk_size < 0 || chunk_size % 32 != 0 || chunk_size > DEFT_MAX_CHUNK) return DEFT_EINVAL;

    try {
        const int32_t n = n_nodes;
        // ---- validation -------------------------------------------------------------------
        std::vector<Range> spans;
        spans.reserve(ext.len.size());
        for (int32_t u = 0; u < n; ++u) {
            int32_t p = node_parent[u];
            if (p < -1 || p >= n || p == u) return DEFT_EINVAL;
            if (node_tok_len[u] < 0) return DEFT_EINVAL;
            int64_t total = 0;
            for (int32_t e = ext.ptr[u]; e < ext.ptr[u + 1]; ++e) {
                const int64_t b = ext.begin[e], len = ext.len[e];
                if (b < 0 || len <= 0 || b + len > (int64_t)ntok) return DEFT_EINVAL;
                spans.push_back({b, b + len});
                total += len;
            }
            if (total != node_tok_len[u]) return DEFT_EINVAL;
        }
        // (a cache that hands out rows in node order, the usual case, is sorted already)
        auto by_begin = [](const Range &a, const Range &b) { return a.begin < b.begin; };
        if (!std::is_sorted(spans.begin(), spans.end(), by_begin)) std::sort(spans.begin(), spans.end(), by_begin);
        for (size_t i = 1; i < spans.size(); ++i)
            if (spans[i].begin < spans[i - 1].end) return DEFT_EINVAL;
        for (int32_t j = 0; j < nq; ++j)
            if (query_node[j] < 0 || query_node[j] >= n) return DEFT_EINVAL;

        // same parents and same query map as prev: same depth-first order, same query intervals
        const bool same_topology =
            prev && prev->n_nodes == n && prev->nq == nq &&
            std::memcmp(prev->in_parent.data(), node_parent, (size_t)n * sizeof(int32_t)) == 0 &&
            (nq == 0 || std::memcmp(prev->in_query_node.data(), query_node, (size_t)nq * sizeof(int32_t)) == 0);

        deft_plan_t *P = new deft_plan_s();
        std::unique_ptr<deft_plan_t> guard(P);
        P->chunk_size = chunk_size;
        P->n_nodes = n;
        P->nq = nq;
        P->ntok = ntok;
        P->mode = mode;
        P->precise_all = (flags & DEFT_PRECISE_WEIGHTS) != 0;
        P->flags = flags;
        P->in_parent.assign(node_parent, node_parent + n);
        P->in_query_node.assign(query_node, query_node + nq);
        P->in_tok_len.assign(node_tok_len, node_tok_len + n);
        P->in_ext_ptr = ext.ptr;
        P->in_ext_begin = ext.begin;
        P->in_ext_len = ext.len;

        std::vector<int32_t> &pre = P->pre;
        if (same_topology) {
            pre = prev->pre;
        } else {
            std::vector<int32_t> first_child, next_sibling;
            if (!preorder(node_parent, n, pre, first_child, next_sibling)) return DEFT_EINVAL;  // cycle
        }

        // ---- depth-first renumbering of the queries ------------------------------------------
        // A node's own queries come first, then its subtrees, so the queries whose path contains u
        // are one interval.  q_hi[u] = q_lo[u] + (number of queries in u's subtree).
        if (same_topology) {
            P->node_q_lo = prev->node_q_lo;
            P->node_q_hi = prev->node_q_hi;
            P->q_order = prev->q_order;
        } else {
        std::vector<int32_t> own(n, 0), sub(n, 0);
        for (int32_t j = 0; j < nq; ++j) ++own[query_node[j]];
        sub = own;
        for (int32_t i = n - 1; i >= 0; --i) {  // reverse preorder: children before parents
            int32_t u = pre[i], p = node_parent[u];
            if (p >= 0) sub[p] += sub[u];
        }
        P->node_q_lo.assign(n, 0);
        P->node_q_hi.assign(n, 0);
        std::vector<int32_t> own_begin(n, 0);
        {
            // In preorder a node's interval starts where the previous node's own queries end or,
            // when leaving subtrees, where those subtrees end: a running counter does both.
            int32_t ctr = 0;
            for (int32_t i = 0; i < n; ++i) {
                int32_t u = pre[i];
                P->node_q_lo[u] = ctr;
                P->node_q_hi[u] = ctr + sub[u];
                own_begin[u] = ctr;
                ctr += own[u];
            }
        }
        P->q_order.assign(nq, 0);
        {
            std::vector<int32_t> cursor = own_begin;  // next free plan position among u's own queries
            for (int32_t j = 0; j < nq; ++j) P->q_order[cursor[query_node[j]]++] = j;
        }
        }

        // tokens on each query's whole path (parents come before children in preorder)
        {
            std::vector<int64_t> plen(n, 0);
            for (int32_t i = 0; i < n; ++i) {
                const int32_t u = pre[i], p = node_parent[u];
                plen[u] = (p >= 0 ? plen[p] : 0) + node_tok_len[u];
            }
            P->q_path_len.resize(nq);
            for (int32_t pos = 0; pos < nq; ++pos)
                P->q_path_len[pos] = (int32_t)std::min<int64_t>(plen[query_node[P->q_order[pos]]], INT32_MAX);
        }

        // ---- the split: chunks as runs of node pieces ---------------------------------------------
        const int32_t S = chunk_size;
        int64_t flat = 0;
        bool open = false;
        int32_t at_i = 0, at_done = 0;  // where the split loops are: position in `pre`, tokens of that node already placed

        // ---- chunks taken over from prev: all that end in front of the first node whose tokens differ ----
        int32_t i_resume = 0, done_resume = 0, c_keep = 0;
        if (same_topology && prev->chunk_size == chunk_size && prev->flags == flags && mode != DEFT_GROUP_QUERY) {
            auto differs = [&](int32_t u) {
                if (prev->in_tok_len[u] != node_tok_len[u]) return true;
                const int32_t a0 = prev->in_ext_ptr[u], a1 = prev->in_ext_ptr[u + 1], b0 = ext.ptr[u], b1 = ext.ptr[u + 1];
                if (a1 - a0 != b1 - b0) return true;
                for (int32_t k = 0; k < a1 - a0; ++k)
                    if (prev->in_ext_begin[a0 + k] != ext.begin[b0 + k] || prev->in_ext_len[a0 + k] != ext.len[b0 + k])
                        return true;
                return false;
            };
            int32_t i0 = 0;
            while (i0 < n && !differs(pre[i0])) ++i0;
            // A chunk is taken over if the chunk behind it also starts in front of the first change: what closed it
            // (it was full, or the next piece would have made it too dear) is then the same as before.  The split
            // goes on where the first chunk not taken over started.
            const int32_t m_prev = prev->n_chunks();
            while (c_keep + 1 < m_prev && prev->chunk_first_i[c_keep + 1] < i0) ++c_keep;
            if (m_prev > 0) {
                i_resume = prev->chunk_first_i[c_keep];
                done_resume = prev->chunk_first_done[c_keep];
                flat = prev->chunk_flat_begin[c_keep];
            }
            const int32_t s_keep = m_prev > 0 ? prev->chunk_seg_ptr[c_keep] : 0;
            auto head = [](std::vector<int32_t> &dst, const std::vector<int32_t> &src, int32_t cnt) {
                dst.assign(src.begin(), src.begin() + cnt);
            };
            head(P->chunk_seg_ptr, prev->chunk_seg_ptr, c_keep);
            head(P->chunk_first_i, prev->chunk_first_i, c_keep);
            head(P->chunk_first_done, prev->chunk_first_done, c_keep);
            head(P->chunk_last_i, prev->chunk_last_i, c_keep);
            P->chunk_flat_begin.assign(prev->chunk_flat_begin.begin(), prev->chunk_flat_begin.begin() + c_keep);
            head(P->seg_tok_begin, prev->seg_tok_begin, s_keep);
            head(P->seg_len, prev->seg_len, s_keep);
            head(P->seg_qlo, prev->seg_qlo, s_keep);
            head(P->seg_qhi, prev->seg_qhi, s_keep);
            head(P->seg_node, prev->seg_node, s_keep);
            head(P->chunk_qlo, prev->chunk_qlo, c_keep);
            head(P->chunk_qhi, prev->chunk_qhi, c_keep);
            if (m_prev > 0) {
                head(P->chunk_slot_base, prev->chunk_slot_base, c_keep + 1);
                head(P->seg_mask_ptr, prev->seg_mask_ptr, s_keep + 1);
                P->seg_mask.assign(prev->seg_mask.begin(), prev->seg_mask.begin() + prev->seg_mask_ptr[s_keep]);
            }
        }

        {
            // room for the usual number of pieces: one per extent plus one per cut
            const size_t guess = ext.len.size() + (size_t)(ntok / S) + 8;
            for (std::vector<int32_t> *v : {&P->seg_tok_begin, &P->seg_len, &P->seg_qlo, &P->seg_qhi, &P->seg_node,
                                            &P->seg_mask_ptr})
                v->reserve(guess);
            P->seg_mask.reserve(guess);
        }
        auto piece = [&](int32_t begin, int32_t len, int32_t lo, int32_t hi, int32_t node) {
            if (!open) {
                P->chunk_seg_ptr.push_back(P->n_segs());
                P->chunk_first_i.push_back(at_i);
                P->chunk_first_done.push_back(at_done);
                P->chunk_last_i.push_back(at_i);
                P->chunk_flat_begin.push_back(flat);
                open = true;
            }
            P->chunk_last_i.back() = at_i;
            P->seg_tok_begin.push_back(begin);
            P->seg_len.push_back(len);
            P->seg_qlo.push_back(lo);
            P->seg_qhi.push_back(hi);
            P->seg_node.push_back(node);
            flat += len;
        };
        auto close = [&]() { open = false; };
        auto reached = [&](int32_t u) { return P->node_q_hi[u] > P->node_q_lo[u] && node_tok_len[u] > 0; };
        // tokens [off, off+take) of node u, cut where the node's storage is not contiguous
        auto node_range = [&](int32_t u, int32_t off, int32_t take, int32_t lo, int32_t hi) {
            int32_t skip = off;
            for (int32_t e = ext.ptr[u]; e < ext.ptr[u + 1] && take > 0; ++e) {
                if (skip >= ext.len[e]) {
                    skip -= ext.len[e];
                    continue;
                }
                const int32_t here = std::min(take, ext.len[e] - skip);
                piece(ext.begin[e] + skip, here, lo, hi, u);
                take -= here;
                skip = 0;
            }
        };
        switch (mode) {
            case DEFT_SPLIT_FLATTEN: {
                // Flattened Tree KV Splitting (Remark 3.1): depth-first order, a cut every S tokens
                int32_t room = S;
                for (int32_t i = i_resume; i < n; ++i) {
                    const int32_t u = pre[i];
                    if (!reached(u)) continue;
                    int32_t done = i == i_resume ? done_resume : 0;
                    const int32_t len = node_tok_len[u];
                    while (done < len) {
                        if (room == 0) {
                            close();
                            room = S;
                        }
                        const int32_t take = std::min(room, len - done);
                        at_i = i;
                        at_done = done;
                        node_range(u, done, take, P->node_q_lo[u], P->node_q_hi[u]);
                        done += take;
                        room -= take;
                    }
                }
                break;
            }
            case DEFT_SPLIT_NODE:
                // DeFT-Node (Algorithm 1): one group per tree node, whatever its length
                for (int32_t i = i_resume; i < n; ++i) {
                    const int32_t u = pre[i];
                    if (!reached(u)) continue;
                    at_i = i;
                    at_done = 0;
                    node_range(u, 0, node_tok_len[u], P->node_q_lo[u], P->node_q_hi[u]);
                    close();
                }
                break;
            case DEFT_SPLIT_NODE_CHUNK:
                // DeFT-Node-Chunk: node-wise groups, every node cut into blocks of S tokens on its own
                for (int32_t i = i_resume; i < n; ++i) {
                    const int32_t u = pre[i];
                    if (!reached(u)) continue;
                    for (int32_t done = i == i_resume ? done_resume : 0; done < node_tok_len[u]; done += S) {
                        at_i = i;
                        at_done = done;
                        node_range(u, done, std::min(S, node_tok_len[u] - done), P->node_q_lo[u], P->node_q_hi[u]);
                        close();
                    }
                }
                break;
            case DEFT_GROUP_QUERY: {
                // Q-guided grouping with the Flash-Decoding split: each query with its own root-to-node KV
                std::vector<int32_t> path;
                for (int32_t pos = 0; pos < nq; ++pos) {
                    path.clear();
                    for (int32_t u = query_node[P->q_order[pos]]; u != -1; u = node_parent[u]) path.push_back(u);
                    int32_t room = S;
                    for (auto it = path.rbegin(); it != path.rend(); ++it) {
                        const int32_t u = *it, len = node_tok_len[u];
                        int32_t done = 0;
                        while (done < len) {
                            if (room == 0) {
                                close();
                                room = S;
                            }
                            const int32_t take = std::min(room, len - done);
                            at_i = 0;  // chunks of this split are never taken over by a later plan
                            at_done = 0;
                            node_range(u, done, take, pos, pos + 1);
                            done += take;
                            room -= take;
                        }
                    }
                    close();
                }
                break;
            }
            case DEFT_SPLIT_BALANCED: {
                // Depth-first order as for DEFT_SPLIT_FLATTEN, but a chunk is weighed by tokens x rows: a piece joins
                // the open chunk only if the joint chunk costs no more than the two apart plus the cost of opening
                // one, and a chunk whose group needs t tasks may hold min(t, 4) * S tokens.
                const int64_t G = rows_per_query > 0 ? rows_per_query : 1;
                struct Weight {
                    int64_t per_token, tasks;
                };
                auto weight = [&](int64_t width) {
                    const int64_t tiles = (width * G + 15) / 16;
                    const int64_t tasks = std::max<int64_t>(1, (tiles + 7) / 8);
                    const int64_t per_task = (tiles + tasks - 1) / tasks;
                    return Weight{tasks * (2 + per_task), tasks};
                };
                constexpr int64_t kOpenCost = 192, kMaxStretch = 4;
                auto limit = [&](int64_t tasks) {
                    return std::min<int64_t>(S * std::min(tasks, kMaxStretch), DEFT_MAX_CHUNK);
                };
                int64_t held = 0;
                int32_t c_lo = 0, c_hi = 0;
                for (int32_t i = i_resume; i < n; ++i) {
                    const int32_t u = pre[i];
                    if (!reached(u)) continue;
                    const int32_t u_lo = P->node_q_lo[u], u_hi = P->node_q_hi[u];
                    const Weight own = weight(u_hi - u_lo);
                    int32_t done = i == i_resume ? done_resume : 0;
                    const int32_t len = node_tok_len[u];
                    while (done < len) {
                        const int64_t left = len - done;
                        int32_t lo = u_lo, hi = u_hi;
                        int64_t take;
                        if (open) {
                            lo = std::min(c_lo, u_lo);
                            hi = std::max(c_hi, u_hi);
                            const Weight joint = weight(hi - lo), cur = weight(c_hi - c_lo);
                            take = std::min<int64_t>(left, limit(joint.tasks) - held);
                            if (take <= 0 || (held + take) * joint.per_token >
                                                 held * cur.per_token + take * own.per_token + kOpenCost) {
                                close();
                                held = 0;
                                continue;
                            }
                        } else {
                            take = std::min<int64_t>(left, limit(own.tasks));
                        }
                        at_i = i;
                        at_done = done;
                        node_range(u, done, (int32_t)take, u_lo, u_hi);
                        held += take;
                        c_lo = lo;
                        c_hi = hi;
                        done += (int32_t)take;
                    }
                }
                break;
            }
            default: return DEFT_EINVAL;
        }
        if (flat > INT32_MAX || P->seg_len.size() > (size_t)INT32_MAX / 2) return DEFT_EINVAL;
        P->n_flat = (int32_t)flat;
        P->chunk_seg_ptr.push_back(P->n_segs());  // closes the last chunk; {0} when there is none
        const int32_t m = (int32_t)P->chunk_seg_ptr.size() - 1;
        // The kernels expand a chunk of several pieces into a per-token table of at most DEFT_MAX_CHUNK entries; a
        // single piece needs none and may have any length.  Only DEFT_SPLIT_NODE can produce a longer chunk of
        // several pieces (a long node scattered over pages): such a plan could not be decoded and is refused here.
        for (int32_t c = 0; c < m; ++c) {
            const int32_t s0 = P->chunk_seg_ptr[c], s1 = P->chunk_seg_ptr[c + 1];
            if (s1 - s0 < 2) continue;
            int64_t len = 0;
            for (int32_t s = s0; s < s1; ++s) len += P->seg_len[s];
            if (len > DEFT_MAX_CHUNK) return DEFT_EINVAL;
        }

        // ---- KV-guided grouping: the queries of each chunk, and the slots of their partials ----
        // (chunks taken over from an earlier plan bring their groups, slots and masks with them)
        if (c_keep > m) return DEFT_EINVAL;  // cannot happen: the split only appends
        P->chunk_qlo.resize(m);
        P->chunk_qhi.resize(m);
        if (P->chunk_slot_base.empty()) P->chunk_slot_base.assign(1, 0);
        int64_t slots = P->chunk_slot_base[c_keep];
        P->chunk_slot_base.resize(m + 1);
        for (int32_t c = c_keep; c < m; ++c) {
            int32_t lo = INT32_MAX, hi = INT32_MIN;
            for (int32_t s = P->chunk_seg_ptr[c]; s < P->chunk_seg_ptr[c + 1]; ++s) {
                lo = std::min(lo, P->seg_qlo[s]);
                hi = std::max(hi, P->seg_qhi[s]);
            }
            P->chunk_qlo[c] = lo;
            P->chunk_qhi[c] = hi;
            slots += hi - lo;
            if (slots > INT32_MAX) return DEFT_EINVAL;
            P->chunk_slot_base[c + 1] = (int32_t)slots;
        }

        // ---- bit causal masks --------------------------------------------------------------------
        if (P->seg_mask_ptr.empty()) P->seg_mask_ptr.assign(1, 0);
        for (int32_t c = c_keep; c < m; ++c) {
            const int32_t lo = P->chunk_qlo[c], w = P->chunk_qhi[c] - lo;
            const int32_t words = (w + 63) / 64;
            for (int32_t s = P->chunk_seg_ptr[c]; s < P->chunk_seg_ptr[c + 1]; ++s) {
                const int32_t a = P->seg_qlo[s] - lo, b = P->seg_qhi[s] - lo;  // bits [a, b) are set
                for (int32_t k = 0; k < words; ++k) {
                    int32_t x = std::max(a, 64 * k) - 64 * k, y = std::min(b, 64 * (k + 1)) - 64 * k;
                    uint64_t word = 0;
                    if (y > x) word = (y - x == 64 ? ~0ull : ((1ull << (y - x)) - 1)) << x;
                    P->seg_mask.push_back(word);
                }
                if (P->seg_mask.size() > (size_t)INT32_MAX) return DEFT_EINVAL;
                P->seg_mask_ptr.push_back((int32_t)P->seg_mask.size());
            }
        }

        // ---- per query: chunks it takes part in (ascending) and the slots to reduce -------------
        P->q_part_ptr.assign(nq + 1, 0);
        for (int32_t c = 0; c < m; ++c)
            for (int32_t p = P->chunk_qlo[c]; p < P->chunk_qhi[c]; ++p) ++P->q_part_ptr[p + 1];
        for (int32_t p = 0; p < nq; ++p) P->q_part_ptr[p + 1] += P->q_part_ptr[p];
        P->q_part_chunk.assign((size_t)slots, 0);
        P->q_part_slot.assign((size_t)slots, 0);
        {
            std::vector<int32_t> cursor(P->q_part_ptr.begin(), P->q_part_ptr.end() - 1);
            for (int32_t c = 0; c < m; ++c)
                for (int32_t p = P->chunk_qlo[c]; p < P->chunk_qhi[c]; ++p) {
                    int32_t at = cursor[p]++;
                    P->q_part_chunk[at] = c;
                    P->q_part_slot[at] = P->chunk_slot_base[c] + (p - P->chunk_qlo[c]);
                }
        }

        *out_plan = guard.release();
        return DEFT_OK;
    } catch (const std::bad_alloc &) {
        return DEFT_ENOMEM;
    } catch (...) {
        return DEFT_EINVAL;
    }
}

}  // namespace

namespace {

int plan_contiguous(const int32_t *node_tok_begin, const int32_t *node_tok_len, const int32_t *node_parent,
                    int32_t n_nodes, const int32_t *query_node, int32_t nq, int32_t ntok, int32_t chunk_size,
                    uint32_t flags, deft_plan_t **out_plan, const deft_plan_t *prev) {
    if (out_plan) *out_plan = nullptr;
    if (!out_plan || !node_tok_begin || !node_tok_len || !node_parent || n_nodes < 1) return DEFT_EINVAL;
    try {
        NodeExtents ext;
        ext.ptr.reserve((size_t)n_nodes + 1);
        ext.begin.reserve((size_t)n_nodes);
        ext.len.reserve((size_t)n_nodes);
        ext.ptr.assign(1, 0);
        for (int32_t u = 0; u < n_nodes; ++u) {
            if (node_tok_begin[u] < 0 || node_tok_len[u] < 0 || (int64_t)node_tok_begin[u] + node_tok_len[u] > ntok)
                return DEFT_EINVAL;
            if (node_tok_len[u] > 0) {
                ext.begin.push_back(node_tok_begin[u]);
                ext.len.push_back(node_tok_len[u]);
            }
            ext.ptr.push_back((int32_t)ext.len.size());
        }
        return plan_impl(ext, node_tok_len, node_parent, n_nodes, query_node, nq, ntok, chunk_size, flags, out_plan, prev);
    } catch (const std::bad_alloc &) {
        return DEFT_ENOMEM;
    }
}

int plan_paged(const int32_t *node_page_ptr, const int32_t *page_ids, int32_t page_size, int32_t n_pool_pages,
               const int32_t *node_tok_len, const int32_t *node_parent, int32_t n_nodes, const int32_t *query_node,
               int32_t nq, int32_t chunk_size, uint32_t flags, deft_plan_t **out_plan, const deft_plan_t *prev) {
    if (out_plan) *out_plan = nullptr;
    if (!out_plan || !node_page_ptr || !node_tok_len || !node_parent || n_nodes < 1) return DEFT_EINVAL;
    if (page_size < 1 || n_pool_pages < 0 || (int64_t)page_size * n_pool_pages > INT32_MAX) return DEFT_EINVAL;
    try {
        NodeExtents ext;
        ext.ptr.assign(1, 0);
        if (node_page_ptr[0] != 0) return DEFT_EINVAL;
        for (int32_t u = 0; u < n_nodes; ++u) {
            const int32_t p0 = node_page_ptr[u], p1 = node_page_ptr[u + 1], len = node_tok_len[u];
            if (p1 < p0 || len < 0) return DEFT_EINVAL;
            const int64_t need = ((int64_t)len + page_size - 1) / page_size;
            if (p1 - p0 < need || (need > 0 && !page_ids)) return DEFT_EINVAL;
            for (int32_t i = 0; i < need; ++i) {
                const int32_t pg = page_ids[p0 + i];
                if (pg < 0 || pg >= n_pool_pages) return DEFT_EINVAL;
                const int32_t begin = pg * page_size, cnt = std::min(page_size, len - i * page_size);
                // a page that follows the previous one in the pool extends the previous extent
                if ((int32_t)ext.len.size() > ext.ptr.back() && ext.begin.back() + ext.len.back() == begin)
                    ext.len.back() += cnt;
                else {
                    ext.begin.push_back(begin);
                    ext.len.push_back(cnt);
                }
            }
            ext.ptr.push_back((int32_t)ext.len.size());
        }
        return plan_impl(ext, node_tok_len, node_parent, n_nodes, query_node, nq, n_pool_pages * page_size,
                         chunk_size, flags, out_plan, prev);
    } catch (const std::bad_alloc &) {
        return DEFT_ENOMEM;
    }
}

}  // namespace

extern "C" int deft_plan(const int32_t *node_tok_begin, const int32_t *node_tok_len, const int32_t *node_parent,
                         int32_t n_nodes, const int32_t *query_node, int32_t nq, int32_t ntok, int32_t chunk_size,
                         uint32_t flags, deft_plan_t **out_plan) {
    return plan_contiguous(node_tok_begin, node_tok_len, node_parent, n_nodes, query_node, nq, ntok, chunk_size, flags,
                           out_plan, nullptr);
}

extern "C" int deft_plan_paged(const int32_t *node_page_ptr, const int32_t *page_ids, int32_t page_size,
                               int32_t n_pool_pages, const int32_t *node_tok_len, const int32_t *node_parent,
                               int32_t n_nodes, const int32_t *query_node, int32_t nq, int32_t chunk_size,
                               uint32_t flags, deft_plan_t **out_plan) {
    return plan_paged(node_page_ptr, page_ids, page_size, n_pool_pages, node_tok_len, node_parent, n_nodes, query_node,
                      nq, chunk_size, flags, out_plan, nullptr);
}

extern "C" int deft_plan_update(const deft_plan_t *prev, const int32_t *node_tok_begin, const int32_t *node_tok_len,
                                const int32_t *node_parent, int32_t n_nodes, const int32_t *query_node, int32_t nq,
                                int32_t ntok, int32_t chunk_size, uint32_t flags, deft_plan_t **out_plan) {
    return plan_contiguous(node_tok_begin, node_tok_len, node_parent, n_nodes, query_node, nq, ntok, chunk_size, flags,
                           out_plan, prev);
}

extern "C" int deft_plan_paged_update(const deft_plan_t *prev, const int32_t *node_page_ptr, const int32_t *page_ids,
                                      int32_t page_size, int32_t n_pool_pages, const int32_t *node_tok_len,
                                      const int32_t *node_parent, int32_t n_nodes, const int32_t *query_node, int32_t nq,
                                      int32_t chunk_size, uint32_t flags, deft_plan_t **out_plan) {
    return plan_paged(node_page_ptr, page_ids, page_size, n_pool_pages, node_tok_len, node_parent, n_nodes, query_node,
                      nq, chunk_size, flags, out_plan, prev);
}

// Chunk size that fills an MI355X once.  Stage 1 runs one workgroup per (chunk, KV head, 128 rows of the
// chunk's group) and the chip holds two such workgroups on each of its 256 compute units; since a compute
// unit streams at a fixed rate however many workgroups it holds, the kernel is fastest when every unit
// gets the same number of bytes, i.e. when there are about 512 equal tasks.  The estimate weighs each
// reached node's tokens by the number of 128-row tasks its own query group needs.
extern "C" int32_t deft_suggest_chunk_size(const int32_t *node_tok_len, const int32_t *node_parent, int32_t n_nodes,
                                           const int32_t *query_node, int32_t nq, int32_t Hq, int32_t Hkv,
                                           uint32_t flags) {
    if (!node_tok_len || !node_parent || n_nodes < 1 || nq < 0 || (nq > 0 && !query_node)) return DEFT_EINVAL;
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return DEFT_EINVAL;
    const uint32_t mode = flags & 0xffu;
    if (mode > DEFT_SPLIT_BALANCED) return DEFT_EINVAL;
    try {
        for (int32_t u = 0; u < n_nodes; ++u)
            if (node_parent[u] < -1 || node_parent[u] >= n_nodes || node_parent[u] == u || node_tok_len[u] < 0)
                return DEFT_EINVAL;
        for (int32_t j = 0; j < nq; ++j)
            if (query_node[j] < 0 || query_node[j] >= n_nodes) return DEFT_EINVAL;
        std::vector<int32_t> pre, fc, ns;
        if (!preorder(node_parent, n_nodes, pre, fc, ns)) return DEFT_EINVAL;
        std::vector<int64_t> sub(n_nodes, 0);
        for (int32_t j = 0; j < nq; ++j) ++sub[query_node[j]];
        for (int32_t i = n_nodes - 1; i >= 0; --i) {
            const int32_t u = pre[i], p = node_parent[u];
            if (p >= 0) sub[p] += sub[u];
        }
        const int64_t G = Hq / Hkv;
        long double task_tokens = 0, reached_tokens = 0;
        bool wide = false;  // some tokens are shared by more rows than one task takes
        for (int32_t u = 0; u < n_nodes; ++u) {
            if (sub[u] == 0) continue;
            const int64_t row_groups = (sub[u] * G + 127) / 128;
            task_tokens += (long double)node_tok_len[u] * (long double)row_groups;
            reached_tokens += (long double)node_tok_len[u];
            if (row_groups > 1 && node_tok_len[u] > 0) wide = true;
        }
        if (mode == DEFT_SPLIT_BALANCED) {
            // The balanced split stretches the chunks of wide groups by itself, so the size asked for is that of
            // a narrow chunk: one dispatch round of them if the tree is small, 1024 tokens otherwise (measured on
            // the reasoning and long-context trees: 1024 and 1280 are level, 768 costs 2-3 %, 1536 and above 30 %:
            // the chunks of the widest groups then reach the 4096-token limit and leave too few tasks to share
            // compute units with the streaming narrow ones).
            int64_t chunk = ((int64_t)(reached_tokens * Hkv / 512.0L) + 127) / 128 * 128;
            return (int32_t)std::max<int64_t>(128, std::min<int64_t>(1024, chunk));
        }
        const long double per_task = task_tokens * Hkv / 512.0L;
        // a multiple of 128 tokens = 4 waves x 32-token blocks, so a token-split task gives every wave the same work.
        // Above one dispatch round, tasks of about 768 tokens stream best (measured on few-shot trees of 10 to 50
        // branches); trees with groups wider than a task gain from fewer, longer chunks (fewer partial results).
        int64_t chunk = ((int64_t)per_task + 127) / 128 * 128;
        chunk = std::max<int64_t>(128, std::min<int64_t>(wide ? 1024 : 768, chunk));
        return (int32_t)chunk;
    } catch (...) {
        return DEFT_ENOMEM;
    }
}

extern "C" int deft_plan_view(const deft_plan_t *P, deft_plan_view_t *out) {
    if (!P || !out) return DEFT_EINVAL;
    out->chunk_size = P->chunk_size;
    out->n_nodes = P->n_nodes;
    out->nq = P->nq;
    out->n_flat = P->n_flat;
    out->n_chunks = P->n_chunks();
    out->n_segs = P->n_segs();
    out->n_slots = P->n_slots();
    out->n_mask_words = (int32_t)P->seg_mask.size();
    out->q_order = P->q_order.data();
    out->node_q_lo = P->node_q_lo.data();
    out->node_q_hi = P->node_q_hi.data();
    out->chunk_seg_ptr = P->chunk_seg_ptr.data();
    out->seg_tok_begin = P->seg_tok_begin.data();
    out->seg_len = P->seg_len.data();
    out->seg_qlo = P->seg_qlo.data();
    out->seg_qhi = P->seg_qhi.data();
    out->seg_node = P->seg_node.data();
    out->chunk_qlo = P->chunk_qlo.data();
    out->chunk_qhi = P->chunk_qhi.data();
    out->chunk_slot_base = P->chunk_slot_base.data();
    out->seg_mask_ptr = P->seg_mask_ptr.data();
    out->seg_mask = P->seg_mask.data();
    out->q_part_ptr = P->q_part_ptr.data();
    out->q_part_chunk = P->q_part_chunk.data();
    out->q_part_slot = P->q_part_slot.data();
    return DEFT_OK;
}

extern "C" void deft_plan_destroy(deft_plan_t *plan) { delete plan; }

extern "C" const char *deft_strerror(int status) {
    switch (status) {
        case DEFT_OK: return "ok";
        case DEFT_EINVAL: return "invalid argument";
        case DEFT_ENOMEM: return "out of host memory";
        case DEFT_EWORKSPACE: return "workspace or plan image buffer too small";
        case DEFT_EHIP: return "HIP runtime error";
        case DEFT_ENOTREADY: return "no plan image was built for this Hq/Hkv ratio";
        default: return "unknown status";
    }
}

// ------------------------------------------------------------------------------------------------
// Launch schedule.  The rows of a chunk's group, seen from one KV head, are (query of the group) x
// (the G query heads that read this KV head): R = w * G rows, tiled 16 at a time (the N dimension
// of the 16x16x32 MFMA).  A task covers up to eight row tiles of one chunk and is run by a workgroup
// of four waves; wider groups are cut into several tasks that re-read the chunk from L2.  The kernel
// numbers its workgroups task * Hkv + kv_head, so the tasks that re-read one chunk for one head sit
// Hkv workgroups apart; with Hkv a multiple of 8 and workgroups dealt round-robin to the 8 XCDs they
// meet in the same L2.
// ------------------------------------------------------------------------------------------------
namespace deft {

static size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

static void build_schedule(const deft_plan_t *P, int32_t G, Schedule &S) {
    S.group = G;
    S.table_len = 32;
    const int32_t m = P->n_chunks();
    std::vector<int32_t> items;
    std::vector<int32_t> seg_off(P->n_segs(), 0);
    for (int32_t c = 0; c < m; ++c) {
        const int32_t s0 = P->chunk_seg_ptr[c], s1 = P->chunk_seg_ptr[c + 1];
        int32_t len = 0;
        for (int32_t s = s0; s < s1; ++s) {
            seg_off[s] = len;
            len += P->seg_len[s];
        }
        if (s1 - s0 > 1) S.table_len = std::max(S.table_len, (len + 31) / 32 * 32);
        const int32_t width = P->chunk_qhi[c] - P->chunk_qlo[c];
        const int64_t rows = (int64_t)width * G;
        const int32_t tiles = (int32_t)((rows + 15) / 16);
        // two-term softmax weights where some query of the group has a short path
        int32_t precise = P->precise_all ? 1 : 0;
        for (int32_t p = P->chunk_qlo[c]; p < P->chunk_qhi[c] && !precise; ++p)
            if (P->q_path_len[p] < kPreciseBelowTokens) precise = 1;
        // Groups of more than kMaxTilesPerTask tiles become several tasks of (nearly) equal size: the row groups
        // of one chunk then cost the same, are dispatched next to each other and find the chunk in L2 after the
        // first of them has fetched it.
        const int32_t n_tasks = (tiles + kMaxTilesPerTask - 1) / kMaxTilesPerTask;
        const int32_t per_task = n_tasks ? (tiles + n_tasks - 1) / n_tasks : 0;
        for (int32_t t0 = 0; t0 < tiles; t0 += per_task) {
            int32_t d[kItemInts] = {0};
            d[kItChunk] = c;
            d[kItTile0] = t0;
            d[kItNTiles] = std::min<int32_t>(per_task, tiles - t0);
            d[kItSeg0] = s0;
            d[kItNSeg] = s1 - s0;
            d[kItQlo] = P->chunk_qlo[c];
            d[kItWidth] = width;
            d[kItSlotBase] = P->chunk_slot_base[c];
            d[kItLen] = len;
            d[kItBegin0] = P->seg_tok_begin[s0];
            d[kItSegQlo0] = P->seg_qlo[s0];
            d[kItSegQhi0] = P->seg_qhi[s0];
            d[kItPrecise] = precise;
            d[kItCostTiles] = per_task;
            items.insert(items.end(), d, d + kItemInts);
        }
    }

    // Dispatch order: workgroups are handed to compute units in the order of the task list, a new one
    // whenever a slot frees, so the longest tasks go first (tokens x (2 + row tiles) as the estimate) and
    // the short ones fill the tail.  The row groups of one chunk share one estimate (that of the largest of
    // them) and equal estimates keep their chunk order, which leaves them next to each other: they re-read
    // that chunk from the same L2 while it is still there.
    {
        const int32_t n = (int32_t)(items.size() / kItemInts);
        std::vector<int32_t> order(n);
        for (int32_t i = 0; i < n; ++i) order[i] = i;
        auto cost = [&](int32_t i) {
            return (int64_t)items[(size_t)i * kItemInts + kItLen] * (2 + items[(size_t)i * kItemInts + kItCostTiles]);
        };
        auto precise = [&](int32_t i) { return items[(size_t)i * kItemInts + kItPrecise]; };
        // tasks with two-term weights run in a kernel of their own and come last in the list
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
            if (precise(x) != precise(y)) return precise(x) < precise(y);
            return cost(x) > cost(y);
        });
        S.n_items_precise = 0;
        for (int32_t i = 0; i < n; ++i) S.n_items_precise += precise(i);
        std::vector<int32_t> sorted(items.size());
        for (int32_t i = 0; i < n; ++i)
            std::memcpy(&sorted[(size_t)i * kItemInts], &items[(size_t)order[i] * kItemInts], kItemInts * sizeof(int32_t));
        items.swap(sorted);
    }

    size_t off = 0;
    auto place = [&](size_t count) {
        size_t at = off;
        off = align16(off + count * sizeof(int32_t));
        return at;
    };
    const int32_t nseg = P->n_segs(), nq = P->nq, slots = P->n_slots();
    S.off_seg_tok_begin = place(nseg);
    S.off_seg_len = place(nseg);
    S.off_seg_qlo = place(nseg);
    S.off_seg_qhi = place(nseg);
    S.off_seg_off = place(nseg);
    S.off_q_order = place(nq);
    S.off_q_part_ptr = place(nq + 1);
    S.off_q_part_slot = place(slots);
    off = (off + 63) & ~(size_t)63;  // per-query records and descriptors are aligned 64-byte records
    S.off_q_head = place((size_t)nq * kQueryHeadInts);
    S.n_items = (int32_t)(items.size() / kItemInts);
    S.off_items = place(items.size());
    S.bytes = std::max<size_t>(off, 16);
    S.host_image.assign(S.bytes, 0);
    auto put = [&](size_t at, const std::vector<int32_t> &v) {
        if (!v.empty()) std::memcpy(S.host_image.data() + at, v.data(), v.size() * sizeof(int32_t));
    };
    put(S.off_seg_tok_begin, P->seg_tok_begin);
    put(S.off_seg_len, P->seg_len);
    put(S.off_seg_qlo, P->seg_qlo);
    put(S.off_seg_qhi, P->seg_qhi);
    put(S.off_seg_off, seg_off);
    put(S.off_q_order, P->q_order);
    put(S.off_q_part_ptr, P->q_part_ptr);
    put(S.off_q_part_slot, P->q_part_slot);
    put(S.off_items, items);
    {
        std::vector<int32_t> head((size_t)nq * kQueryHeadInts, 0);
        for (int32_t p = 0; p < nq; ++p) {
            int32_t *r = &head[(size_t)p * kQueryHeadInts];
            const int32_t s0 = P->q_part_ptr[p], n = P->q_part_ptr[p + 1] - s0;
            r[0] = n;
            r[1] = P->q_order[p];
            for (int32_t k = 0; k < kQueryInlineSlots && k < n; ++k) r[2 + k] = P->q_part_slot[s0 + k];
        }
        put(S.off_q_head, head);
    }
}

const Schedule *get_schedule(const deft_plan_t *plan, int32_t group) {
    std::lock_guard<std::mutex> lock(plan->mu);
    auto it = plan->schedules.find(group);
    if (it == plan->schedules.end()) {
        Schedule S;
        build_schedule(plan, group, S);
        it = plan->schedules.emplace(group, std::move(S)).first;
    }
    return &it->second;
}

const Schedule *find_schedule(const deft_plan_t *plan, int32_t group) {
    std::lock_guard<std::mutex> lock(plan->mu);
    auto it = plan->schedules.find(group);
    return it == plan->schedules.end() ? nullptr : &it->second;
}

}  // namespace deft

extern "C" size_t deft_plan_device_bytes(const deft_plan_t *plan, int32_t Hq, int32_t Hkv) {
    if (!plan || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return 0;
    try {
        return deft::get_schedule(plan, Hq / Hkv)->bytes;
    } catch (...) {
        return 0;
    }
}

extern "C" size_t deft_workspace_bytes(const deft_plan_t *plan, int32_t Hq, int32_t Hkv, int32_t d) {
    if (!plan || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || (d != 64 && d != 128)) return 0;
    const size_t rows = (size_t)plan->n_slots() * (size_t)Hq;
    // acc [slots, Hq, d] + m [slots, Hq] + l [slots, Hq], fp32; never zero so callers can allocate it
    return std::max<size_t>(16, (rows * (size_t)d + 2 * rows) * sizeof(float) + 32);
}
