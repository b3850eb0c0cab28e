// Host-only exerciser for the planner (deft_plan.cpp), built with -fsanitize=address,undefined by
// tests/test_sanitizers.py: random forests, every split, paged and contiguous storage, and corrupted inputs
// that the planner must refuse without reading or writing out of bounds.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "deft.h"

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}
static int32_t below(int32_t n) { return n > 0 ? (int32_t)(rnd() % (uint32_t)n) : 0; }

int main() {
    long plans = 0, refused = 0, chunks = 0;
    for (int it = 0; it < 3000; ++it) {
        const int32_t n = 1 + below(24), nq = below(40);
        std::vector<int32_t> begin(n), len(n), parent(n), qn(nq);
        int32_t cur = below(4);
        for (int32_t u = 0; u < n; ++u) {
            parent[u] = u == 0 ? -1 : (below(8) == 0 ? -1 : below(u));
            len[u] = below(6) == 0 ? 0 : 1 + below(200);
            begin[u] = cur;
            cur += len[u] + below(3);
        }
        int32_t ntok = cur + below(5);
        for (int32_t j = 0; j < nq; ++j) qn[j] = below(n);
        int32_t chunk = 32 * (1 + below(8));
        // one input in three is damaged
        if (it % 3 == 0) {
            switch (below(7)) {
                case 0: parent[below(n)] = n + below(3); break;
                case 1: parent[below(n)] = below(n); break;  // may close a cycle or be harmless
                case 2: len[below(n)] = -1 - below(5); break;
                case 3: begin[below(n)] = ntok + below(10); break;
                case 4: if (nq) qn[below(nq)] = n + below(4); break;
                case 5: chunk = 31 + below(3); break;
                case 6: ntok = below(ntok + 1); break;
            }
        }
        const uint32_t mode = (uint32_t)below(5);
        const uint32_t flags = mode | (below(2) ? DEFT_PRECISE_WEIGHTS : 0u) | DEFT_ROWS_PER_QUERY(1 + below(8));
        deft_plan_t *plan = nullptr;
        int rc = deft_plan(begin.data(), len.data(), parent.data(), n, nq ? qn.data() : nullptr, nq, ntok, chunk, flags,
                           &plan);
        (void)deft_suggest_chunk_size(len.data(), parent.data(), n, nq ? qn.data() : nullptr, nq, 8, 2, flags);
        if (rc == DEFT_OK) {
            deft_plan_view_t v;
            if (deft_plan_view(plan, &v) != DEFT_OK) return 2;
            // touch every array the view exposes, to its stated length
            long sum = 0;
            for (int32_t i = 0; i < v.nq; ++i) sum += v.q_order[i];
            for (int32_t i = 0; i <= v.n_chunks; ++i) sum += v.chunk_seg_ptr[i] + v.chunk_slot_base[i];
            for (int32_t i = 0; i < v.n_segs; ++i) sum += v.seg_tok_begin[i] + v.seg_len[i] + v.seg_qlo[i] + v.seg_qhi[i] + v.seg_node[i];
            for (int32_t i = 0; i <= v.n_segs; ++i) sum += v.seg_mask_ptr[i];
            for (int32_t i = 0; i < v.n_mask_words; ++i) sum += (long)(v.seg_mask[i] & 1);
            for (int32_t i = 0; i <= v.nq; ++i) sum += v.q_part_ptr[i];
            for (int32_t i = 0; i < v.n_slots; ++i) sum += v.q_part_chunk[i] + v.q_part_slot[i];
            if (sum == -12345) puts("");
            // the device image for two head ratios (host packing only)
            if (deft_plan_device_bytes(plan, 8, 2) == 0 || deft_plan_device_bytes(plan, 4, 4) == 0) return 3;
            if (deft_workspace_bytes(plan, 8, 2, 128) == 0) return 4;
            chunks += v.n_chunks;
            ++plans;
            // the tree after a decode iteration or two, planned from the old plan and from scratch: same sizes
            for (int round = 0; round < 2; ++round) {
                for (int32_t u = 0; u < n; ++u)
                    if (len[u] > 0 && below(3) == 0 && u + 1 < n && begin[u] + len[u] < begin[u + 1]) ++len[u];
                if (below(5) == 0 && nq) qn[below(nq)] = below(n);
                deft_plan_t *next = nullptr, *fresh = nullptr;
                const int r1 = deft_plan_update(plan, begin.data(), len.data(), parent.data(), n, nq ? qn.data() : nullptr, nq,
                                                ntok, chunk, flags, &next);
                const int r2 = deft_plan(begin.data(), len.data(), parent.data(), n, nq ? qn.data() : nullptr, nq, ntok, chunk,
                                         flags, &fresh);
                if (r1 != r2) return 7;
                if (r1 == DEFT_OK) {
                    deft_plan_view_t a, b;
                    deft_plan_view(next, &a);
                    deft_plan_view(fresh, &b);
                    if (a.n_chunks != b.n_chunks || a.n_segs != b.n_segs || a.n_slots != b.n_slots || a.n_flat != b.n_flat) return 8;
                    for (int32_t i = 0; i < a.n_segs; ++i)
                        if (a.seg_tok_begin[i] != b.seg_tok_begin[i] || a.seg_len[i] != b.seg_len[i]) return 9;
                    deft_plan_destroy(plan);
                    plan = next;
                    deft_plan_destroy(fresh);
                    ++plans;
                } else {
                    break;
                }
            }
            deft_plan_destroy(plan);
        } else {
            if (plan) return 5;
            ++refused;
        }
        // the same tree over pages of a few sizes
        if (it % 4 == 1) {
            const int32_t P = 1 + below(20);
            std::vector<int32_t> ptr(n + 1, 0), ids;
            int32_t total = 0;
            for (int32_t u = 0; u < n; ++u) {
                const int32_t need = len[u] > 0 ? (len[u] + P - 1) / P : 0;
                total += need;
                ptr[u + 1] = total;
            }
            for (int32_t i = 0; i < total; ++i) ids.push_back(i);
            for (int32_t i = total - 1; i > 0; --i) std::swap(ids[i], ids[below(i + 1)]);
            if (it % 8 == 1 && total > 1) ids[below(total)] = ids[below(total)];  // may own a page twice
            plan = nullptr;
            rc = deft_plan_paged(ptr.data(), ids.empty() ? nullptr : ids.data(), P, total + below(3), len.data(), parent.data(), n,
                                 nq ? qn.data() : nullptr, nq, chunk, flags, &plan);
            if (rc == DEFT_OK) {
                (void)deft_plan_device_bytes(plan, 8, 2);
                ++plans;
                deft_plan_destroy(plan);
            } else {
                ++refused;
            }
        }
    }
    std::printf("plans %ld refused %ld chunks %ld\n", plans, refused, chunks);
    return plans > 1000 && refused > 100 ? 0 : 6;
}
