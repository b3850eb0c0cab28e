// Internal definitions shared by the planner (host C++) and the decode launcher (HIP).
#pragma once

#include <cstdint>
#include <map>
#include <mutex>
#include <vector>

#include "deft.h"

namespace deft {

// A stage-1 task is a (chunk, range of up to eight 16-row tiles) pair; with the KV head taken from the
// workgroup id it is the job of one workgroup.  Its descriptor is kItemInts int32, read with scalar
// loads, and carries everything the workgroup needs to start streaming a single-segment chunk
// without touching any other table.
constexpr int kItemInts = 16;
constexpr int kMaxTilesPerTask = 8;
// Stage 2 reads one kQueryHeadInts-int32 record per plan query: {number of partials n, caller's query index,
// the first kQueryInlineSlots slot ids}; queries with more partials go on to the CSR lists.
constexpr int kQueryHeadInts = 32;
constexpr int kQueryInlineSlots = kQueryHeadInts - 2;
enum ItemField {
    kItChunk = 0,     // chunk id
    kItTile0 = 1,     // first 16-row tile of the chunk's group handled by this task
    kItNTiles = 2,    // number of tiles, 1..kMaxTilesPerTask
    kItSeg0 = 3,      // first segment of the chunk
    kItNSeg = 4,      // number of segments
    kItQlo = 5,       // chunk_qlo
    kItWidth = 6,     // chunk_qhi - chunk_qlo
    kItSlotBase = 7,  // chunk_slot_base
    kItLen = 8,       // tokens in the chunk
    kItBegin0 = 9,    // first segment: physical row of its first token,
    kItSegQlo0 = 10,  //                its query interval
    kItSegQhi0 = 11,
    kItPrecise = 12,  // 1: the softmax weights enter the products as two bf16 terms (short paths, or on request)
    kItCostTiles = 13,  // host only: tiles of the largest task of this chunk, the key of the dispatch order
};
// A group one of whose queries has fewer tokens than this on its whole path gets two-term weights.
constexpr int kPreciseBelowTokens = 1024;

// Launch schedule + image layout for one Hq/Hkv ratio.
struct Schedule {
    int32_t group = 0;        // G = Hq / Hkv, rows per query within one KV head
    size_t bytes = 0;         // total image size
    // byte offsets of the canonical arrays inside the image
    size_t off_seg_tok_begin = 0, off_seg_len = 0, off_seg_qlo = 0, off_seg_qhi = 0, off_seg_off = 0;
    size_t off_q_order = 0;
    size_t off_q_part_ptr = 0, off_q_part_slot = 0;
    size_t off_q_head = 0;    // per-query records for stage 2
    size_t off_items = 0;     // task descriptors
    int32_t n_items = 0;
    int32_t n_items_precise = 0;  // the last n_items_precise tasks of the list want two-term weights
    int32_t table_len = 32;   // longest chunk made of several pieces, rounded up to whole blocks: LDS table size
    std::vector<uint8_t> host_image;  // packed image, kept for repeated uploads
};

}  // namespace deft

struct deft_plan_s {
    int32_t chunk_size = 0, n_nodes = 0, nq = 0, ntok = 0, n_flat = 0;
    uint32_t mode = 0;  // DEFT_SPLIT_* / DEFT_GROUP_QUERY
    bool precise_all = false;  // DEFT_PRECISE_WEIGHTS was given
    std::vector<int32_t> q_path_len;  // tokens on the whole path of plan position p (saturating)

    // What the plan was built from and where its chunks start, kept so that deft_plan_update can tell what a new
    // tree has in common with this one and take over the chunks in front of the first change.
    uint32_t flags = 0;
    std::vector<int32_t> in_parent, in_query_node, in_tok_len, in_ext_ptr, in_ext_begin, in_ext_len;
    std::vector<int32_t> pre;              // depth-first order of the nodes
    std::vector<int32_t> chunk_first_i;    // position in `pre` of the node of a chunk's first piece,
    std::vector<int32_t> chunk_first_done; // tokens of that node that lie in earlier chunks,
    std::vector<int32_t> chunk_last_i;     // position in `pre` of the node of its last piece,
    std::vector<int64_t> chunk_flat_begin; // flattened position of its first token
    std::vector<int32_t> q_order, node_q_lo, node_q_hi;
    std::vector<int32_t> chunk_seg_ptr, seg_tok_begin, seg_len, seg_qlo, seg_qhi, seg_node;
    std::vector<int32_t> chunk_qlo, chunk_qhi, chunk_slot_base;
    std::vector<int32_t> seg_mask_ptr;
    std::vector<uint64_t> seg_mask;
    std::vector<int32_t> q_part_ptr, q_part_chunk, q_part_slot;

    int32_t n_chunks() const { return (int32_t)chunk_qlo.size(); }
    int32_t n_segs() const { return (int32_t)seg_len.size(); }
    int32_t n_slots() const { return chunk_slot_base.empty() ? 0 : chunk_slot_base.back(); }

    // schedules by G, built on demand (the canonical arrays above never change)
    mutable std::mutex mu;
    mutable std::map<int32_t, deft::Schedule> schedules;
};

namespace deft {
// Builds (or returns the cached) schedule for G = Hq/Hkv.  Thread-safe.
const Schedule *get_schedule(const deft_plan_t *plan, int32_t group);
const Schedule *find_schedule(const deft_plan_t *plan, int32_t group);
}  // namespace deft
