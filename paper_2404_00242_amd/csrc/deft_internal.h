// Internal definitions shared by the planner (host C++) and the decode launcher (HIP).
#pragma once

#include <cstdint>
#include <map>
#include <mutex>
#include <vector>

#include "deft.h"

namespace deft {

// One launch list of stage-1 work items.  An item is a (chunk, 16-row-tile range) pair;
// the kernel instance NT handles up to NT row tiles per wave.  Each item is two int32:
// {chunk, tile_begin | n_tiles << 24}.
struct ItemList {
    int nt = 0;               // row tiles per wave of the kernel instance that runs this list
    int32_t n_items = 0;
    size_t offset = 0;        // byte offset of the item array inside the device image
};

// Launch schedule + image layout for one Hq/Hkv ratio.
struct Schedule {
    int32_t group = 0;        // G = Hq / Hkv, rows per query within one KV head
    size_t bytes = 0;         // total image size
    // byte offsets of the canonical arrays inside the image
    size_t off_chunk_seg_ptr = 0, off_seg_tok_begin = 0, off_seg_len = 0, off_seg_qlo = 0, off_seg_qhi = 0;
    size_t off_chunk_qlo = 0, off_chunk_qhi = 0, off_chunk_slot_base = 0, off_q_order = 0;
    size_t off_q_part_ptr = 0, off_q_part_slot = 0;
    std::vector<ItemList> lists;
    std::vector<uint8_t> host_image;  // packed image, kept for repeated uploads
};

}  // namespace deft

struct deft_plan_s {
    int32_t chunk_size = 0, n_nodes = 0, nq = 0, ntok = 0, n_flat = 0;
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
