/*
 * libdeft -- tree-attention decode (DeFT-Flatten) for AMD MI355X (gfx950), C ABI.
 *
 * Every query token of a decoding tree attends over the KV cache along its own
 * root-to-node path.  The work is split as in the paper: a host-side QKV
 * preparation phase (deft_plan) that groups each piece of KV with all queries
 * sharing it (KV-guided grouping) after flattening the tree depth-first and
 * cutting it into even chunks tagged with bit causal masks (Flattened Tree KV
 * Splitting), and a device-side attention phase (deft_tree_attn_decode) of
 * per-chunk partial attention followed by a log-sum-exp global reduction.
 *
 * Conventions
 *   - All functions return 0 (DEFT_OK) or a negative deft_status; nothing throws.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory on the current device.  The library allocates no device memory (only, at
 *     the first deft_plan_upload on a device, 2 MiB of pinned host memory for staging):
 *     Q/K/V/O, the plan's device image and the workspace all belong to the caller.
 *   - deft_tree_attn_decode only enqueues kernels on the given stream; it does not
 *     synchronise.  Calls that share a workspace must be ordered by the caller.
 */
#ifndef DEFT_H_
#define DEFT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum deft_status {
    DEFT_OK = 0,
    DEFT_EINVAL = -1,      /* null pointer, bad size, malformed tree, unsupported head shape */
    DEFT_ENOMEM = -2,      /* host allocation failed */
    DEFT_EWORKSPACE = -3,  /* workspace or plan image buffer too small */
    DEFT_EHIP = -4,        /* a HIP runtime call or kernel launch failed */
    DEFT_ENOTREADY = -5    /* no device image was built for this Hq/Hkv ratio (call deft_plan_upload) */
} deft_status;

/* Output element type of deft_tree_attn_decode (flags argument). */
#define DEFT_OUT_BF16 0u
#define DEFT_OUT_F32 1u

/*
 * How deft_plan partitions the tree's KV and groups it with queries (flags argument).  The paper's
 * method is DEFT_SPLIT_FLATTEN; the others are the strategies it is compared with (Table 2, the
 * split-strategy ablation of Table 6 and the IO comparison of Table 17), expressed in the same plan
 * encoding so that the same kernels run them.
 *   DEFT_SPLIT_FLATTEN     KV-guided; depth-first flatten, a cut every chunk_size tokens (Remark 3.1)
 *   DEFT_SPLIT_NODE        KV-guided; one group per tree node, chunk_size ignored (DeFT-Node, Algorithm 1)
 *   DEFT_SPLIT_NODE_CHUNK  KV-guided; every node cut into blocks of chunk_size tokens on its own
 *   DEFT_GROUP_QUERY       Q-guided; every query grouped with its own root-to-node KV, cut into blocks
 *                          of chunk_size tokens (the Flash-Decoding split): shared prefixes are read
 *                          once per query instead of once
 */
#define DEFT_SPLIT_FLATTEN 0u
#define DEFT_SPLIT_NODE 1u
#define DEFT_SPLIT_NODE_CHUNK 2u
#define DEFT_GROUP_QUERY 3u
/*
 * Not in the paper: the flattened split for a machine on which a chunk costs tokens x rows, not tokens.
 * Remark 3.1 makes chunks of equal token count because decoding is bound by reading the KV cache; on an MI355X
 * a chunk shared by hundreds of query rows is bound by the arithmetic instead, and a chunk that mixes a
 * widely shared node with narrow ones pays every token for every row of the whole group.
 *   DEFT_SPLIT_BALANCED    KV-guided; depth-first order as DEFT_SPLIT_FLATTEN, but a node piece joins the open
 *                          chunk only if the joint chunk costs no more than the two apart plus a fixed cost of
 *                          opening a chunk (cost of a chunk = tokens x t x (2 + tiles per task), for a group
 *                          of `tiles` 16-row tiles worked on by t = ceil(tiles / 8) equal tasks; opening costs
 *                          192), and a chunk may hold min(t, 4) * chunk_size tokens, so that widely shared
 *                          prefixes produce fewer partial results.  Rows = queries of the group x query heads per
 *                          KV head: or DEFT_ROWS_PER_QUERY(Hq / Hkv) to the flags (1 if absent).
 */
#define DEFT_SPLIT_BALANCED 4u
#define DEFT_ROWS_PER_QUERY(g) (((uint32_t)(g) & 0xfffu) << 16)
/*
 * May be or-ed to any of the above.  Stage 1 rounds the softmax weights to bf16 for its matrix products
 * (fp32 sums); a weight then carries a relative error of up to 2^-8.  Over a long path these errors average
 * out; a group one of whose queries has fewer than 1024 tokens on its whole path is therefore always
 * computed with two-term weights (hi + lo bf16, relative error 2^-17).  This flag asks for two-term weights
 * in every group, whatever the path lengths, at the price of half again as many matrix instructions.
 */
#define DEFT_PRECISE_WEIGHTS 0x100u

#define DEFT_DEFAULT_CHUNK 128 /* the paper's default KV block size (chunk-size ablation, Fig. 11) */
#define DEFT_MAX_CHUNK 4096

typedef struct deft_plan_s deft_plan_t;

/*
 * Host view of the canonical plan (borrowed pointers, valid until deft_plan_destroy).
 * The arrays are the outputs of the QKV Preparation Phase of DeFT-Flatten
 * (Algorithm 3; Remark 3.1), encoded as follows.
 *
 *   Depth-first flatten: children in ascending node id, roots ascending.  Queries are
 *   renumbered in that order ("plan positions", ties by caller index) so that the queries
 *   whose path contains node u are exactly positions [node_q_lo[u], node_q_hi[u]);
 *   q_order[p] is the caller's index of plan position p.  Nodes no query reaches and nodes
 *   without tokens are left out; n_flat is the flattened token count.
 *
 *   Even block-wise split: chunk c covers flattened positions [c*S, min((c+1)*S, n_flat)),
 *   n_chunks = ceil(n_flat / S).  The node pieces inside it are segments
 *   chunk_seg_ptr[c] .. chunk_seg_ptr[c+1]-1 (SubInfo): physical rows
 *   [seg_tok_begin, seg_tok_begin + seg_len) of node seg_node, shared by plan positions
 *   [seg_qlo, seg_qhi).
 *
 *   KV-guided grouping: chunk c is grouped with plan positions [chunk_qlo[c], chunk_qhi[c])
 *   (KVMapQ); its partial results occupy slots chunk_slot_base[c] + (p - chunk_qlo[c]).
 *   For plan position p, q_part_chunk / q_part_slot [q_part_ptr[p] .. q_part_ptr[p+1]) list
 *   the chunks it takes part in (QMapKV) and the slots to reduce.
 *
 *   Bit causal mask: segment s owns words seg_mask[seg_mask_ptr[s] .. seg_mask_ptr[s+1]),
 *   ceil(w/64) little-endian 64-bit words for a group of w queries; bit j = 1 means the
 *   j-th query of the chunk's group attends to the segment.
 */
typedef struct deft_plan_view {
    int32_t chunk_size, n_nodes, nq, n_flat, n_chunks, n_segs, n_slots, n_mask_words;
    const int32_t *q_order;         /* [nq] */
    const int32_t *node_q_lo;       /* [n_nodes] */
    const int32_t *node_q_hi;       /* [n_nodes] */
    const int32_t *chunk_seg_ptr;   /* [n_chunks+1] ([1] = {0} when n_chunks == 0) */
    const int32_t *seg_tok_begin;   /* [n_segs] */
    const int32_t *seg_len;         /* [n_segs] */
    const int32_t *seg_qlo;         /* [n_segs] */
    const int32_t *seg_qhi;         /* [n_segs] */
    const int32_t *seg_node;        /* [n_segs] */
    const int32_t *chunk_qlo;       /* [n_chunks] */
    const int32_t *chunk_qhi;       /* [n_chunks] */
    const int32_t *chunk_slot_base; /* [n_chunks+1] */
    const int32_t *seg_mask_ptr;    /* [n_segs+1] */
    const uint64_t *seg_mask;       /* [n_mask_words] */
    const int32_t *q_part_ptr;      /* [nq+1] */
    const int32_t *q_part_chunk;    /* [n_slots] */
    const int32_t *q_part_slot;     /* [n_slots] */
} deft_plan_view_t;

/*
 * QKV Preparation Phase of DeFT-Flatten (Algorithm 3; Section 3.3, Remark 3.1).
 *
 * node_tok_begin/len/parent : host int32[n_nodes].  Node u owns physical cache rows
 *     [begin, begin+len) of K and V; parent is a node id or -1 for a root (forests allowed).
 *     Ranges of non-empty nodes must lie in [0, ntok) and must not overlap; ids need not be
 *     in topological order.
 * query_node : host int32[nq] (may be NULL when nq == 0).  Query j attends over all tokens
 *     of all nodes on the path root -> query_node[j], that node included.  Several queries
 *     may share a node and may sit on inner nodes.
 * chunk_size : S_t, tokens per chunk; 0 selects DEFT_DEFAULT_CHUNK; otherwise a positive
 *     multiple of 32, at most DEFT_MAX_CHUNK.
 * flags      : DEFT_SPLIT_FLATTEN (0, the paper's method) or one of the comparison strategies above,
 *     optionally or-ed with DEFT_PRECISE_WEIGHTS.
 * out_plan   : receives a host object owned by the library; release with deft_plan_destroy.
 *     The plan is immutable, depends on the tree only, and can be reused for every layer
 *     and every call that sees the same tree.
 * Errors: DEFT_EINVAL for any malformed input (null pointer, n_nodes < 1, nq < 0, parent out
 *     of range or cyclic, range outside the cache or overlapping, query node out of range,
 *     bad chunk_size, unknown flags); DEFT_ENOMEM.  *out_plan is NULL on error.  With DEFT_SPLIT_NODE (or
 *     DEFT_SPLIT_BALANCED over few, very wide nodes) a chunk may be longer than chunk_size; a chunk of more
 *     than DEFT_MAX_CHUNK tokens that consists of several pieces (a paged node) is refused with DEFT_EINVAL.
 */
int deft_plan(const int32_t *node_tok_begin, const int32_t *node_tok_len, const int32_t *node_parent,
              int32_t n_nodes, const int32_t *query_node, int32_t nq, int32_t ntok, int32_t chunk_size,
              uint32_t flags, deft_plan_t **out_plan);

/*
 * The same preparation phase for a paged KV cache (the storage the paper's headline results use,
 * Section 4.2: tokens of a node are scattered over fixed-size pages of one pool and nothing is
 * materialised).  K and V are then bf16 [n_pool_pages * page_size, Hkv, d]; token t of node u is row
 * page_ids[node_page_ptr[u] + t / page_size] * page_size + t % page_size.  page_size = 1 is a
 * token-level pool.
 *
 * node_page_ptr : host int32[n_nodes+1], node_page_ptr[0] = 0; node u owns page_ids[node_page_ptr[u] ..
 *                 node_page_ptr[u+1]) and needs at least ceil(node_tok_len[u] / page_size) of them
 *                 (further ones are ignored).  A page may belong to one node only.
 * The plan is the one deft_plan would give for the same tree, except that segments are also cut
 * where a node's storage is not contiguous (consecutive pool pages are joined into one run first).
 * Everything else, including errors, is as for deft_plan; the decode calls are the same.
 */
int deft_plan_paged(const int32_t *node_page_ptr, const int32_t *page_ids, int32_t page_size, int32_t n_pool_pages,
                    const int32_t *node_tok_len, const int32_t *node_parent, int32_t n_nodes,
                    const int32_t *query_node, int32_t nq, int32_t chunk_size, uint32_t flags,
                    deft_plan_t **out_plan);

/*
 * The preparation phase for a tree that has changed since `prev` was planned.  During decoding the branch
 * controller and the KV manager change the tree between two calls of the attention kernel (Appendix A.1:
 * every live leaf gains a token, now and then a leaf forks or a branch is pruned), and the plan has to
 * follow every iteration (Fig. 9 measures latency per iteration).  The arguments after `prev` are those of
 * deft_plan / deft_plan_paged and describe the whole new tree; the result is exactly the plan those calls
 * would give for it (same arrays, same errors).  `prev` only saves work: when the parents and the query map
 * are unchanged, the depth-first order and the renumbering of the queries are taken over, and when split and
 * chunk size are unchanged as well, so is every chunk that lies in front of the first node whose tokens
 * differ, together with the chunk behind it if that one also starts in front of the change.  Anything may have
 * changed; in the worst case the call does what deft_plan does.  prev may be NULL (then it is deft_plan), is
 * not modified, and both plans stay valid and independent.
 */
int deft_plan_update(const deft_plan_t *prev, const int32_t *node_tok_begin, const int32_t *node_tok_len,
                     const int32_t *node_parent, int32_t n_nodes, const int32_t *query_node, int32_t nq, int32_t ntok,
                     int32_t chunk_size, uint32_t flags, deft_plan_t **out_plan);
int deft_plan_paged_update(const deft_plan_t *prev, const int32_t *node_page_ptr, const int32_t *page_ids,
                           int32_t page_size, int32_t n_pool_pages, const int32_t *node_tok_len,
                           const int32_t *node_parent, int32_t n_nodes, const int32_t *query_node, int32_t nq,
                           int32_t chunk_size, uint32_t flags, deft_plan_t **out_plan);

/*
 * A chunk size S_t suited to this tree on an MI355X (the paper leaves S_t as a tuning knob, Fig. 11).
 * flags names the split the size is for (a DEFT_SPLIT_* / DEFT_GROUP_QUERY value; other bits are ignored).
 * For DEFT_SPLIT_BALANCED: the multiple of 128 that gives about one stage-1 task per resident workgroup slot
 * (two per compute unit) if all chunks were narrow, at least 128 and at most 1024 (the split itself makes the
 * chunks of widely shared nodes up to four times longer).  For the other splits: the multiple of 128 that
 * makes the number of stage-1 tasks, (chunk, KV head, 128 rows of the chunk's query group), about twice the
 * number of compute units, so that every unit streams the same number of KV bytes; at least 128 and at most
 * 768, or at most 1024 when some group is wider than one task (fewer partial results).  Heuristics from
 * measurements, not optima.  Host arrays as for deft_plan (token begins are not needed).  Returns the size,
 * or a negative deft_status on malformed input.  Any valid S_t gives the same attention result.
 */
int32_t deft_suggest_chunk_size(const int32_t *node_tok_len, const int32_t *node_parent, int32_t n_nodes,
                                const int32_t *query_node, int32_t nq, int32_t Hq, int32_t Hkv, uint32_t flags);

/* Fills *out with borrowed host pointers to the canonical arrays described above. */
int deft_plan_view(const deft_plan_t *plan, deft_plan_view_t *out);

/*
 * The device image of a plan: the arrays the kernels read (segment table, chunk groups,
 * slot lists, query order) plus the launch schedule for a given ratio Hq/Hkv (how the
 * rows "query x query-head of one KV head" of each chunk's group are tiled over waves).
 * deft_plan_device_bytes returns the size the caller must provide (0 on bad arguments);
 * deft_plan_upload packs the image on the host and copies it into dev_image (device
 * memory, 16-byte aligned) on `stream` (a hipStream_t, NULL = default stream).  Images of
 * up to 256 KiB are staged in pinned host memory that the library keeps per device, and the
 * call only enqueues the copy: work enqueued on `stream` afterwards sees the image, and the
 * plan may be destroyed at once.  Larger images are copied from the plan and the call waits
 * for that copy.  One image serves one Hq/Hkv ratio; a plan may be uploaded for several.
 * Errors: DEFT_EINVAL (null, Hq <= 0, Hkv <= 0, Hq % Hkv != 0), DEFT_EWORKSPACE (bytes
 * too small), DEFT_EHIP.
 */
size_t deft_plan_device_bytes(const deft_plan_t *plan, int32_t Hq, int32_t Hkv);
int deft_plan_upload(deft_plan_t *plan, int32_t Hq, int32_t Hkv, void *dev_image, size_t bytes, void *stream);

/* Bytes of device workspace deft_tree_attn_decode needs (fp32 partial attention, running
 * maxima and sums per (slot, query head)); 0 on bad arguments. */
size_t deft_workspace_bytes(const deft_plan_t *plan, int32_t Hq, int32_t Hkv, int32_t d);

/*
 * Attention Calculation Phase of DeFT-Flatten (Algorithm 4): stage 1 computes, for every
 * QKV group, the masked partial attention of the group's queries over the chunk with an
 * online softmax (bf16 inputs, fp32 accumulation); stage 2 is the tree-topology-aware
 * global reduction of eq. 1 over each query's partial results.  The result equals
 * softmax(scale * q K^T) V over exactly the tokens on each query's path (Section 3.1).
 *
 * dev_image : device image written by deft_plan_upload for the same Hq/Hkv ratio.
 * q         : device bf16 [nq, Hq, d], caller's query order.
 * k, v      : device bf16 [ntok, Hkv, d], row-major, head dimension contiguous; node u's
 *             tokens are rows [node_tok_begin[u], +node_tok_len[u]).  16-byte aligned.  (Fast
 *             placement on MI355X: start the V pool 512 bytes past a 1 KiB boundary when the
 *             K pool starts on one, so that the K and V rows of a head differ in address
 *             bits 7..9; the Python binding's alloc_kv_cache does that.  Optional.)
 * o         : device [nq, Hq, d], bf16 (DEFT_OUT_BF16) or float (DEFT_OUT_F32), caller's
 *             query order, 16-byte aligned.  A query whose path holds no token gets zeros.
 * d         : 64 or 128.  Hq % Hkv == 0.
 * scale     : softmax scale; <= 0 selects 1/sqrt(d).
 * workspace : device memory of at least deft_workspace_bytes(plan, Hq, Hkv, d), 16-byte
 *             aligned; contents are scratch.
 * stream    : hipStream_t (NULL = default stream).  Kernels are enqueued, not awaited.  After one
 *             ordinary call on the device (which sets a kernel attribute), a call made while the
 *             stream is being captured records just its two kernel launches in the graph.
 * Errors: DEFT_EINVAL, DEFT_ENOTREADY, DEFT_EWORKSPACE, DEFT_EHIP (deft_last_hip_error
 * gives the runtime's text).  Nothing is launched when an error is returned, except that a
 * launch failure may leave earlier kernels of the same call enqueued.
 */
int deft_tree_attn_decode(const deft_plan_t *plan, const void *dev_image, const void *q, const void *k,
                          const void *v, void *o, int32_t Hq, int32_t Hkv, int32_t d, float scale,
                          uint32_t flags, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two stages of Algorithm 4 as separate calls, for callers that want to time or overlap them.
 * deft_tree_attn_decode(...) is exactly stage 1 followed by stage 2 on the same stream with the
 * same workspace and scale.  Arguments, alignment rules and errors are those of
 * deft_tree_attn_decode.
 *   stage 1: per QKV group, masked partial attention with an online softmax; writes, for every
 *            (slot, query head), the running maximum m of the raw scores q.k, the sum l of
 *            exp(scale*(s - m)) and the un-normalised sum acc of exp(scale*(s - m)) * v into the
 *            workspace (LSE = scale*m + log l and PA = acc / l in the paper's notation).
 *   stage 2: per (query, query head), the global reduction of eq. 1 over the query's slots;
 *            reads the workspace, writes o.
 */
int deft_stage1_partial_attention(const deft_plan_t *plan, const void *dev_image, const void *q, const void *k,
                                  const void *v, int32_t Hq, int32_t Hkv, int32_t d, float scale, void *workspace,
                                  size_t workspace_bytes, void *stream);
int deft_stage2_global_reduction(const deft_plan_t *plan, const void *dev_image, void *o, int32_t Hq, int32_t Hkv,
                                 int32_t d, float scale, uint32_t flags, void *workspace, size_t workspace_bytes,
                                 void *stream);

/*
 * deft_tree_attn_decode for callers that cannot allocate device memory or hold a workspace of their own
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the partial results
 * live in a fixed array of DEFT_STATIC_SCRATCH_BYTES bytes that is part of the library's device code, one
 * copy per GPU, kept until the process ends.  The call allocates nothing and frees nothing.  Arguments,
 * results and errors are those of deft_tree_attn_decode without the workspace pair; a plan whose
 * deft_workspace_bytes(plan, Hq, Hkv, d) exceeds DEFT_STATIC_SCRATCH_BYTES is refused with DEFT_EWORKSPACE
 * and nothing is launched (use a larger chunk_size, or the call with a caller workspace).  All calls on one
 * GPU share that GPU's array: calls that may overlap on one GPU (different streams, no ordering) race and
 * must be ordered by the caller; the array keeps the last call's partial results and needs no clearing,
 * because stage 2 only reads what stage 1 of the same call wrote.  The first call on a device looks up the
 * array's address and must not be made while a stream is being captured.
 */
#define DEFT_STATIC_SCRATCH_BYTES (64u << 20)
int deft_tree_attn_decode_static(const deft_plan_t *plan, const void *dev_image, const void *q, const void *k,
                                 const void *v, void *o, int32_t Hq, int32_t Hkv, int32_t d, float scale,
                                 uint32_t flags, void *stream);

/*
 * Benchmark aid, not part of the method (no decode call uses it; it exists so that the benchmark can state
 * the machine's read rate next to stage 1's).  Reads `bytes` bytes at dev_buf once with 128-bit loads from
 * every compute unit (DEFT_PROBE_SINK_BYTES / 4 workgroups, grid-stride) and stores, for each workgroup, the xor of the
 * 32-bit words it read into dev_sink (device, DEFT_PROBE_SINK_BYTES bytes, 4-byte aligned; all of it is
 * overwritten), so the xor over the sink is the xor over the buffer.  The rate it reaches is the
 * read-stream ceiling against which the benchmark states the KV read rate of stage 1 (the method is
 * bound by reading the KV cache: Section 3.3, Table 12).  bytes must be a positive multiple of 16 and
 * dev_buf 16-byte aligned (DEFT_EINVAL otherwise); asynchronous on `stream`.
 */
#define DEFT_PROBE_SINK_BYTES 8192
int deft_hbm_read_probe(const void *dev_buf, size_t bytes, void *dev_sink, void *stream);

void deft_plan_destroy(deft_plan_t *plan);

const char *deft_strerror(int status);
const char *deft_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DEFT_H_ */
