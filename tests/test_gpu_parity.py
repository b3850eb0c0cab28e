"""HIP path (through the C ABI) against the fp64 oracle, element by element.  Needs an MI355X.

Tolerance (bf16 inputs, fp32 accumulation), the stated one, on every tree:
  * the five benchmark configurations: max |err| <= 2e-3 over all elements AND, per (query, head)
    row, ||err||_2 / ||ref||_2 <= 1e-2;
  * every other tree: element-wise |err| <= 2e-3 + 1e-2 |ref| and the same row-relative bound (short
    paths give outputs of magnitude O(1), where half a bf16 ulp of the *output* already exceeds 2e-3,
    hence the relative term).
Stage 1 rounds softmax weights to bf16 for its matrix products.  Groups that contain a query with fewer
than 1024 tokens on its path use two-term weights (hi + lo bf16, relative error 2^-17), so for trees whose
paths are all that short and fp32 output the error is bounded far below the stated tolerance:
|err| <= 2^-13 * sum_t w_t |V[t, c]| + 1e-5, which is checked too (sum_t w_t |V[t, c]| is the oracle's
attention over |V|).
"""

import numpy as np
import pytest
import torch

import oracle
from oracle.plan import flatten_plan
from paper_2404_00242_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL = 2e-3, 1e-2
PRECISE_BELOW = 1024     # tokens on a path below which the library uses two-term weights
U_PRECISE = 2.0 ** -13   # bound on the relative error of a two-term weight and the fp32 sums, with margin


def mode_flags(mode, G):
    """deft_plan flags of a split; the balanced one is told how many query heads share a KV head"""
    return binding.SPLIT_MODES[mode] | (binding.rows_per_query(G) if mode == "balanced" else 0)


def run_gpu(t, Q, K, V, chunk_size=0, out_dtype=torch.bfloat16, scale=0.0, mode="flatten"):
    dev = torch.device("cuda:0")
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, chunk_size,
                             mode_flags(mode, t.Hq // t.Hkv))
    q, k, v = Q.to(dev), K.to(dev), V.to(dev)
    o = binding.deft_tree_attn_decode(plan, q, k, v, out_dtype=out_dtype, scale=scale)
    torch.cuda.synchronize()
    return o.float().cpu().numpy().astype(np.float64), plan


def reference(t, Q, K, V, scale=None):
    return oracle.tree_attention(Q, K, V, t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, scale=scale)


def reference_abs_v(t, Q, K, V, scale=None):
    """sum_t w_t |V[t, c]|: what the rounding of the weights is multiplied by (see the module docstring)"""
    return oracle.tree_attention(Q, K, V.abs(), t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node,
                                 scale=scale)


def errors(got, ref):
    err = np.abs(got - ref)
    num = np.sqrt(((got - ref) ** 2).sum(-1))
    den = np.sqrt((ref ** 2).sum(-1))
    rel = np.where(den > 0, num / np.maximum(den, 1e-300), np.where(num > 0, np.inf, 0.0))
    return err, rel


def longest_and_shortest_path(t):
    lens = []
    for u in t.query_node:
        u, n = int(u), 0
        while u >= 0:
            n += int(t.node_tok_len[u])
            u = int(t.node_parent[u])
        lens.append(n)
    return (max(lens), min(lens)) if lens else (0, 0)


def all_paths_short(t):
    """every query's path is short enough for the library to use two-term weights in every group"""
    return longest_and_shortest_path(t)[0] < PRECISE_BELOW


def check(got, ref, strict, abs_v=None, two_term=False):
    """strict: the benchmark configurations' bound, otherwise the element-wise form of the same tolerance.
    two_term (fp32 output, every path short enough for two-term weights) adds the tight bound, for which
    abs_v = reference_abs_v(...)."""
    assert np.isfinite(got).all()
    err, rel = errors(got, ref)
    above = float((err > ABS_TOL).mean())
    print(f"    max|err|={err.max():.3e} max row-rel={rel.max():.3e} max|ref|={np.abs(ref).max():.3f} "
          f"share of elements above 2e-3: {above:.2e}", flush=True)
    if strict:
        assert err.max() <= ABS_TOL
    else:
        assert (err <= ABS_TOL + REL_TOL * np.abs(ref)).all()
    assert rel.max() <= REL_TOL
    if two_term:
        frac = err / (U_PRECISE * abs_v + 1e-5)
        print(f"    two-term weights: largest error as a fraction of 2^-13 attention(|V|) + 1e-5: {frac.max():.3f}", flush=True)
        assert frac.max() <= 1.0


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_benchmark_configs_match_oracle(cfg):
    t = wl.make_config(cfg)
    print(f"\n  config {cfg}: {t.name} ntok={t.ntok} nq={t.nq} Hq={t.Hq} Hkv={t.Hkv} d={t.d}", flush=True)
    Q, K, V = wl.make_qkv(t)
    got, plan = run_gpu(t, Q, K, V)
    ref = reference(t, Q, K, V)
    check(got, ref, strict=True)
    # the plan the kernels ran on is the oracle's plan, bit for bit
    want = flatten_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 128)
    view = plan.view()
    for key in ("seg_tok_begin", "seg_len", "seg_qlo", "seg_qhi", "chunk_qlo", "chunk_qhi", "seg_mask",
                "q_part_slot", "q_order"):
        assert np.array_equal(view[key], want[key]), key


@pytest.mark.parametrize("mode", ["flatten", "balanced"])
@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_benchmark_configs_at_the_chunk_size_bench_uses(cfg, mode):
    t = wl.make_config(cfg)
    chunk = binding.deft_suggest_chunk_size(t.node_tok_len, t.node_parent, t.query_node, t.Hq, t.Hkv,
                                            binding.SPLIT_MODES[mode])
    print(f"\n  config {cfg}, {mode} split at the suggested chunk size {chunk}", flush=True)
    Q, K, V = wl.make_qkv(t)
    got, _ = run_gpu(t, Q, K, V, chunk_size=chunk, mode=mode)
    check(got, reference(t, Q, K, V), strict=True)


def test_stage1_partials_match_algorithm4_and_stage2_completes_them():
    # stage 1 alone, in the paper's notation: LSE_i = scale*m + ln(l), PA_i = acc / l per (slot, head)
    from oracle import deft_flatten

    t = wl.random_tree(7, n_nodes=11, max_len=90, nq=21, Hq=8, Hkv=2, d=128, n_roots=2)
    Q, K, V = wl.make_qkv(t)
    dev = torch.device("cuda:0")
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 64)
    lib = binding.load_library()
    q, k, v = Q.to(dev), K.to(dev), V.to(dev)
    img = plan.image(t.Hq, t.Hkv, dev)
    ws = plan.workspace(t.Hq, t.Hkv, t.d, dev)
    ws.zero_()
    st = torch.cuda.current_stream().cuda_stream
    rc = lib.deft_stage1_partial_attention(plan.handle, img.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                           t.Hq, t.Hkv, t.d, 0.0, ws.data_ptr(), ws.numel(), st)
    assert rc == 0
    torch.cuda.synchronize()
    view = plan.view()
    rows = view["n_slots"] * t.Hq
    wsf = ws.view(torch.float32).cpu().numpy().astype(np.float64)
    acc = wsf[:rows * t.d].reshape(view["n_slots"], t.Hq, t.d)
    m = wsf[rows * t.d:rows * t.d + rows].reshape(view["n_slots"], t.Hq)
    l = wsf[rows * t.d + rows:rows * t.d + 2 * rows].reshape(view["n_slots"], t.Hq)
    want_o, want_lse = deft_flatten.partials_by_plan(view, Q.float().numpy(), K.float().numpy(), V.float().numpy())
    seen = np.isfinite(want_lse)
    assert np.array_equal(seen, l > 0)
    scale = 1.0 / np.sqrt(t.d)
    lse = scale * m[seen] + np.log(l[seen])
    assert np.abs(lse - want_lse[seen]).max() <= 2e-3
    pa = acc[seen] / l[seen][:, None]
    assert (np.abs(pa - want_o[seen]) <= ABS_TOL + REL_TOL * np.abs(want_o[seen])).all()
    # stage 2 on those partials gives the attention
    o = torch.empty((t.nq, t.Hq, t.d), dtype=torch.float32, device=dev)
    rc = lib.deft_stage2_global_reduction(plan.handle, img.data_ptr(), o.data_ptr(), t.Hq, t.Hkv, t.d, 0.0, 1,
                                          ws.data_ptr(), ws.numel(), st)
    assert rc == 0
    torch.cuda.synchronize()
    check(o.cpu().numpy().astype(np.float64), reference(t, Q, K, V), strict=False, abs_v=reference_abs_v(t, Q, K, V),
          two_term=all_paths_short(t))


@pytest.mark.parametrize("mode", ["node", "node_chunk", "query", "balanced"])
def test_other_partitioning_strategies_give_the_same_attention(mode):
    # DeFT-Node, DeFT-Node-Chunk, Q-guided grouping and the tokens x rows split run on the same kernels through the plan
    for cfg in (1, 2, 3):
        t = wl.make_config(cfg)
        print(f"\n  config {cfg} mode {mode}", flush=True)
        Q, K, V = wl.make_qkv(t)
        got, _ = run_gpu(t, Q, K, V, chunk_size=128, mode=mode)
        check(got, reference(t, Q, K, V), strict=True)
    for seed in range(6):
        t = wl.random_tree(500 + seed, n_nodes=3 + 2 * seed, max_len=150, nq=3 + 4 * seed, Hq=8, Hkv=2, d=128,
                           n_roots=1 + seed % 2)
        Q, K, V = wl.make_qkv(t)
        got, _ = run_gpu(t, Q, K, V, chunk_size=64, out_dtype=torch.float32, mode=mode)
        check(got, reference(t, Q, K, V), strict=False, abs_v=reference_abs_v(t, Q, K, V), two_term=all_paths_short(t))


def test_tiny_variant_with_320_tokens():
    t = wl.config1_tiny(leaf_len=16)
    Q, K, V = wl.make_qkv(t)
    got, _ = run_gpu(t, Q, K, V)
    check(got, reference(t, Q, K, V), strict=True)


@pytest.mark.parametrize("cfg,chunk", [(2, 32), (2, 512), (3, 32), (3, 4096), (4, 1024), (5, 2048)])
def test_other_chunk_sizes(cfg, chunk):
    # the result does not depend on S_t (the paper's chunk-size ablation only moves latency)
    t = wl.make_config(cfg)
    print(f"\n  config {cfg} chunk {chunk}", flush=True)
    Q, K, V = wl.make_qkv(t)
    got, _ = run_gpu(t, Q, K, V, chunk_size=chunk)
    check(got, reference(t, Q, K, V), strict=True)


@pytest.mark.parametrize("seed", range(24))
def test_random_forests(seed):
    # ragged node lengths, zero-length and unreached nodes, repeated / inner-node queries, shuffled and
    # gapped cache, forests; sizes span several 32-token blocks, several chunks and a ragged tail
    shapes = [(4, 4, 64), (8, 2, 128), (32, 8, 128), (6, 1, 128), (2, 2, 64), (12, 4, 128)]
    Hq, Hkv, d = shapes[seed % len(shapes)]
    t = wl.random_tree(seed, n_nodes=2 + seed % 19, max_len=40 + 17 * (seed % 7), nq=1 + (seed * 3) % 29,
                       Hq=Hq, Hkv=Hkv, d=d, n_roots=1 + seed % 3)
    print(f"\n  seed {seed}: nodes={t.n_nodes} ntok={t.ntok} nq={t.nq} Hq={Hq} Hkv={Hkv} d={d}", flush=True)
    Q, K, V = wl.make_qkv(t)
    ref, abs_v = reference(t, Q, K, V), reference_abs_v(t, Q, K, V)
    for chunk in (32, 128):
        got, _ = run_gpu(t, Q, K, V, chunk_size=chunk, out_dtype=torch.float32)
        check(got, ref, strict=False, abs_v=abs_v, two_term=all_paths_short(t))
    got, _ = run_gpu(t, Q, K, V, chunk_size=64)
    check(got, ref, strict=False)


def test_wide_groups_and_many_row_tiles():
    # 150 queries x 4 query heads per KV head = 600 rows on the shared root: 38 row tiles, ten waves per chunk
    t = wl._finish("star", [300] + [5] * 150, [-1] + [0] * 150, list(range(1, 151)), 8, 2, 128, 77)
    Q, K, V = wl.make_qkv(t)
    got, _ = run_gpu(t, Q, K, V, out_dtype=torch.float32)
    check(got, reference(t, Q, K, V), strict=False, abs_v=reference_abs_v(t, Q, K, V), two_term=True)


@pytest.mark.parametrize("root_len", [1, 2, 3, 31, 33, 34, 35, 63, 64, 65, 97, 161])
@pytest.mark.parametrize("nq,G", [(12, 4), (20, 4), (30, 4)])  # 48, 80 and 120 rows: 3, 5 and 8 row tiles
def test_wide_single_piece_chunks_with_ragged_last_blocks(root_len, nq, G):
    """Wide groups over one node whose last 32-token block holds 1, 2, 3 ... rows, both paths of the pipelined
    loop (a tile per wave, two tiles per wave), long paths (bf16 weights) and short ones, d = 128 (addressed
    from a block pointer and a clamped row) and d = 64 (general addressing).  The clamp of the last block's
    rows is what these shapes exercise: the loads of a wave that fetches V cover four consecutive rows."""
    for d in (128, 64):
        for pad in (0, 1100):  # pad: a second, long node above the shared one lifts every path over 1024 tokens
            if pad:
                lens, par, qn = [pad, root_len] + [1] * nq, [-1, 0] + [1] * nq, list(range(2, nq + 2))
            else:
                lens, par, qn = [root_len] + [1] * nq, [-1] + [0] * nq, list(range(1, nq + 1))
            t = wl._finish("ragged", lens, par, qn, 2 * G, 2, d, 500 + root_len + nq)
            Q, K, V = wl.make_qkv(t)
            ref = reference(t, Q, K, V)
            for mode in ("flatten", "node"):
                got, _ = run_gpu(t, Q, K, V, chunk_size=4096, out_dtype=torch.float32, mode=mode)
                check(got, ref, strict=False)


def test_explicit_scale_and_empty_paths():
    t = wl.random_tree(3, n_nodes=6, max_len=50, nq=5, Hq=4, Hkv=2, d=128)
    Q, K, V = wl.make_qkv(t)
    got, _ = run_gpu(t, Q, K, V, out_dtype=torch.float32, scale=0.31)
    check(got, reference(t, Q, K, V, scale=0.31), strict=False, abs_v=reference_abs_v(t, Q, K, V, scale=0.31),
          two_term=True)
    # queries whose path has no token: zeros, and no kernel reads K/V
    t2 = wl._finish("empty", [0, 0, 7], [-1, 0, -1], [1, 1, 2], 4, 2, 64, 5, begins=[0, 0, 0], ntok=7)
    Q, K, V = wl.make_qkv(t2)
    got, _ = run_gpu(t2, Q, K, V, out_dtype=torch.float32)
    assert np.all(got[:2] == 0)
    check(got, reference(t2, Q, K, V), strict=False, abs_v=reference_abs_v(t2, Q, K, V), two_term=True)
    # no queries at all
    t3 = wl._finish("noq", [9], [-1], [], 4, 2, 64, 5)
    Q, K, V = wl.make_qkv(t3)
    got, _ = run_gpu(t3, Q, K, V)
    assert got.shape == (0, 4, 64)


def test_repeated_calls_and_plan_reuse_are_deterministic():
    t = wl.make_config(1)
    Q, K, V = wl.make_qkv(t)
    dev = torch.device("cuda:0")
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok)
    q, k, v = Q.to(dev), K.to(dev), V.to(dev)
    a = binding.deft_tree_attn_decode(plan, q, k, v).clone()
    for _ in range(3):
        b = binding.deft_tree_attn_decode(plan, q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    # a side stream works too
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        c = binding.deft_tree_attn_decode(plan, q, k, v, stream=s)
    s.synchronize()
    assert torch.equal(a, c)
    # also when the image's upload is still queued on another stream: the first call (which uploads) sits behind
    # a long fill on the current stream, the second call comes on a side stream that waits for nothing but the
    # workspace's owner; the binding orders it behind the upload
    plan3 = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok)
    big = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    for _ in range(3):
        big.add_(1)
    plan3.image(t.Hq, t.Hkv, dev)                      # upload enqueued behind the fills
    s2 = torch.cuda.Stream()
    ws2 = torch.empty(plan3.workspace_bytes(t.Hq, t.Hkv, t.d), dtype=torch.uint8, device=dev)
    with torch.cuda.stream(s2):
        e = binding.deft_tree_attn_decode(plan3, q, k, v, workspace=ws2, stream=s2)
    s2.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(a, e)


def test_error_paths_do_not_launch():
    t = wl.make_config(1)
    Q, K, V = wl.make_qkv(t)
    dev = torch.device("cuda:0")
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok)
    q, k, v = Q.to(dev), K.to(dev), V.to(dev)
    with pytest.raises(binding.DeftError):   # cache shorter than the plan's rows
        binding.deft_tree_attn_decode(plan, q, k[:100].contiguous(), v[:100].contiguous())
    with pytest.raises(binding.DeftError):   # CPU tensors: there is no CPU path
        binding.deft_tree_attn_decode(plan, Q, K, V)
    small = torch.empty(64, dtype=torch.uint8, device=dev)
    with pytest.raises(binding.DeftError) as e:
        binding.deft_tree_attn_decode(plan, q, k, v, workspace=small)
    assert e.value.status == -3
    lib = binding.load_library()
    o = torch.empty_like(q)
    ws = plan.workspace(4, 4, 64, dev)
    # decode before any image exists for this head ratio
    plan2 = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok)
    rc = lib.deft_tree_attn_decode(plan2.handle, ws.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                   o.data_ptr(), 4, 4, 64, 0.0, 0, ws.data_ptr(), ws.numel(), None)
    assert rc == -5
    rc = lib.deft_tree_attn_decode(plan.handle, plan.image(4, 4, dev).data_ptr(), q.data_ptr(), k.data_ptr(),
                                   v.data_ptr(), o.data_ptr(), 4, 4, 96, 0.0, 0, ws.data_ptr(), ws.numel(), None)
    assert rc == -1
    torch.cuda.synchronize()


def test_read_probe_reads_every_word_once():
    """The read-stream probe leaves the xor of every 32-bit word of the buffer in its sink (so no load can have been
    skipped), for a buffer that is not a multiple of the grid and for a tiny one; bad sizes are refused."""
    import ctypes

    lib = binding.load_library()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    g = torch.Generator().manual_seed(11)
    for n_words in (4, 4 * 1000 + 4, 4 * (1 << 20) + 12):
        n_words -= n_words % 4
        host = torch.randint(-2**31, 2**31 - 1, (n_words,), generator=g, dtype=torch.int32)
        buf = host.cuda()
        sink = torch.full((2048,), 77, dtype=torch.int32, device="cuda")
        rc = lib.deft_hbm_read_probe(ctypes.c_void_p(buf.data_ptr()), n_words * 4, ctypes.c_void_p(sink.data_ptr()), st)
        assert rc == 0
        torch.cuda.synchronize()
        want = int(np.bitwise_xor.reduce(host.numpy().view(np.uint32)))
        assert int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))) == want
    assert lib.deft_hbm_read_probe(ctypes.c_void_p(buf.data_ptr()), 24, ctypes.c_void_p(sink.data_ptr()), st) == -1
    assert lib.deft_hbm_read_probe(None, 16, ctypes.c_void_p(sink.data_ptr()), st) == -1


def test_staggered_kv_pools_are_placed_as_documented_and_decode_the_same():
    t = wl.config1_tiny()
    Q, K, V = wl.make_qkv(t)
    k, v = binding.alloc_kv_cache(t.ntok, t.Hkv, t.d)
    assert k.shape == v.shape == (t.ntok, t.Hkv, t.d) and k.dtype == v.dtype == torch.bfloat16
    assert k.data_ptr() % 1024 == 0 and v.data_ptr() % 1024 == binding.KV_STAGGER_BYTES
    assert v.data_ptr() >= k.data_ptr() + k.numel() * 2  # no overlap
    k.copy_(K)
    v.copy_(V)
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 128)
    a = binding.deft_tree_attn_decode(plan, Q.cuda(), k, v)
    b = binding.deft_tree_attn_decode(plan, Q.cuda(), K.cuda(), V.cuda())
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("Hq,Hkv,d", [(6, 3, 128), (5, 5, 64), (14, 7, 128), (24, 24, 64)])
def test_head_counts_that_do_not_divide_the_dispatch_round(Hq, Hkv, d):
    """More than 256 workgroups with a KV-head count that does not divide 256: the head a workgroup takes is
    moved on per dispatch round, and every (task, head) pair must still be visited exactly once."""
    n_leaves = 120
    t = wl._finish("many_tasks", [3000] + [33] * n_leaves, [-1] + [0] * n_leaves, list(range(1, n_leaves + 1)),
                   Hq, Hkv, d, 91)
    Q, K, V = wl.make_qkv(t)
    got, plan = run_gpu(t, Q, K, V, chunk_size=32, out_dtype=torch.float32)
    assert plan.view()["n_chunks"] * Hkv > 512
    check(got, reference(t, Q, K, V), strict=False)


def test_rows_beyond_four_gigabytes_are_addressed_correctly():
    """KV pools larger than 4 GiB: the rows of the far node start 4.5 GB into each pool.  The oracle runs on a
    compact cache holding the same tokens (moving nodes leaves the attention unchanged)."""
    Hq, Hkv, d = 32, 32, 128
    n_rows = 600_000                       # x 8 KiB per row = 4.9 GB per pool
    lens = [150, 300, 40]
    begins_far = [10, 550_000, 599_950]    # root near the start, the others beyond 2^32 bytes
    parents = [-1, 0, 1]
    qn = [2, 1, 2]
    compact = wl._finish("compact", lens, parents, qn, Hq, Hkv, d, 123)
    Q, K, V = wl.make_qkv(compact)
    ref, abs_v = reference(compact, Q, K, V), reference_abs_v(compact, Q, K, V)
    k = torch.empty((n_rows, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v = torch.empty((n_rows, Hkv, d), dtype=torch.bfloat16, device="cuda")
    for u in range(3):
        b0, n = int(compact.node_tok_begin[u]), lens[u]
        k[begins_far[u]:begins_far[u] + n] = K[b0:b0 + n].cuda()
        v[begins_far[u]:begins_far[u] + n] = V[b0:b0 + n].cuda()
    plan = binding.deft_plan(begins_far, lens, parents, qn, n_rows, 64)
    got = binding.deft_tree_attn_decode(plan, Q.cuda(), k, v, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check(got.cpu().numpy().astype(np.float64), ref, strict=False, abs_v=abs_v, two_term=True)


def test_decode_calls_captured_in_a_hip_graph_replay_to_the_eager_result():
    """A decode call only enqueues two kernels on the caller's stream, so a layer loop can be captured once and
    replayed.  Several replays, with eager work and synchronisations between them and fresh inputs written into
    the captured buffers, each give exactly what the eager call gives."""
    t = wl.random_tree(21, n_nodes=14, max_len=300, nq=11, Hq=8, Hkv=4, d=128)
    L = 3
    plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 128)
    g = torch.Generator().manual_seed(5)

    def fresh():
        return [torch.randn((t.nq, t.Hq, t.d), generator=g).to(torch.bfloat16).cuda() for _ in range(L)], \
               [torch.randn((t.ntok, t.Hkv, t.d), generator=g).to(torch.bfloat16).cuda() for _ in range(L)], \
               [torch.randn((t.ntok, t.Hkv, t.d), generator=g).to(torch.bfloat16).cuda() for _ in range(L)]

    qs, ks, vs = fresh()
    outs = [torch.empty((t.nq, t.Hq, t.d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    ws = plan.workspace(t.Hq, t.Hkv, t.d, "cuda")
    # eager warm-up: uploads the image and sets the kernel's LDS limit, neither of which belongs in a graph
    for i in range(L):
        binding.deft_tree_attn_decode(plan, qs[i], ks[i], vs[i], out=outs[i], workspace=ws)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(L):
            binding.deft_tree_attn_decode(plan, qs[i], ks[i], vs[i], out=outs[i], workspace=ws)
    for rep in range(4):
        nq_, nk, nv = fresh()
        for i in range(L):
            qs[i].copy_(nq_[i])
            ks[i].copy_(nk[i])
            vs[i].copy_(nv[i])
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        want = [binding.deft_tree_attn_decode(plan, qs[i], ks[i], vs[i]) for i in range(L)]
        torch.cuda.synchronize()
        for i in range(L):
            assert torch.equal(got[i], want[i]), (rep, i)
    ref = reference(t, qs[0].cpu(), ks[0].cpu(), vs[0].cpu())
    check(got[0].float().cpu().numpy().astype(np.float64), ref, strict=False)


def test_randomised_sweep_of_shapes_strategies_and_storage():
    """120 random trees; head counts, head dimension, chunk size, partitioning strategy and storage form
    (contiguous / paged) drawn independently for each, a quarter of them with long nodes and wide groups."""
    rng = np.random.default_rng(2024)
    modes = list(binding.SPLIT_MODES)
    worst = worst_abs = worst_rel = 0.0
    n_short = 0
    for it in range(120):
        Hkv = int(rng.choice([1, 2, 3, 4, 8]))
        G = int(rng.choice([1, 2, 4, 5, 8]))
        d = int(rng.choice([64, 128]))
        seed = int(rng.integers(1 << 30))
        big = rng.random() < 0.25
        t = wl.random_tree(seed, n_nodes=int(rng.integers(1, 40)), max_len=int(rng.integers(1, 2500 if big else 400)),
                           nq=int(rng.integers(1, 300 if big else 80)), Hq=Hkv * G, Hkv=Hkv, d=d,
                           n_roots=int(rng.integers(1, 4)), zero_len_prob=float(rng.choice([0, 0.1, 0.3])))
        Q, K, V = wl.make_qkv(t)
        chunk = int(rng.choice([32, 64, 96, 128, 256, 512, 1024, 4096]))
        mode = modes[int(rng.integers(len(modes)))]
        page = int(rng.choice([1, 4, 16, 64])) if rng.random() < 0.3 else 0
        case = f"case {it}: seed={seed} Hkv={Hkv} G={G} d={d} chunk={chunk} mode={mode} page={page} nodes={t.n_nodes} nq={t.nq}"
        ref, abs_v = reference(t, Q, K, V), reference_abs_v(t, Q, K, V)
        if page:
            pp, pg, npool, row_of = wl.to_paged(t, page, seed=seed)
            kp = wl.scatter_to_pool(K, row_of, npool * page, 1).cuda()
            vp = wl.scatter_to_pool(V, row_of, npool * page, 2).cuda()
            plan = binding.deft_plan_paged(pp, pg, page, npool, t.node_tok_len, t.node_parent, t.query_node, chunk,
                                           mode_flags(mode, G))
            got = binding.deft_tree_attn_decode(plan, Q.cuda(), kp, vp, out_dtype=torch.float32)
        else:
            plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, chunk,
                                     mode_flags(mode, G))
            got = binding.deft_tree_attn_decode(plan, Q.cuda(), K.cuda(), V.cuda(), out_dtype=torch.float32)
        torch.cuda.synchronize()
        got = got.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), case
        err, rel = errors(got, ref)
        assert (err <= ABS_TOL + REL_TOL * np.abs(ref)).all(), case
        assert rel.max() <= REL_TOL, case
        worst_abs = max(worst_abs, float((err / (ABS_TOL + REL_TOL * np.abs(ref))).max()))
        worst_rel = max(worst_rel, float(rel.max()))
        if all_paths_short(t):
            n_short += 1
            frac = err / (U_PRECISE * abs_v + 1e-5)
            worst = max(worst, float(frac.max()))
            assert frac.max() <= 1.0, case
    print(f"\n    120 cases: largest error as a fraction of 2e-3 + 1e-2|ref|: {worst_abs:.3f}; largest row-relative "
          f"error {worst_rel:.2e}; {n_short} trees with short paths only, largest error as a fraction of the "
          f"two-term bound: {worst:.3f}", flush=True)


def test_uploads_are_only_enqueued_and_may_outrun_the_stream():
    """Twenty plans are uploaded and used back to back without any synchronisation (more than the library's
    eight pinned staging slots, so slots are reused while earlier copies may still be queued), and every
    plan object is dropped as soon as its calls are enqueued; then one synchronisation, and every result is
    checked."""
    dev = torch.device("cuda:0")
    cases = []
    for seed in range(20):
        t = wl.random_tree(300 + seed, n_nodes=4 + seed % 9, max_len=200, nq=2 + seed % 11, Hq=8, Hkv=2, d=128)
        Q, K, V = wl.make_qkv(t)
        cases.append((t, Q, K, V, Q.to(dev), K.to(dev), V.to(dev)))
    # something long on the stream first, so that the uploads really queue up behind it
    big = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    for _ in range(4):
        big.add_(1)
    outs = []
    for (t, Q, K, V, q, k, v) in cases:
        plan = binding.deft_plan(t.node_tok_begin, t.node_tok_len, t.node_parent, t.query_node, t.ntok, 64)
        outs.append(binding.deft_tree_attn_decode(plan, q, k, v, out_dtype=torch.float32))
        del plan
    torch.cuda.synchronize()
    for (t, Q, K, V, *_), o in zip(cases, outs):
        check(o.cpu().numpy().astype(np.float64), reference(t, Q, K, V), strict=False,
              abs_v=reference_abs_v(t, Q, K, V), two_term=all_paths_short(t))
