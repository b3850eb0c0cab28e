// Device side of libdeft: the Attention Calculation Phase of DeFT-Flatten (Algorithm 4) for gfx950.
//
// Stage 1 (deft_stage1): one workgroup of four waves per task = (chunk, KV head, up to eight 16-row
// tiles).  The rows of a tile are (query of the chunk's group) x (query head reading this KV head).
// A wave streams 32 tokens at a time straight from HBM into MFMA operand registers:
//
//   S^T[token, row] = K[token, :] . Q[row, :]      v_mfma_f32_16x16x32_bf16, A = K tile (a lane holds
//                                                   8 consecutive d of one token = one 128-bit load),
//                                                   B = Q (resident in registers for the whole chunk)
//   online softmax over tokens, per row             a row lives in the 4 lanes {n, n+16, n+32, n+48}
//   O^T[d, row]  += V^T[d, token] . P^T[token, row] A = V^T, built from 128-bit row loads by a 2x2
//                                                   16-bit interleave in registers (v_perm_b32),
//                                                   B = P^T, which is S^T's accumulator layout as is
//
// Each token row of one head (2*d bytes, contiguous) is fetched from HBM exactly once per task and every
// byte of every 64-byte sector requested is used.  A narrow group (one row tile) splits the chunk's
// tokens over the four waves, each keeping two blocks of loads in flight in registers.  A wider group
// gives each wave its own row tile (two tiles for tasks of more than four); the waves that need the same
// block each fetch a share of it and pass the operand registers to the others through LDS.  The waves' partial results are merged in LDS before
// one (m, l, acc) triple per (chunk, row) is written.
//
// Stage 2 (deft_stage2): one wave per (query, query head) merges that query's partial results with
// the log-sum-exp weights of eq. 1.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>

#include "deft_internal.h"

// Partial-result workspace of deft_tree_attn_decode_static: device memory inside the code object, one copy
// per GPU at its own address, held until the process ends.  Host code never uses this name as an address;
// it asks the runtime for the device address once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[DEFT_STATIC_SCRATCH_BYTES];

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) int32_t i32x4;

struct Stage1Args {
    const uint16_t *q, *k, *v;
    float *part_acc, *part_m, *part_l;
    const int32_t *seg_tok_begin, *seg_len, *seg_qlo, *seg_qhi, *seg_off;
    const int32_t *q_order;
    const int32_t *items;  // deft::kItemInts int32 per work item, see deft_internal.h
    int32_t n_items, Hq, Hkv, G;
    int32_t table_len;  // entries of the LDS per-token table: longest multi-piece chunk, in whole blocks
    float c;  // scale * log2(e): probabilities are 2^((s - m) * c)
};

struct Stage2Args {
    const float *part_acc, *part_m, *part_l;
    const int32_t *q_head, *q_part_ptr, *q_part_slot;
    void *out;
    int32_t nq, Hq, out_f32;
    float c;
};

__device__ __forceinline__ u32x4 load16(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }
// K/V rows of a chunk whose group fits one task (one or two row tiles): no other workgroup will read them,
// so they are streamed without being kept in the caches (non-temporal); measured 2 % faster on the few-shot
// trees.  Chunks of wider groups are re-read by the other row groups and by the waves of the K pattern, and
// lose with it.
__device__ __forceinline__ u32x4 load16_once(const uint16_t *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}
template <bool ONCE>
__device__ __forceinline__ u32x4 load16_kv(const uint16_t *p) {
    return ONCE ? load16_once(p) : load16(p);
}

__device__ __forceinline__ float wave_row_max(float x) {
    // a row of a 16-row tile lives in lanes {n, n+16, n+32, n+48}
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
}

constexpr int kWaves = 4;              // waves per stage-1 workgroup
constexpr int kXbufBytes = 64 * 1024;  // LDS register-exchange area: 2 token parts x 2 stages x 16 KB
static_assert(4 * DEFT_MAX_CHUNK * sizeof(int32_t) <= kXbufBytes, "piece records are parked in the exchange area");

// What a wave needs to know about its chunk to address tokens.
struct ChunkCtx {
    const uint16_t *kbase, *vbase;  // K/V pointers already offset to this head and this lane's d slice
    const uint16_t *khead, *vhead;  // the same without the lane's slice (wave-uniform), and the slices in bytes
    uint32_t klane, vlane;
    size_t row_stride;              // elements between consecutive token rows
    const int32_t *s_row, *s_qlo, *s_qhi;  // LDS per-token table (only when !uniform), padded to whole blocks
    int clen;                       // tokens in the chunk
    int uniform;                    // the chunk is one piece of one node: rows are begin0 + x
    int begin0, qlo0, qhi0;
    int n16, g;
};

// One 32-token block as MFMA operands: K as the A operand of S^T = K Q^T (token 16a + n16, d = 32kk + 8g..+7),
// V as loaded, row-major (token 16a + 4g + i, d = 8*n16..+7).  The layout is the same in every wave, whatever
// row tile the wave works on, which is what lets waves exchange these registers through LDS unchanged.
template <int D>
struct KVRegs {
    bf16x8 k[2][D / 32];
    u32x4 v[8];
};

// physical row of chunk position x; positions past the chunk's end give a row that exists (their scores are masked)
__device__ __forceinline__ int tok_row(const ChunkCtx &c, int x) {
    return c.uniform ? c.begin0 + min(x, c.clen - 1) : c.s_row[x];
}

// Loads are issued unconditionally: a block past the end of the wave's work (valid == false) re-reads the
// chunk's first row instead (one cached row, no HBM traffic).  With the same sequence of memory
// instructions on every path the compiler can count exactly how many younger loads may stay in flight when
// an older block is consumed, which is what keeps the software pipeline full.
template <int D>
__device__ __forceinline__ void load_block(KVRegs<D> &r, const ChunkCtx &c, int x0, bool valid) {
    if (!valid) x0 = 0;
#pragma unroll
    for (int aa = 0; aa < 2; ++aa) {
        const int rowk = valid ? tok_row(c, x0 + 16 * aa + c.n16) : c.begin0;
        const uint16_t *kp = c.kbase + (size_t)rowk * c.row_stride;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) r.k[aa][kk] = __builtin_bit_cast(bf16x8, load16_once(kp + 32 * kk));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rowv = valid ? tok_row(c, x0 + 16 * aa + 4 * c.g + i) : c.begin0;
            r.v[4 * aa + i] = load16_once(c.vbase + (size_t)rowv * c.row_stride);
        }
    }
}

// Running softmax state of one row (held redundantly by the row's four lanes).
//   mc  : the reference subtracted inside the exponential, in units of the exponent: the weights are
//         2^(s * cs - mc).  The row's reference maximum in units of the scores is mc / cs.
//   thr : what an exponent s * cs - mc must exceed for the reference to be raised: kLazyLog2, or -inf while
//         the row has seen no visible token (mc is 0 then and stands for "no reference yet")
//   l   : sum over all tokens so far of the bf16-rounded weights, i.e. of exactly the numbers that enter the
//         P.V product.  It is accumulated by one more MFMA per block whose A operand is all ones (every row
//         of that product is the column sum of P^T), which costs the idle matrix pipe 16 cycles instead of 8
//         VALU adds and leaves the total in every lane of the row.
// The reference is only raised when some score exceeds it by more than kLazyLog2 / cs (probabilities may
// then reach 2^kLazyLog2, harmless in bf16 and fp32); otherwise a block costs no cross-lane traffic and
// no rescaling of the accumulators.  Any reference gives the same (m, l, acc) up to rounding, because the
// merge of eq. 1 only needs the three to be consistent.
struct RowState {
    float mc, thr;
    f32x4 l;  // four identical copies (rows 4g..4g+3 of the all-ones product)
    // reference maximum in units of the scores, as the partial result states it
    __device__ __forceinline__ float m(float inv_cs) const { return thr == -INFINITY ? -INFINITY : mc * inv_cs; }
};
constexpr float kLazyLog2 = 8.0f;

// Everything a wave keeps for one of its 16-row tiles: Q as the B operand of S^T = K Q^T (resident for the
// whole chunk), the plan position of this lane's row (-1: no such row), the softmax state and the O^T
// accumulators (oacc[c'][i] is d = 32g + 8i + c' of row n16).
template <int D>
struct TileState {
    bf16x8 q[D / 32];
    int qpos;
    RowState rs;
    f32x4 o[8];
};

// Online-softmax step of one wave over one 32-token block, for its NT row tiles.  The K and V operands are
// shared by the tiles, so the loads (or LDS reads) and the V interleave are paid once per block.
//
// PRECISE: every weight enters the P.V product and the denominator as the sum of two bf16 numbers, hi =
// bf16(p) and lo = bf16(p - hi), through a second set of MFMAs, so it carries a relative error of 2^-17
// instead of bf16's 2^-9.  The plan asks for it where some query of the group has a short path: there a
// handful of rounded weights does not average out and an output element would be off by up to
// 2^-7 * sum_t w_t |V_t|.  The matrix pipe has the room (a bandwidth-bound block keeps it busy for a sixth
// of its time).
//
// The pieces of a block's work, in the order compute_block strings them together.  The pipelined loop of the
// wide tasks (WidePipe) calls them separately so that one block's weights and the next block's scores can be
// issued side by side.

// S^T = K Q^T : sacc[t][a][i] is the score of token 16a + 4g + i against row n16 of tile t
template <int D, int NT>
__device__ __forceinline__ void qk_block(const bf16x8 (&k)[2][D / 32], const TileState<D> (&ts)[NT], f32x4 (&sacc)[NT][2]) {
    constexpr int KK = D / 32;
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[aa][kk], ts[t].q[kk], acc, 0, 0, 0);
            sacc[t][aa] = acc;
        }
}

// mask: a token is visible to plan position qpos iff qlo <= qpos < qhi of the node piece it belongs to.
// A full block of a single-piece chunk is visible to every row of the chunk's group: nothing to mask
// (rows past the group's end have Q = 0, finite scores, and are never written).
template <int D, int NT>
__device__ __forceinline__ void mask_block(const ChunkCtx &c, int x0, const TileState<D> (&ts)[NT], f32x4 (&sacc)[NT][2]) {
    if (!(c.uniform && x0 + 32 <= c.clen)) {
#pragma unroll
        for (int aa = 0; aa < 2; ++aa) {
            const int xv = x0 + 16 * aa + 4 * c.g;
            i32x4 qlo, qhi;
            if (c.uniform) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool in = xv + i < c.clen;
                    qlo[i] = in ? c.qlo0 : 0;
                    qhi[i] = in ? c.qhi0 : 0;
                }
            } else {
                qlo = *reinterpret_cast<const i32x4 *>(&c.s_qlo[xv]);
                qhi = *reinterpret_cast<const i32x4 *>(&c.s_qhi[xv]);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool on = (ts[t].qpos >= qlo[i]) && (ts[t].qpos < qhi[i]);
                    sacc[t][aa][i] = on ? sacc[t][aa][i] : -INFINITY;
                }
        }
    }
}

// scores -> exponents of the weights: e = s * cs - mc, in place
template <int D, int NT>
__device__ __forceinline__ void shift_block(const TileState<D> (&ts)[NT], f32x4 (&sacc)[NT][2], const float cs) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
#pragma unroll
            for (int i = 0; i < 4; ++i) sacc[t][aa][i] = fmaf(sacc[t][aa][i], cs, -ts[t].rs.mc);
}

// lazy reference, on the shifted scores of shift_block: it is raised (for every tile of the wave) only when
// some exponent exceeds kLazyLog2, i.e. some score exceeds the reference by more than kLazyLog2 / cs.  The
// exponents come out of an fma, so their maximum needs no canonicalisation and takes four instructions per tile.
template <int D, int NT>
__device__ __forceinline__ void raise_block(TileState<D> (&ts)[NT], f32x4 (&sacc)[NT][2]) {
    float mx[NT];
    bool need = false;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        mx[t] = fmaxf(fmaxf(fmaxf(sacc[t][0][0], sacc[t][0][1]), fmaxf(sacc[t][0][2], sacc[t][0][3])),
                      fmaxf(fmaxf(sacc[t][1][0], sacc[t][1][1]), fmaxf(sacc[t][1][2], sacc[t][1][3])));
        need = need || (mx[t] > ts[t].rs.thr);
    }
    if (__any(need)) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            // move the reference of every row up to its running maximum (never down), rescale what was
            // accumulated and move this block's exponents to the new reference
            RowState &st = ts[t].rs;
            const float r = wave_row_max(mx[t]);  // largest exponent of the row in this block, -inf if all masked
            const bool had = st.thr != -INFINITY;
            const float d = had ? fmaxf(r, 0.f) : (r == -INFINITY ? 0.f : r);
            const float alpha = had ? __builtin_amdgcn_exp2f(-d) : 0.f;  // nothing was accumulated before the first
            st.mc += d;
            st.thr = (had || r != -INFINITY) ? kLazyLog2 : -INFINITY;
            st.l *= alpha;
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) ts[t].o[cc] *= alpha;
#pragma unroll
            for (int aa = 0; aa < 2; ++aa)
#pragma unroll
                for (int i = 0; i < 4; ++i) sacc[t][aa][i] -= d;
        }
    }
}

// weights of the block, 2^(shifted score), as bf16 B operands (PRECISE: plus what the rounding to bf16 dropped, itself rounded to
// bf16; hi widens to fp32 by a 16-bit shift)
template <int D, int NT, bool PRECISE>
__device__ __forceinline__ void weights_block(const TileState<D> (&ts)[NT], const f32x4 (&sacc)[NT][2], const float cs,
                                              bf16x8 (&preg)[NT], bf16x8 (&plo)[NT]) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float pv[8];
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
#pragma unroll
            for (int i = 0; i < 4; ++i) pv[4 * aa + i] = __builtin_amdgcn_exp2f(sacc[t][aa][i]);
        const u32x4 pk = {pack_bf16(pv[0], pv[1]), pack_bf16(pv[2], pv[3]), pack_bf16(pv[4], pv[5]),
                          pack_bf16(pv[6], pv[7])};
        preg[t] = __builtin_bit_cast(bf16x8, pk);
        if (PRECISE) {
            u32x4 lk;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float h0 = __builtin_bit_cast(float, pk[j] << 16);
                const float h1 = __builtin_bit_cast(float, pk[j] & 0xffff0000u);
                lk[j] = pack_bf16(pv[2 * j] - h0, pv[2 * j + 1] - h1);
            }
            plo[t] = __builtin_bit_cast(bf16x8, lk);
        }
    }
}

// l += column sums of P^T;  O^T += V^T P^T
// READY: v[2*c2] and v[2*c2 + 1] already are the interleaved operands vt_lo and vt_hi described below (the
// waves that fetched V interleaved it before passing it on).
template <int D, int NT, bool PRECISE, bool READY = false>
__device__ __forceinline__ void pv_block(const u32x4 (&v)[8], const bf16x8 (&preg)[NT], const bf16x8 (&plo)[NT],
                                         TileState<D> (&ts)[NT]) {
    {
        const u32x4 one4 = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // eight bf16 1.0
        const bf16x8 ones = __builtin_bit_cast(bf16x8, one4);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            ts[t].rs.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, preg[t], ts[t].rs.l, 0, 0, 0);
            if (PRECISE) ts[t].rs.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, plo[t], ts[t].rs.l, 0, 0, 0);
        }
    }
    // The V^T operand of product c' = 2*c2 + {0,1} is a 16-bit interleave of token pairs:
    // vt[p] = {V[tok 2p][8*n16 + c'], V[tok 2p+1][8*n16 + c']}
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) {
        u32x4 vt_lo, vt_hi;
        if (READY) {
            vt_lo = v[2 * c2];
            vt_hi = v[2 * c2 + 1];
        } else {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t lo = v[2 * p][c2], hi = v[2 * p + 1][c2];
                vt_lo[p] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                vt_hi[p] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            ts[t].o[2 * c2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt_lo), preg[t],
                                                                       ts[t].o[2 * c2], 0, 0, 0);
            ts[t].o[2 * c2 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt_hi), preg[t],
                                                                           ts[t].o[2 * c2 + 1], 0, 0, 0);
            if (PRECISE) {
                ts[t].o[2 * c2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt_lo), plo[t],
                                                                           ts[t].o[2 * c2], 0, 0, 0);
                ts[t].o[2 * c2 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt_hi), plo[t],
                                                                               ts[t].o[2 * c2 + 1], 0, 0, 0);
            }
        }
    }
}

template <int D, int NT, bool PRECISE>
__device__ __forceinline__ void compute_block(const KVRegs<D> &r, const ChunkCtx &c, int x0, TileState<D> (&ts)[NT],
                                              const float cs, const float inv_cs) {
    f32x4 sacc[NT][2];
    qk_block<D, NT>(r.k, ts, sacc);
    mask_block<D, NT>(c, x0, ts, sacc);
    shift_block<D, NT>(ts, sacc, cs);
    raise_block<D, NT>(ts, sacc);
    bf16x8 preg[NT], plo[NT];
    weights_block<D, NT, PRECISE>(ts, sacc, cs, preg, plo);
    pv_block<D, NT, PRECISE>(r.v, preg, plo, ts);
}

// ---- token-split path (groups of one row tile): every wave streams its own blocks, two in flight ----
// wave w takes blocks w, w+4, w+8, ... (neighbouring waves read neighbouring rows at the same time)
template <int D>
struct SplitPipe {
    KVRegs<D> b0, b1;
    __device__ __forceinline__ void prime(const ChunkCtx &ctx, int wave, int nblk) {
        load_block<D>(b0, ctx, wave * 32, wave < nblk);
        load_block<D>(b1, ctx, (wave + kWaves) * 32, wave + kWaves < nblk);
    }
    template <bool PRECISE>
    __device__ __forceinline__ void run(const ChunkCtx &ctx, int wave, int nblk, TileState<D> (&ts)[1], float cs,
                                        float inv_cs) {
        for (int blk = wave; blk < nblk; blk += 2 * kWaves) {
            compute_block<D, 1, PRECISE>(b0, ctx, blk * 32, ts, cs, inv_cs);
            load_block<D>(b0, ctx, (blk + 2 * kWaves) * 32, blk + 2 * kWaves < nblk);
            if (blk + kWaves < nblk) compute_block<D, 1, PRECISE>(b1, ctx, (blk + kWaves) * 32, ts, cs, inv_cs);
            load_block<D>(b1, ctx, (blk + 3 * kWaves) * 32, blk + 3 * kWaves < nblk);
        }
    }
};

// ---- row-split path (groups of TR = 2 or 4 row tiles): the TR waves that work on the same blocks each
//      fetch 1/TR of a block from HBM and pass it to the others through LDS, so the block is read once.
// A block is 2*KK + 8 register images of 1 KB (K tile a, step kk -> image a*KK + kk; V token j -> image
// 2*KK + j).  With TR = 2 wave t fetches K tile t and V tokens 4t..4t+3; with TR = 4 waves 0 and 1 fetch the
// two K tiles and waves 2 and 3 four V tokens each.  Either way every 2*d-byte token row is read whole, by
// one wave, in back-to-back loads.
template <int D, int TR>
struct Share {
    static constexpr int KK = D / 32;
    static constexpr int NSLOT = 2 * KK + 8;
    static constexpr int NX = TR == 2 ? KK + 4 : (KK > 4 ? KK : 4);
    u32x4 x[NX];
};

template <int D, int TR>
__device__ __forceinline__ void share_issue(Share<D, TR> &s, const ChunkCtx &c, int t, int x0, bool valid) {
    constexpr int KK = D / 32;
    if (!valid) x0 = 0;
    if (TR == 2 || t < 2) {
        const int rowk = valid ? tok_row(c, x0 + 16 * t + c.n16) : c.begin0;
        const uint16_t *kp = c.kbase + (size_t)rowk * c.row_stride;
#pragma unroll
        for (int q = 0; q < KK; ++q) s.x[q] = load16_kv<TR == 2>(kp + 32 * q);
    }
    if (TR == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rowv = valid ? tok_row(c, x0 + 16 * t + 4 * c.g + q) : c.begin0;
            s.x[KK + q] = load16_once(c.vbase + (size_t)rowv * c.row_stride);
        }
    } else if (t >= 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rowv = valid ? tok_row(c, x0 + 16 * (t - 2) + 4 * c.g + q) : c.begin0;
            s.x[q] = load16(c.vbase + (size_t)rowv * c.row_stride);
        }
    }
}

template <int D, int TR, int NT, bool PRECISE>
__device__ __forceinline__ void share_step(Share<D, TR> &s, const ChunkCtx &c, u32x4 *xs, int t, int lane, int blk,
                                           int next_blk, int nblk, TileState<D> (&ts)[NT], float cs, float inv_cs) {
    constexpr int KK = D / 32;
    const bool live = blk < nblk;
    if (live) {
        if (TR == 2 || t < 2) {
#pragma unroll
            for (int q = 0; q < KK; ++q) xs[(t * KK + q) * 64 + lane] = s.x[q];
        }
        if (TR == 2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) xs[(2 * KK + 4 * t + q) * 64 + lane] = s.x[KK + q];
        } else if (t >= 2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) xs[(2 * KK + 4 * (t - 2) + q) * 64 + lane] = s.x[q];
        }
    }
    __syncthreads();
    share_issue<D, TR>(s, c, t, next_blk * 32, next_blk < nblk);
    if (live) {
        KVRegs<D> r;
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) r.k[aa][kk] = __builtin_bit_cast(bf16x8, xs[(aa * KK + kk) * 64 + lane]);
#pragma unroll
        for (int j = 0; j < 8; ++j) r.v[j] = xs[(2 * KK + j) * 64 + lane];
        compute_block<D, NT, PRECISE>(r, c, blk * 32, ts, cs, inv_cs);
    }
}

// Used for tasks of two row tiles (TR = 2, NT = 1: two waves per tile, the two pairs take alternate blocks);
// wider tasks go through WidePipe below.
template <int D, int TR, int NT>
struct SharedPipe {
    using S = Share<D, TR>;
    static constexpr int NP = kWaves / TR;  // token parts: part p takes blocks p, p+NP, ...
    static constexpr int DEPTH = 2;  // blocks whose shares a wave keeps in flight
    Share<D, TR> st[DEPTH];
    __device__ __forceinline__ void prime(const ChunkCtx &ctx, int wave, int nblk) {
        const int t = wave % TR, part = wave / TR;
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) share_issue<D, TR>(st[u], ctx, t, (part + u * NP) * 32, part + u * NP < nblk);
    }
    template <bool PRECISE>
    __device__ __forceinline__ void run(const ChunkCtx &ctx, u32x4 *xbuf, int wave, int lane, int nblk,
                                        TileState<D> (&ts)[NT], float cs, float inv_cs) {
        const int t = wave % TR, part = wave / TR;
        const int iters = (nblk + NP - 1) / NP;  // the same for every wave: barriers stay aligned
        u32x4 *xb = xbuf + (size_t)part * 2 * S::NSLOT * 64;
        // whole rounds of DEPTH steps; steps past the last block only keep the barrier and a dummy load
        for (int it0 = 0; it0 < iters; it0 += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int it = it0 + u;
                const int blk = part + it * NP;
                // LDS exchange stages alternate; stage (it & 1) was last read two steps ago, before the
                // barrier of the previous step
                share_step<D, TR, NT, PRECISE>(st[u], ctx, xb + (it & 1) * S::NSLOT * 64, t, lane, blk, blk + DEPTH * NP, nblk,
                                      ts, cs, inv_cs);
            }
        }
    }
};

// ---- row-split path for groups of 3 to 8 row tiles (TR = 4: the four waves share every block), pipelined
//      across blocks.  A wave's vector work on a block (32 exponentials and their scaling and packing, for two
//      tiles) takes longer than the block's MFMAs, and inside one basic block the matrix pipe and the vector
//      pipe run side by side; so the weights of block b-1 are formed while the scores of block b are
//      multiplied, and the P.V products of block b-1 follow.  Between two barriers a wave therefore holds the
//      scores and V of one block and K of the next.
//      UNIFORM: the chunk is one piece of one node, so its rows are consecutive.  A whole block's share is
//      then addressed as (wave-uniform pointer that moves on by one block per step) + (a byte offset per lane
//      that never changes): no vector arithmetic per load.  The last, partial block and the dummy loads past
//      the end go through the general addressing.
template <int D, int NT, bool UNIFORM>
struct WidePipe {
    static constexpr int KK = D / 32;
    using S = Share<D, 4>;
    // blocks whose shares a wave keeps in flight: with a tile per wave one measured faster than two (a 64-row
    // group over a 4000-token prefix: 19.5 us against 20.5 us); such a task is short and what is queued deeper
    // only waits behind the other workgroup's loads
    static constexpr int DEPTH = NT == 1 ? 1 : 2;
    S st[DEPTH];
    uint32_t lane_row, lane_col;  // UNIFORM: first row of this lane's loads inside a block, byte offset inside a row

    // UNIFORM: load q of the share is (wave-uniform pointer of the block) + (row of the lane, clamped to the
    // chunk's last row) * row bytes + the lane's column; a K loader reads four 64-byte columns of one row, a V
    // loader one column of four rows.  No branch on any path: blocks past the end repeat the last block, so the same four load instructions are
    // issued whatever happens and the compiler's s_waitcnt vmcnt counts stay exact.
    __device__ __forceinline__ void issue(S &sh, const ChunkCtx &c, int t, int blk, int nblk) {
        if (UNIFORM) {
            static_assert(KK == 4 || !UNIFORM, "a K loader issues four loads");
            const int blk_e = min(blk, nblk - 1);
            const uint32_t row_bytes = (uint32_t)c.row_stride * 2;
            const size_t first = ((size_t)c.begin0 + 32 * (size_t)blk_e) * row_bytes;
            const int lim = min(31, c.clen - 1 - 32 * blk_e);  // last row of the block that exists
            const bool kl = t < 2;
            const char *base = reinterpret_cast<const char *>(kl ? c.khead : c.vhead) + first;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // K loader: four 64-byte columns of row lane_row; V loader: rows lane_row .. lane_row + 3
                const int row = min((int)lane_row + (kl ? 0 : q), lim);
                const uint32_t off = (uint32_t)row * row_bytes + lane_col + (kl ? 64u * q : 0u);
                sh.x[q] = *reinterpret_cast<const u32x4 *>(base + off);
            }
        } else {
            share_issue<D, 4>(sh, c, t, blk * 32, blk < nblk);
        }
    }

    __device__ __forceinline__ void prime(const ChunkCtx &ctx, int wave, int nblk) {
        lane_row = wave < 2 ? 16 * wave + ctx.n16 : 16 * (wave - 2) + 4 * ctx.g;
        lane_col = wave < 2 ? ctx.klane : ctx.vlane;
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) issue(st[u], ctx, wave, u, nblk);
    }

    // pass this wave's share of a block to the others and fetch the share of a later block
    __device__ __forceinline__ void exchange(S &sh, const ChunkCtx &c, u32x4 *xs, int t, int lane, int next_blk, int nblk) {
        if (t < 2) {
#pragma unroll
            for (int q = 0; q < KK; ++q) xs[(t * KK + q) * 64 + lane] = sh.x[q];
        } else {
            // V: this wave holds tokens 16(t-2) + 4g + {0..3}, i.e. the token pairs p = 2(t-2) and 2(t-2) + 1 of
            // every lane's eight; it interleaves them once for all four waves (pv_block, READY) and writes its
            // half (8 bytes) of each of the eight operand images
            uint2 *xh = reinterpret_cast<uint2 *>(xs + 2 * KK * 64) + (t - 2);
#pragma unroll
            for (int c2 = 0; c2 < 4; ++c2) {
                const uint32_t lo0 = sh.x[0][c2], hi0 = sh.x[1][c2], lo1 = sh.x[2][c2], hi1 = sh.x[3][c2];
                xh[((2 * c2) * 64 + lane) * 2] = make_uint2(__builtin_amdgcn_perm(hi0, lo0, 0x05040100u),
                                                            __builtin_amdgcn_perm(hi1, lo1, 0x05040100u));
                xh[((2 * c2 + 1) * 64 + lane) * 2] = make_uint2(__builtin_amdgcn_perm(hi0, lo0, 0x07060302u),
                                                                __builtin_amdgcn_perm(hi1, lo1, 0x07060302u));
            }
        }
        __syncthreads();
        issue(sh, c, t, next_blk, nblk);
    }
    static __device__ __forceinline__ void read_k(const u32x4 *xs, int lane, bf16x8 (&k)[2][KK]) {
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) k[aa][kk] = __builtin_bit_cast(bf16x8, xs[(aa * KK + kk) * 64 + lane]);
    }
    static __device__ __forceinline__ void read_v(const u32x4 *xs, int lane, u32x4 (&v)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = xs[(2 * KK + j) * 64 + lane];
    }

    // one steady-state step: block `blk` arrives, block blk-1 (scores in sacc, V in vreg) is finished
    template <bool PRECISE>
    __device__ __forceinline__ void step(S &sh, const ChunkCtx &c, u32x4 *xs, int t, int lane, int blk, int nblk,
                                         TileState<D> (&ts)[NT], f32x4 (&sacc)[NT][2], u32x4 (&vreg)[8], float cs,
                                         float inv_cs) {
        exchange(sh, c, xs, t, lane, blk + DEPTH, nblk);
        bf16x8 k[2][KK];
        read_k(xs, lane, k);
        bf16x8 preg[NT], plo[NT];
        f32x4 snew[NT][2];
        weights_block<D, NT, PRECISE>(ts, sacc, cs, preg, plo);
        qk_block<D, NT>(k, ts, snew);
        pv_block<D, NT, PRECISE, true>(vreg, preg, plo, ts);
        read_v(xs, lane, vreg);
        mask_block<D, NT>(c, blk * 32, ts, snew);
        shift_block<D, NT>(ts, snew, cs);
        raise_block<D, NT>(ts, snew);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            sacc[tt][0] = snew[tt][0];
            sacc[tt][1] = snew[tt][1];
        }
    }

    template <bool PRECISE>
    __device__ __forceinline__ void run(const ChunkCtx &ctx, u32x4 *xbuf, int wave, int lane, int nblk,
                                        TileState<D> (&ts)[NT], float cs, float inv_cs) {
        const int t = wave;
        constexpr int STAGE = S::NSLOT * 64;  // u32x4 per LDS exchange stage; stage (blk & 1) holds block blk
        f32x4 sacc[NT][2];
        u32x4 vreg[8];
        {   // block 0: scores only
            exchange(st[0], ctx, xbuf, t, lane, DEPTH, nblk);
            bf16x8 k[2][KK];
            read_k(xbuf, lane, k);
            qk_block<D, NT>(k, ts, sacc);
            read_v(xbuf, lane, vreg);
            mask_block<D, NT>(ctx, 0, ts, sacc);
            shift_block<D, NT>(ts, sacc, cs);
            raise_block<D, NT>(ts, sacc);
        }
        // steady state, DEPTH steps per round so that the shares in flight are addressed statically.  Whole
        // rounds only inside the loop (a round that could stop half way would make the compiler assume, for the
        // waits of the next round, that the share it consumes is the youngest one in flight).
        int b0 = 1;
        for (; b0 + DEPTH <= nblk; b0 += DEPTH) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int blk = b0 + u;
                step<PRECISE>(st[(1 + u) % DEPTH], ctx, xbuf + (blk & 1) * STAGE, t, lane, blk, nblk, ts, sacc, vreg, cs, inv_cs);
            }
        }
        if (DEPTH == 2 && b0 < nblk)
            step<PRECISE>(st[1], ctx, xbuf + (b0 & 1) * STAGE, t, lane, b0, nblk, ts, sacc, vreg, cs, inv_cs);
        {   // last block: weights and products
            bf16x8 preg[NT], plo[NT];
            weights_block<D, NT, PRECISE>(ts, sacc, cs, preg, plo);
            pv_block<D, NT, PRECISE, true>(vreg, preg, plo, ts);
        }
    }
};

// Stage 1: one workgroup of four waves per task = (chunk, KV head, up to 128 rows of the chunk's group).
// The rows are (query of the group) x (query head reading this KV head), tiled 16 at a time.  A task of
// 1, 2 or 3-4 tiles splits its rows over TR = 1, 2 or 4 waves and its tokens over the 4 / TR parts that
// remain: wave w works on tile w % TR and token part w / TR.  A task of 5-8 tiles gives every wave two
// tiles.  The parts' partial results are merged in LDS, so one (m, l, acc) triple per (chunk, row)
// reaches the workspace.
//
// PRECISE selects two-term softmax weights (see compute_block).  The two variants are separate kernels so
// that the extra registers of the precise one do not weigh on the other; a plan's tasks are listed by
// variant and a call launches each non-empty list.
template <int D, bool PRECISE>
__global__ __launch_bounds__(64 * kWaves, 2) void deft_stage1(Stage1Args a) {
    constexpr int KK = D / 32;  // k-steps of the Q.K^T contraction
    // The P.V product runs as 8 MFMAs per block (a lane loads 8 d of V per token).  With D = 64 lanes
    // n16 >= 8 repeat the loads of n16 - 8 and half of each product is discarded; that shape only occurs
    // in tiny, latency-bound cases.
    static_assert(D == 64 || D == 128, "head dimension");
    constexpr int OP = D + 4;  // padded row pitch (floats) of the merge buffer

    extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
    u32x4 *xbuf = reinterpret_cast<u32x4 *>(s_raw);                     // register exchange, kXbufBytes
    float *mO = reinterpret_cast<float *>(s_raw);                       // merge buffer, aliases the exchange
    float *mM = mO + kWaves * 16 * OP;
    float *mL = mM + kWaves * 16;
    int32_t *s_row = reinterpret_cast<int32_t *>(s_raw + kXbufBytes);   // per-token table
    int32_t *s_qlo = s_row + a.table_len;
    int32_t *s_qhi = s_qlo + a.table_len;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the block loops on scalar branches
    const int n16 = lane & 15;
    const int g = lane >> 4;
    const int item = blockIdx.x / a.Hkv;
    // KV head of this workgroup.  Workgroups b and b + 256 land on the same compute unit (the dispatcher goes
    // round the 256 units), and with Hkv dividing 256 they would stream the same head: K and V rows whose
    // addresses agree in bits 7..12.  A unit whose streams all share those bits reads measurably slower (its
    // L1 keeps fewer lines in flight), so every further round of 256 workgroups is moved on by one head.
    // The shift depends on the task only, so a task still visits every head exactly once.
    const int h = (blockIdx.x - item * a.Hkv + ((item * a.Hkv) >> 8)) % a.Hkv;
    const int32_t *it = a.items + (size_t)item * deft::kItemInts;
    const int tile0 = it[deft::kItTile0], ntiles = it[deft::kItNTiles];
    const int seg0 = it[deft::kItSeg0], nseg = it[deft::kItNSeg];
    const int cqlo = it[deft::kItQlo];
    const int R = it[deft::kItWidth] * a.G;
    const int slot_base = it[deft::kItSlotBase];
    const int clen = it[deft::kItLen];
    const int TR = ntiles <= 1 ? 1 : (ntiles == 2 ? 2 : 4);  // waves that split the rows; 4 / TR token parts

    ChunkCtx ctx;
    ctx.row_stride = (size_t)a.Hkv * D;
    ctx.kbase = a.k + (size_t)h * D + 8 * g;
    ctx.vbase = a.v + (size_t)h * D + 8 * (D == 128 ? n16 : (n16 & 7));
    ctx.khead = a.k + (size_t)h * D;
    ctx.vhead = a.v + (size_t)h * D;
    ctx.klane = 16u * g;
    ctx.vlane = 16u * (D == 128 ? n16 : (n16 & 7));
    ctx.s_row = s_row;
    ctx.s_qlo = s_qlo;
    ctx.s_qhi = s_qhi;
    ctx.clen = clen;
    ctx.uniform = (nseg == 1);
    ctx.begin0 = it[deft::kItBegin0];
    ctx.qlo0 = it[deft::kItSegQlo0];
    ctx.qhi0 = it[deft::kItSegQhi0];
    ctx.n16 = n16;
    ctx.g = g;
    const int nblk = (clen + 31) >> 5;

    // ---- chunks made of several node pieces: per-token table (physical row, interval of plan
    //      positions that attend) expanded from the plan's segment table into LDS
    if (nseg > 1) {
        // the piece records are fetched with one thread per piece (one round trip for the whole chunk) and
        // parked in the exchange area, which is idle until the main loop; then one thread per token finds its
        // piece by bisection over the pieces' offsets
        int32_t *p_off = reinterpret_cast<int32_t *>(s_raw);
        int32_t *p_beg = p_off + DEFT_MAX_CHUNK;
        int32_t *p_lo = p_beg + DEFT_MAX_CHUNK;
        int32_t *p_hi = p_lo + DEFT_MAX_CHUNK;
        for (int s = tid; s < nseg; s += 64 * kWaves) {
            p_off[s] = a.seg_off[seg0 + s];
            p_beg[s] = a.seg_tok_begin[seg0 + s];
            p_lo[s] = a.seg_qlo[seg0 + s];
            p_hi[s] = a.seg_qhi[seg0 + s];
        }
        __syncthreads();
        for (int x = tid; x < nblk * 32; x += 64 * kWaves) {
            if (x < clen) {
                int lo = 0, hi = nseg - 1;  // largest s with p_off[s] <= x
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (p_off[mid] <= x) lo = mid; else hi = mid - 1;
                }
                s_row[x] = p_beg[lo] + (x - p_off[lo]);
                s_qlo[x] = p_lo[lo];
                s_qhi[x] = p_hi[lo];
            } else {  // last block's padding: a real row, masked
                s_row[x] = ctx.begin0;
                s_qlo[x] = 0;
                s_qhi[x] = 0;
            }
        }
        __syncthreads();
    }

    // ---- this wave's rows: tile (wave % TR) of the task and, for tasks of more than four tiles, tile
    //      (wave % TR) + 4 as well.  Q is the B operand, resident for the whole chunk.  The query indices are
    //      fetched first, the first K/V blocks are put in flight while they travel, then Q itself is fetched;
    //      one full wait before the main loop leaves nothing but the block pipeline outstanding inside it.
    const int NTW = ntiles > 4 ? 2 : 1;  // tiles per wave
    TileState<D> ts[2];
    int q_user[2], q_head[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int tile = wave % TR + 4 * u;
        const int r = 16 * (tile0 + tile) + n16;
        const bool ok = (u < NTW) && (tile < ntiles) && (r < R);
        const int pl = r / a.G;
        q_head[u] = r - pl * a.G;
        ts[u].qpos = ok ? cqlo + pl : -1;
        q_user[u] = 0;
        if (ok) q_user[u] = a.q_order[cqlo + pl];
        ts[u].rs = RowState{0.f, -INFINITY, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) ts[u].o[cc] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto load_q = [&](int ntw) {
        const u32x4 z = {0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u >= ntw) break;
            const uint16_t *qp = a.q + ((size_t)q_user[u] * a.Hq + (size_t)h * a.G + q_head[u]) * D + 8 * g;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                ts[u].q[kk] = __builtin_bit_cast(bf16x8, ts[u].qpos >= 0 ? load16(qp + 32 * kk) : z);
        }
        __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0)
    };
    const float inv_cs = 1.0f / a.c;  // turns a reference in exponent units back into score units
    TileState<D>(&ts1)[1] = reinterpret_cast<TileState<D>(&)[1]>(ts);  // the one-tile paths use ts[0] only

    if (TR == 1) {
        SplitPipe<D> pipe;
        pipe.prime(ctx, wave, nblk);
        load_q(1);
        pipe.template run<PRECISE>(ctx, wave, nblk, ts1, a.c, inv_cs);
    } else if (TR == 2) {
        SharedPipe<D, 2, 1> pipe;
        pipe.prime(ctx, wave, nblk);
        load_q(1);
        pipe.template run<PRECISE>(ctx, xbuf, wave, lane, nblk, ts1, a.c, inv_cs);
    } else if (NTW == 1 && ctx.uniform) {
        WidePipe<D, 1, D == 128> pipe;
        pipe.prime(ctx, wave, nblk);
        load_q(1);
        pipe.template run<PRECISE>(ctx, xbuf, wave, lane, nblk, ts1, a.c, inv_cs);
    } else if (NTW == 1) {
        WidePipe<D, 1, false> pipe;
        pipe.prime(ctx, wave, nblk);
        load_q(1);
        pipe.template run<PRECISE>(ctx, xbuf, wave, lane, nblk, ts1, a.c, inv_cs);
    } else if (ctx.uniform) {
        WidePipe<D, 2, D == 128> pipe;  // the fast addressing is written for four loads per K loader
        pipe.prime(ctx, wave, nblk);
        load_q(2);
        pipe.template run<PRECISE>(ctx, xbuf, wave, lane, nblk, ts, a.c, inv_cs);
    } else {
        WidePipe<D, 2, false> pipe;
        pipe.prime(ctx, wave, nblk);
        load_q(2);
        pipe.template run<PRECISE>(ctx, xbuf, wave, lane, nblk, ts, a.c, inv_cs);
    }

    // ---- merge the token parts in LDS and write one partial result per (chunk, row):
    //      m = reference maximum of the raw scores, l = sum of exp, acc = un-normalised weighted values.
    //      One round per tile of the wave; the exchange buffer is dead by now and the merge buffer takes its place.
    constexpr int EPL = D / 16;  // floats of a row per lane when 16 lanes share a row
    const int NP = kWaves / TR;  // parts to merge per row
    const int rr = lane >> 4, dc = lane & 15;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        if (u >= NTW) break;
        const float l_tot = ts[u].rs.l[0];
        __syncthreads();
        if (g == 0) {
            mM[wave * 16 + n16] = ts[u].rs.m(inv_cs);
            mL[wave * 16 + n16] = l_tot;
        }
        if (D == 128 || g < 2) {
            // this lane owns d in [32g, 32g+32) of row n16: d = 32g + 8i + c'
            float *dst = mO + (wave * 16 + n16) * OP + 32 * g;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const f32x4 lo4 = {ts[u].o[0][i], ts[u].o[1][i], ts[u].o[2][i], ts[u].o[3][i]};
                const f32x4 hi4 = {ts[u].o[4][i], ts[u].o[5][i], ts[u].o[6][i], ts[u].o[7][i]};
                *reinterpret_cast<f32x4 *>(dst + 8 * i) = lo4;
                *reinterpret_cast<f32x4 *>(dst + 8 * i + 4) = hi4;
            }
        }
        __syncthreads();

        for (int ps = 0; ps < TR; ++ps) {
            const int gr = 4 * TR * wave + 4 * ps + rr;  // row among the tiles of this round: 16 * (wave % TR) + n
            const int wt = gr >> 4, n = gr & 15;
            const int tile = wt + 4 * u;
            const int r = 16 * (tile0 + tile) + n;
            if (tile >= ntiles || r >= R) continue;
            float M = -INFINITY;
            for (int sp = 0; sp < NP; ++sp) M = fmaxf(M, mM[(wt + TR * sp) * 16 + n]);
            const float m_use = (M == -INFINITY) ? 0.f : M;
            float L = 0.f;
            float o[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] = 0.f;
            for (int sp = 0; sp < NP; ++sp) {
                const int src = wt + TR * sp;
                const float w = __builtin_amdgcn_exp2f((mM[src * 16 + n] - m_use) * a.c);
                L += w * mL[src * 16 + n];
                const float *row = mO + (src * 16 + n) * OP + EPL * dc;
#pragma unroll
                for (int e = 0; e < EPL; e += 4) {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(row + e);
                    o[e] += w * x[0];
                    o[e + 1] += w * x[1];
                    o[e + 2] += w * x[2];
                    o[e + 3] += w * x[3];
                }
            }
            const int pl = r / a.G, gh = r - pl * a.G;
            const size_t ro = (size_t)(slot_base + pl) * a.Hq + (size_t)h * a.G + gh;
            if (dc == 0) {
                a.part_m[ro] = M;
                a.part_l[ro] = L;
            }
            float *dst = a.part_acc + ro * D + EPL * dc;
#pragma unroll
            for (int e = 0; e < EPL; e += 4)
                *reinterpret_cast<f32x4 *>(dst + e) = f32x4{o[e], o[e + 1], o[e + 2], o[e + 3]};
        }
    }
}

// Stage 2: tree-topology-aware global reduction (eq. 1 with the largest maximum subtracted).
// One wave per (query, query head).  Weights are computed with lanes across the query's slots;
// the weighted rows are then summed with D/4 lanes per row (128-bit loads), several rows at a time.
template <int D>
__global__ __launch_bounds__(64) void deft_stage2(Stage2Args a) {
    constexpr int LPR = D / 4;     // lanes per partial row
    constexpr int RPI = 64 / LPR;  // rows per iteration
    const int lane = threadIdx.x;
    const int p = blockIdx.x / a.Hq;
    const int qh = blockIdx.x - p * a.Hq;
    // one 128-byte record per query: how many partials, where the result goes, the first slot ids
    const int hd = a.q_head[(size_t)p * deft::kQueryHeadInts + (lane & (deft::kQueryHeadInts - 1))];
    const int n = __shfl(hd, 0);
    const int q_user = __shfl(hd, 1);
    const int sub = lane / LPR, col = lane - sub * LPR;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f;
    constexpr int FAST = 8 * RPI < deft::kQueryInlineSlots ? 8 * RPI : deft::kQueryInlineSlots;  // rows held in registers
    if (n > 0 && n <= FAST) {
        // few partials (the usual case): the slot ids came with the record, so m, l and every row are
        // fetched in the next round trip and the weights are applied to rows that are already in registers
        const int slot_all = __shfl(hd, (lane < n ? lane : 0) + 2);
        const int slot = lane < n ? slot_all : 0;
        const size_t ro = (size_t)slot * a.Hq + qh;
        const float mj = lane < n ? a.part_m[ro] : -INFINITY;
        const float lj = lane < n ? a.part_l[ro] : 0.f;
        f32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int jj = u * RPI + sub;
            const int sj = __shfl(slot, jj);  // lanes >= n hold slot 0, which exists
            x[u] = *reinterpret_cast<const f32x4 *>(a.part_acc + ((size_t)sj * a.Hq + qh) * D + 4 * col);
        }
        float mx = mj;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        const float w = (lane < n && mx != -INFINITY) ? __builtin_amdgcn_exp2f((mj - mx) * a.c) : 0.f;
        lsum = w * lj;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float wu = __shfl(w, u * RPI + sub);
            acc += wu * x[u];
        }
    } else if (n > 0) {
        const int s0 = a.q_part_ptr[p];
        float mx = -INFINITY;
        for (int i = lane; i < n; i += 64) mx = fmaxf(mx, a.part_m[(size_t)a.q_part_slot[s0 + i] * a.Hq + qh]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        if (mx != -INFINITY) {
            for (int base = 0; base < n; base += 64) {
                const int i = base + lane;
                float w = 0.f;
                int slot = 0;
                if (i < n) {
                    slot = a.q_part_slot[s0 + i];
                    const size_t ro = (size_t)slot * a.Hq + qh;
                    w = __builtin_amdgcn_exp2f((a.part_m[ro] - mx) * a.c);
                    lsum += w * a.part_l[ro];
                }
                const int cnt = min(64, n - base);
                for (int j = 0; j < cnt; j += 4 * RPI) {
                    // four independent row loads per trip; rows past cnt get weight 0 and read slot 0, which exists
                    float wj[4];
                    f32x4 x[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int jj = j + u * RPI + sub;
                        const float ws = __shfl(w, jj & 63);
                        const int sj = __shfl(slot, jj & 63);
                        wj[u] = jj < cnt ? ws : 0.f;
                        const int sr = jj < cnt ? sj : 0;
                        x[u] = *reinterpret_cast<const f32x4 *>(a.part_acc + ((size_t)sr * a.Hq + qh) * D + 4 * col);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc += wj[u] * x[u];
                }
            }
        }
    }
#pragma unroll
    for (int o = 32; o >= LPR; o >>= 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += __shfl_xor(acc[e], o);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lsum += __shfl_xor(lsum, o);
    if (sub != 0) return;
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    const size_t oo = ((size_t)q_user * a.Hq + qh) * D + 4 * col;
    if (a.out_f32) {
        *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(a.out) + oo) = acc * inv;
    } else {
        typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
        u32x2 pk = {pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv)};
        *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(a.out) + oo) = pk;
    }
}

// Plain read of a buffer with 128-bit loads, every byte once, all compute units busy: the rate this
// reaches is the practical ceiling for a kernel whose job is to read HBM (Section 3.3's premise is that
// the KV read dominates).  Workgroup b leaves the xor of the words it read in sink[b], so that no load
// can be dropped and a caller can check that every word was read exactly once.
constexpr int kProbeGroups = DEFT_PROBE_SINK_BYTES / 4;

__global__ __launch_bounds__(256) void deft_read_probe(const u32x4 *__restrict__ p, size_t n16, uint32_t *sink) {
    __shared__ uint32_t part[4];
    size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i < n16; i += stride) acc ^= p[i];
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

thread_local std::string g_hip_error;

bool hip_ok(hipError_t e, const char *what) {
    if (e == hipSuccess) return true;
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return false;
}

// The kernels may use more than the default 64 KB of dynamic LDS: the limit of both variants is raised once
// per device, at the first call that launches either of them.
template <int D>
bool configure_stage1() {
    static std::atomic<uint64_t> configured;  // bit i set: done on device i (one flag per head dimension)
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return false;
    if (dev >= 0 && dev < 64 && ((configured.load(std::memory_order_acquire) >> dev) & 1)) return true;
    const int bytes = kXbufBytes + 3 * DEFT_MAX_CHUNK * (int)sizeof(int32_t);
    if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void *>(&deft_stage1<D, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, bytes), "deft_stage1 LDS size") ||
        !hip_ok(hipFuncSetAttribute(reinterpret_cast<const void *>(&deft_stage1<D, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, bytes), "deft_stage1 LDS size"))
        return false;
    if (dev >= 0 && dev < 64) configured.fetch_or(1ull << dev, std::memory_order_release);
    return true;
}

template <int D, bool PRECISE>
bool launch_stage1_variant(Stage1Args a1, const int32_t *items, int32_t n_items, hipStream_t stream) {
    if (n_items == 0) return true;
    a1.items = items;
    a1.n_items = n_items;
    const size_t lds = kXbufBytes + 3 * (size_t)a1.table_len * sizeof(int32_t);
    const unsigned grid = (unsigned)n_items * (unsigned)a1.Hkv;
    hipLaunchKernelGGL((deft_stage1<D, PRECISE>), dim3(grid), dim3(64 * kWaves), lds, stream, a1);
    return hip_ok(hipGetLastError(), "deft_stage1 launch");
}

// The task list holds the tasks with bf16 weights first, then those with two-term weights.
template <int D>
bool launch_stage1(const deft::Schedule &S, const Stage1Args &a1, const uint8_t *image, hipStream_t stream) {
    if (S.n_items == 0) return true;
    if (!configure_stage1<D>()) return false;
    const int32_t *items = reinterpret_cast<const int32_t *>(image + S.off_items);
    const int32_t n_fast = S.n_items - S.n_items_precise;
    return launch_stage1_variant<D, false>(a1, items, n_fast, stream) &&
           launch_stage1_variant<D, true>(a1, items + (size_t)n_fast * deft::kItemInts, S.n_items_precise, stream);
}

template <int D>
bool launch_stage2(const Stage2Args &a2, hipStream_t stream) {
    if (a2.nq == 0) return true;
    hipLaunchKernelGGL((deft_stage2<D>), dim3((unsigned)a2.nq * (unsigned)a2.Hq), dim3(64), 0, stream, a2);
    return hip_ok(hipGetLastError(), "deft_stage2 launch");
}

// Everything the two stages share: argument checks, the schedule, the workspace carve-up.
struct Call {
    const deft::Schedule *S = nullptr;
    const uint8_t *img = nullptr;
    float *acc = nullptr, *pm = nullptr, *pl = nullptr;
    float c = 0.f;
    hipStream_t stream = nullptr;
};

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int prepare(const deft_plan_t *plan, const void *dev_image, int32_t Hq, int32_t Hkv, int32_t d, float scale,
            void *workspace, size_t workspace_bytes, void *stream, Call &call) {
    if (!plan || !dev_image || !workspace) return DEFT_EINVAL;
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || (d != 64 && d != 128)) return DEFT_EINVAL;
    if (!aligned16(workspace) || !aligned16(dev_image)) return DEFT_EINVAL;
    call.S = deft::find_schedule(plan, Hq / Hkv);
    if (!call.S) return DEFT_ENOTREADY;
    if (workspace_bytes < deft_workspace_bytes(plan, Hq, Hkv, d)) return DEFT_EWORKSPACE;
    if ((int64_t)call.S->n_items * Hkv > INT32_MAX) return DEFT_EINVAL;  // grid sizes are 32-bit
    if ((int64_t)plan->nq * Hq > INT32_MAX) return DEFT_EINVAL;
    const size_t rows = (size_t)plan->n_slots() * (size_t)Hq;
    call.img = static_cast<const uint8_t *>(dev_image);
    call.acc = static_cast<float *>(workspace);
    call.pm = call.acc + rows * (size_t)d;
    call.pl = call.pm + rows;
    if (!(scale > 0.f)) scale = 1.0f / std::sqrt((float)d);
    call.c = scale * 1.4426950408889634f;  // log2(e)
    call.stream = reinterpret_cast<hipStream_t>(stream);
    return DEFT_OK;
}

int run_stage1(const deft_plan_t *plan, const Call &call, const void *q, const void *k, const void *v, int32_t Hq,
               int32_t Hkv, int32_t d) {
    if (plan->n_chunks() == 0) return DEFT_OK;
    if (!q || !k || !v || !aligned16(q) || !aligned16(k) || !aligned16(v)) return DEFT_EINVAL;
    const deft::Schedule &S = *call.S;
    auto at = [&](size_t off) { return reinterpret_cast<const int32_t *>(call.img + off); };
    Stage1Args a1{};
    a1.q = static_cast<const uint16_t *>(q);
    a1.k = static_cast<const uint16_t *>(k);
    a1.v = static_cast<const uint16_t *>(v);
    a1.part_acc = call.acc;
    a1.part_m = call.pm;
    a1.part_l = call.pl;
    a1.seg_tok_begin = at(S.off_seg_tok_begin);
    a1.seg_len = at(S.off_seg_len);
    a1.seg_qlo = at(S.off_seg_qlo);
    a1.seg_qhi = at(S.off_seg_qhi);
    a1.seg_off = at(S.off_seg_off);
    a1.q_order = at(S.off_q_order);
    a1.Hq = Hq;
    a1.Hkv = Hkv;
    a1.G = Hq / Hkv;
    a1.table_len = S.table_len;
    a1.c = call.c;
    const bool ok = d == 128 ? launch_stage1<128>(S, a1, call.img, call.stream)
                             : launch_stage1<64>(S, a1, call.img, call.stream);
    return ok ? DEFT_OK : DEFT_EHIP;
}

int run_stage2(const deft_plan_t *plan, const Call &call, void *o, int32_t Hq, int32_t d, uint32_t flags) {
    if (flags != DEFT_OUT_BF16 && flags != DEFT_OUT_F32) return DEFT_EINVAL;
    if (plan->nq == 0) return DEFT_OK;
    if (!o || !aligned16(o)) return DEFT_EINVAL;
    const deft::Schedule &S = *call.S;
    auto at = [&](size_t off) { return reinterpret_cast<const int32_t *>(call.img + off); };
    Stage2Args a2{};
    a2.part_acc = call.acc;
    a2.part_m = call.pm;
    a2.part_l = call.pl;
    a2.q_head = at(S.off_q_head);
    a2.q_part_ptr = at(S.off_q_part_ptr);
    a2.q_part_slot = at(S.off_q_part_slot);
    a2.out = o;
    a2.nq = plan->nq;
    a2.Hq = Hq;
    a2.out_f32 = (flags == DEFT_OUT_F32);
    a2.c = call.c;
    const bool ok = d == 128 ? launch_stage2<128>(a2, call.stream) : launch_stage2<64>(a2, call.stream);
    return ok ? DEFT_OK : DEFT_EHIP;
}

// Pinned host staging for plan images: a ring of slots per device, allocated at the first upload on that
// device and kept until the process ends.  An image is copied into the next slot and sent from there with
// an asynchronous copy, so deft_plan_upload neither waits for the stream nor depends on the plan staying
// alive.  A slot is reused only after the event recorded behind its last copy has completed.
constexpr int kStageSlots = 8;
constexpr size_t kStageSlotBytes = 256 * 1024;
struct Staging {
    std::mutex mu;
    uint8_t *base = nullptr;
    hipEvent_t done[kStageSlots] = {};
    bool used[kStageSlots] = {};
    int next = 0;
};
Staging g_staging[64];

// Returns 1 when the image went out through the ring, 0 when the caller has to take the plain path
// (image larger than a slot, device index out of range), -1 on a runtime error.
int upload_staged(void *dev_image, const uint8_t *src, size_t bytes, hipStream_t st) {
    int dev = 0;
    if (bytes > kStageSlotBytes) return 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return -1;
    if (dev < 0 || dev >= 64) return 0;
    Staging &g = g_staging[dev];
    std::lock_guard<std::mutex> lock(g.mu);
    if (!g.base) {
        void *p = nullptr;
        if (!hip_ok(hipHostMalloc(&p, kStageSlots * kStageSlotBytes, hipHostMallocDefault), "pinned staging")) return -1;
        for (int i = 0; i < kStageSlots; ++i) {
            if (!hip_ok(hipEventCreateWithFlags(&g.done[i], hipEventDisableTiming), "staging event")) {
                for (int j = 0; j < i; ++j) (void)hipEventDestroy(g.done[j]);
                (void)hipHostFree(p);
                return -1;
            }
        }
        g.base = static_cast<uint8_t *>(p);
    }
    const int i = g.next;
    g.next = (g.next + 1) % kStageSlots;
    if (g.used[i] && !hip_ok(hipEventSynchronize(g.done[i]), "staging slot")) return -1;
    uint8_t *slot = g.base + (size_t)i * kStageSlotBytes;
    std::memcpy(slot, src, bytes);
    if (!hip_ok(hipMemcpyAsync(dev_image, slot, bytes, hipMemcpyHostToDevice, st), "plan upload")) return -1;
    if (!hip_ok(hipEventRecord(g.done[i], st), "staging event record")) return -1;
    g.used[i] = true;
    return 1;
}

}  // namespace

extern "C" const char *deft_last_hip_error(void) { return g_hip_error.c_str(); }

extern "C" int deft_hbm_read_probe(const void *dev_buf, size_t bytes, void *dev_sink, void *stream) {
    if (!dev_buf || !dev_sink || bytes == 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(dev_buf) & 15)) return DEFT_EINVAL;
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(deft_read_probe, dim3(kProbeGroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(dev_buf), n16, static_cast<uint32_t *>(dev_sink));
    return hip_ok(hipGetLastError(), "deft_read_probe launch") ? DEFT_OK : DEFT_EHIP;
}

extern "C" int deft_plan_upload(deft_plan_t *plan, int32_t Hq, int32_t Hkv, void *dev_image, size_t bytes, void *stream) {
    if (!plan || !dev_image || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return DEFT_EINVAL;
    if (!aligned16(dev_image)) return DEFT_EINVAL;
    const deft::Schedule *S = nullptr;
    try {
        S = deft::get_schedule(plan, Hq / Hkv);
    } catch (...) {
        return DEFT_ENOMEM;
    }
    if (bytes < S->bytes) return DEFT_EWORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int staged = upload_staged(dev_image, S->host_image.data(), S->bytes, st);
    if (staged < 0) return DEFT_EHIP;
    if (staged > 0) return DEFT_OK;
    // an image larger than a staging slot goes from the plan's own (pageable) copy, and the call waits for it
    if (!hip_ok(hipMemcpyAsync(dev_image, S->host_image.data(), S->bytes, hipMemcpyHostToDevice, st), "plan upload"))
        return DEFT_EHIP;
    if (!hip_ok(hipStreamSynchronize(st), "plan upload sync")) return DEFT_EHIP;
    return DEFT_OK;
}

extern "C" int deft_stage1_partial_attention(const deft_plan_t *plan, const void *dev_image, const void *q,
                                             const void *k, const void *v, int32_t Hq, int32_t Hkv, int32_t d,
                                             float scale, void *workspace, size_t workspace_bytes, void *stream) {
    Call call;
    int rc = prepare(plan, dev_image, Hq, Hkv, d, scale, workspace, workspace_bytes, stream, call);
    if (rc != DEFT_OK) return rc;
    return run_stage1(plan, call, q, k, v, Hq, Hkv, d);
}

extern "C" int deft_stage2_global_reduction(const deft_plan_t *plan, const void *dev_image, void *o, int32_t Hq,
                                            int32_t Hkv, int32_t d, float scale, uint32_t flags, void *workspace,
                                            size_t workspace_bytes, void *stream) {
    Call call;
    int rc = prepare(plan, dev_image, Hq, Hkv, d, scale, workspace, workspace_bytes, stream, call);
    if (rc != DEFT_OK) return rc;
    return run_stage2(plan, call, o, Hq, d, flags);
}

extern "C" int deft_tree_attn_decode(const deft_plan_t *plan, const void *dev_image, const void *q, const void *k,
                                     const void *v, void *o, int32_t Hq, int32_t Hkv, int32_t d, float scale,
                                     uint32_t flags, void *workspace, size_t workspace_bytes, void *stream) {
    Call call;
    int rc = prepare(plan, dev_image, Hq, Hkv, d, scale, workspace, workspace_bytes, stream, call);
    if (rc != DEFT_OK) return rc;
    // check both stages' arguments before launching anything
    if (flags != DEFT_OUT_BF16 && flags != DEFT_OUT_F32) return DEFT_EINVAL;
    if (plan->nq > 0 && (!o || !aligned16(o))) return DEFT_EINVAL;
    rc = run_stage1(plan, call, q, k, v, Hq, Hkv, d);
    if (rc != DEFT_OK) return rc;
    return run_stage2(plan, call, o, Hq, d, flags);
}

namespace {

// Device address of `scratch` on the current device, looked up once per device.
std::mutex g_scratch_mu;
void *g_scratch_ptr[64] = {};

int static_scratch(void **out) {
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return DEFT_EHIP;
    if (dev < 0 || dev >= 64) return DEFT_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "address of the static workspace")) return DEFT_EHIP;
        if (!p || !aligned16(p)) return DEFT_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DEFT_OK;
}

}  // namespace

extern "C" int deft_tree_attn_decode_static(const deft_plan_t *plan, const void *dev_image, const void *q,
                                            const void *k, const void *v, void *o, int32_t Hq, int32_t Hkv, int32_t d,
                                            float scale, uint32_t flags, void *stream) {
    // size first: a plan whose partial results do not fit is refused before anything touches the device
    const size_t need = deft_workspace_bytes(plan, Hq, Hkv, d);
    if (need == 0) return DEFT_EINVAL;
    if (need > (size_t)DEFT_STATIC_SCRATCH_BYTES) return DEFT_EWORKSPACE;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != DEFT_OK) return rc;
    // every (slot, head) stage 2 reads was written by stage 1 of the same call, so nothing has to be cleared
    return deft_tree_attn_decode(plan, dev_image, q, k, v, o, Hq, Hkv, d, scale, flags, ws, DEFT_STATIC_SCRATCH_BYTES,
                                 stream);
}
