// Device side of libdeft: the Attention Calculation Phase of DeFT-Flatten (Algorithm 4) for gfx950.
//
// Stage 1 (deft_stage1): one wave per work item = (chunk, KV head, range of 16-row tiles).  The
// rows of a tile are (query of the chunk's group) x (query head reading this KV head).  The wave
// streams the chunk 32 tokens at a time straight from HBM into MFMA operand registers:
//
//   S^T[token, row] = K[token, :] . Q[row, :]      v_mfma_f32_16x16x32_bf16, A = K tile (a lane holds
//                                                   8 consecutive d of one token = one 128-bit load),
//                                                   B = Q (resident in registers for the whole chunk)
//   online softmax over tokens, per row             a row lives in the 4 lanes {n, n+16, n+32, n+48}
//   O^T[d, row]  += V^T[d, token] . P^T[token, row] A = V^T, built from 128-bit row loads by a 2x2
//                                                   16-bit interleave in registers (v_perm_b32),
//                                                   B = P^T, which is S^T's accumulator layout as is
//
// Each token row of one head (2*d bytes, contiguous) is fetched exactly once per work item and every
// byte of every 64-byte sector requested is used, so nothing is staged through LDS; LDS only holds the
// chunk's per-token table (physical row, query interval) expanded from the plan's segment table.
//
// Stage 2 (deft_stage2): one wave per (query, query head) merges that query's partial results with
// the log-sum-exp weights of eq. 1.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <string>

#include "deft_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) int32_t i32x4;

struct Stage1Args {
    const uint16_t *q, *k, *v;
    float *part_acc, *part_m, *part_l;
    const int32_t *chunk_seg_ptr, *seg_tok_begin, *seg_len, *seg_qlo, *seg_qhi;
    const int32_t *chunk_qlo, *chunk_qhi, *chunk_slot_base, *q_order;
    const int32_t *items;
    int32_t n_items, Hq, Hkv, G, chunk_size;
    float c;  // scale * log2(e): probabilities are 2^((s - m) * c)
};

struct Stage2Args {
    const float *part_acc, *part_m, *part_l;
    const int32_t *q_order, *q_part_ptr, *q_part_slot;
    void *out;
    int32_t nq, Hq, out_f32;
    float c;
};

__device__ __forceinline__ u32x4 load16(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }

__device__ __forceinline__ float wave_row_max(float x) {
    // rows live in lanes {n, n+16, n+32, n+48}
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}
__device__ __forceinline__ float wave_row_sum(float x) {
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
}

template <int D, int NT>
__global__ __launch_bounds__(64) void deft_stage1(Stage1Args a) {
    constexpr int KK = D / 32;   // k-steps of the Q.K^T contraction
    constexpr int DT = 8;        // P.V products per block (index c' below): a lane loads 8 d of V per token.
                                 // With D = 64 lanes n16 >= 8 repeat the loads of n16 - 8 and half of each
                                 // product is discarded; that shape only occurs in tiny, latency-bound cases.
    static_assert(D == 64 || D == 128, "head dimension");

    extern __shared__ int32_t s_tab[];
    int32_t *s_row = s_tab;
    int32_t *s_qlo = s_tab + a.chunk_size;
    int32_t *s_qhi = s_tab + 2 * a.chunk_size;

    const int lane = threadIdx.x;
    const int n16 = lane & 15;
    const int g = lane >> 4;
    const int item = blockIdx.x / a.Hkv;
    const int h = blockIdx.x - item * a.Hkv;
    const int chunk = a.items[2 * item];
    const int tile0 = a.items[2 * item + 1] & 0xffffff;
    const int ntiles = a.items[2 * item + 1] >> 24;
    const int seg0 = a.chunk_seg_ptr[chunk], seg1 = a.chunk_seg_ptr[chunk + 1];
    const int cqlo = a.chunk_qlo[chunk];
    const int R = (a.chunk_qhi[chunk] - cqlo) * a.G;

    // ---- per-token table of the chunk: physical row and the interval of plan positions that attend
    int clen = 0;
    for (int s = seg0; s < seg1; ++s) {
        const int b = a.seg_tok_begin[s], n = a.seg_len[s], lo = a.seg_qlo[s], hi = a.seg_qhi[s];
        for (int i = lane; i < n; i += 64) {
            s_row[clen + i] = b + i;
            s_qlo[clen + i] = lo;
            s_qhi[clen + i] = hi;
        }
        clen += n;
    }
    const int nblk = (clen + 31) >> 5;
    {
        const int pad_row = a.seg_tok_begin[seg0];  // a row that exists; its scores are masked out
        for (int i = clen + lane; i < nblk * 32; i += 64) {
            s_row[i] = pad_row;
            s_qlo[i] = 0;
            s_qhi[i] = 0;
        }
    }
    __syncthreads();

    // ---- rows of this wave, and Q as the B operand (resident for the whole chunk)
    int qpos[NT];
    bf16x8 qreg[NT][KK];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int r = 16 * (tile0 + t) + n16;
        const bool ok = (t < ntiles) && (r < R);
        const int pl = r / a.G, gh = r - pl * a.G;
        qpos[t] = ok ? cqlo + pl : -1;
        u32x4 z = {0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qreg[t][kk] = __builtin_bit_cast(bf16x8, z);
        if (ok) {
            const int j = a.q_order[cqlo + pl];
            const uint16_t *qp = a.q + ((size_t)j * a.Hq + (size_t)h * a.G + gh) * D + 8 * g;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qreg[t][kk] = __builtin_bit_cast(bf16x8, load16(qp + 32 * kk));
        }
    }

    float m_run[NT], l_run[NT];
    f32x4 oacc[NT][DT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        m_run[t] = -INFINITY;
        l_run[t] = 0.f;
#pragma unroll
        for (int c = 0; c < DT; ++c) oacc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const size_t row_stride = (size_t)a.Hkv * D;     // elements between consecutive tokens
    const uint16_t *kbase = a.k + (size_t)h * D + 8 * g;
    const uint16_t *vbase = a.v + (size_t)h * D + 8 * (D == 128 ? n16 : (n16 & 7));

    for (int blk = 0; blk < nblk; ++blk) {
        const int x0 = blk * 32;
        // K: token (16a + n16) of the block, d = 32kk + 8g .. +7
        bf16x8 kreg[2][KK];
#pragma unroll
        for (int aa = 0; aa < 2; ++aa) {
            const uint16_t *kp = kbase + (size_t)s_row[x0 + 16 * aa + n16] * row_stride;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kreg[aa][kk] = __builtin_bit_cast(bf16x8, load16(kp + 32 * kk));
        }
        // V: tokens (16a + 4g + i), d = 8*n16 .. +7; these are also the tokens of this lane's scores
        u32x4 vraw[8];
        i32x4 tqlo[2], tqhi[2];
#pragma unroll
        for (int aa = 0; aa < 2; ++aa) {
            const i32x4 rows = *reinterpret_cast<const i32x4 *>(&s_row[x0 + 16 * aa + 4 * g]);
            tqlo[aa] = *reinterpret_cast<const i32x4 *>(&s_qlo[x0 + 16 * aa + 4 * g]);
            tqhi[aa] = *reinterpret_cast<const i32x4 *>(&s_qhi[x0 + 16 * aa + 4 * g]);
#pragma unroll
            for (int i = 0; i < 4; ++i) vraw[4 * aa + i] = load16(vbase + (size_t)rows[i] * row_stride);
        }

        // S^T = K Q^T
        f32x4 sacc[2][NT];
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[aa][kk], qreg[t][kk], acc, 0, 0, 0);
                sacc[aa][t] = acc;
            }

        // V^T operand: 16-bit interleave of token pairs; vt[c'][p] = {V[tok 2p][8*n16 + c'], V[tok 2p+1][..]}
        u32x4 vt[8];
#pragma unroll
        for (int c2 = 0; c2 < 4; ++c2)
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t lo = vraw[2 * p][c2], hi = vraw[2 * p + 1][c2];
                vt[2 * c2][p] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                vt[2 * c2 + 1][p] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
            }

        // masked online softmax, one row tile at a time
        bf16x8 preg[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float mx = -INFINITY;
#pragma unroll
            for (int aa = 0; aa < 2; ++aa)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool on = (qpos[t] >= tqlo[aa][i]) && (qpos[t] < tqhi[aa][i]);
                    const float s = on ? sacc[aa][t][i] : -INFINITY;
                    sacc[aa][t][i] = s;
                    mx = fmaxf(mx, s);
                }
            mx = wave_row_max(mx);
            const float m_new = fmaxf(m_run[t], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f((m_run[t] - m_use) * a.c);
            m_run[t] = m_new;
            const float mc = m_use * a.c;
            float pv[8];
            float psum = 0.f;
#pragma unroll
            for (int aa = 0; aa < 2; ++aa)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float e = __builtin_amdgcn_exp2f(fmaf(sacc[aa][t][i], a.c, -mc));
                    pv[4 * aa + i] = e;
                    psum += e;
                }
            l_run[t] = l_run[t] * alpha + psum;
            u32x4 pk = {pack_bf16(pv[0], pv[1]), pack_bf16(pv[2], pv[3]), pack_bf16(pv[4], pv[5]),
                        pack_bf16(pv[6], pv[7])};
            preg[t] = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
            for (int c = 0; c < DT; ++c) oacc[t][c] *= alpha;
        }

        // O^T += V^T P^T
#pragma unroll
        for (int c = 0; c < DT; ++c)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                oacc[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[c]), preg[t],
                                                                      oacc[t][c], 0, 0, 0);
    }

    // ---- partial results: (m, l, un-normalised acc) per (slot, query head)
    const int slot_base = a.chunk_slot_base[chunk];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const float l_tot = wave_row_sum(l_run[t]);
        if (qpos[t] < 0) continue;
        const int r = 16 * (tile0 + t) + n16;
        const int pl = r / a.G, gh = r - pl * a.G;
        const size_t ro = (size_t)(slot_base + pl) * a.Hq + (size_t)h * a.G + gh;
        if (g == 0) {
            a.part_m[ro] = m_run[t];
            a.part_l[ro] = l_tot;
        }
        // this lane owns d in [32g, 32g+32) of its row: d = 32g + 8i + c'
        if (D == 128 || g < 2) {
            float *dst = a.part_acc + ro * D + 32 * g;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                f32x4 lo4 = {oacc[t][0][i], oacc[t][1][i], oacc[t][2][i], oacc[t][3][i]};
                f32x4 hi4 = {oacc[t][4][i], oacc[t][5][i], oacc[t][6][i], oacc[t][7][i]};
                *reinterpret_cast<f32x4 *>(dst + 8 * i) = lo4;
                *reinterpret_cast<f32x4 *>(dst + 8 * i + 4) = hi4;
            }
        }
    }
}

// Stage 2: tree-topology-aware global reduction (eq. 1 with the running maximum subtracted).
template <int D>
__global__ __launch_bounds__(64) void deft_stage2(Stage2Args a) {
    constexpr int E = D / 64;  // output elements per lane
    const int lane = threadIdx.x;
    const int p = blockIdx.x / a.Hq;
    const int qh = blockIdx.x - p * a.Hq;
    const int s0 = a.q_part_ptr[p], s1 = a.q_part_ptr[p + 1];

    float mx = -INFINITY;
    for (int i = s0 + lane; i < s1; i += 64) mx = fmaxf(mx, a.part_m[(size_t)a.q_part_slot[i] * a.Hq + qh]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));

    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    float lsum = 0.f;
    if (mx != -INFINITY) {
        for (int i = s0; i < s1; ++i) {
            const size_t ro = (size_t)a.q_part_slot[i] * a.Hq + qh;
            const float w = __builtin_amdgcn_exp2f((a.part_m[ro] - mx) * a.c);
            lsum += w * a.part_l[ro];
            const float *src = a.part_acc + ro * D + E * lane;
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] += w * src[e];
        }
    }
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    const size_t oo = ((size_t)a.q_order[p] * a.Hq + qh) * D + E * lane;
    if (a.out_f32) {
        float *o = reinterpret_cast<float *>(a.out) + oo;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = acc[e] * inv;
    } else {
        __bf16 *o = reinterpret_cast<__bf16 *>(a.out) + oo;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = (__bf16)(acc[e] * inv);
    }
}

thread_local std::string g_hip_error;

bool hip_ok(hipError_t e, const char *what) {
    if (e == hipSuccess) return true;
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return false;
}

template <int D, int NT>
bool launch_stage1(const Stage1Args &args, hipStream_t stream) {
    if (args.n_items == 0) return true;
    const size_t lds = 3 * (size_t)args.chunk_size * sizeof(int32_t);
    const unsigned grid = (unsigned)args.n_items * (unsigned)args.Hkv;
    hipLaunchKernelGGL((deft_stage1<D, NT>), dim3(grid), dim3(64), lds, stream, args);
    return hip_ok(hipGetLastError(), "deft_stage1 launch");
}

template <int D>
bool launch_stage1_lists(const deft::Schedule &S, Stage1Args a1, const uint8_t *image, hipStream_t stream) {
    for (const deft::ItemList &L : S.lists) {
        a1.items = reinterpret_cast<const int32_t *>(image + L.offset);
        a1.n_items = L.n_items;
        bool ok = true;
        switch (L.nt) {
            case 1: ok = launch_stage1<D, 1>(a1, stream); break;
            case 2: ok = launch_stage1<D, 2>(a1, stream); break;
            case 4: ok = launch_stage1<D, 4>(a1, stream); break;
            default: ok = false; g_hip_error = "unknown row-tile class"; break;
        }
        if (!ok) return false;
    }
    return true;
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
    for (const deft::ItemList &L : call.S->lists)
        if ((int64_t)L.n_items * Hkv > INT32_MAX) return DEFT_EINVAL;  // grid sizes are 32-bit
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
    a1.chunk_seg_ptr = at(S.off_chunk_seg_ptr);
    a1.seg_tok_begin = at(S.off_seg_tok_begin);
    a1.seg_len = at(S.off_seg_len);
    a1.seg_qlo = at(S.off_seg_qlo);
    a1.seg_qhi = at(S.off_seg_qhi);
    a1.chunk_qlo = at(S.off_chunk_qlo);
    a1.chunk_qhi = at(S.off_chunk_qhi);
    a1.chunk_slot_base = at(S.off_chunk_slot_base);
    a1.q_order = at(S.off_q_order);
    a1.Hq = Hq;
    a1.Hkv = Hkv;
    a1.G = Hq / Hkv;
    a1.chunk_size = plan->chunk_size;
    a1.c = call.c;
    const bool ok = d == 128 ? launch_stage1_lists<128>(S, a1, call.img, call.stream)
                             : launch_stage1_lists<64>(S, a1, call.img, call.stream);
    return ok ? DEFT_OK : DEFT_EHIP;
}

int run_stage2(const deft_plan_t *plan, const Call &call, void *o, int32_t Hq, int32_t d, uint32_t flags) {
    if (flags != DEFT_OUT_BF16 && flags != DEFT_OUT_F32) return DEFT_EINVAL;
    if (plan->nq == 0) return DEFT_OK;
    if (!o || (reinterpret_cast<uintptr_t>(o) & 3)) return DEFT_EINVAL;
    const deft::Schedule &S = *call.S;
    auto at = [&](size_t off) { return reinterpret_cast<const int32_t *>(call.img + off); };
    Stage2Args a2{};
    a2.part_acc = call.acc;
    a2.part_m = call.pm;
    a2.part_l = call.pl;
    a2.q_order = at(S.off_q_order);
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

}  // namespace

extern "C" const char *deft_last_hip_error(void) { return g_hip_error.c_str(); }

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
    if (plan->nq > 0 && (!o || (reinterpret_cast<uintptr_t>(o) & 3))) return DEFT_EINVAL;
    rc = run_stage1(plan, call, q, k, v, Hq, Hkv, d);
    if (rc != DEFT_OK) return rc;
    return run_stage2(plan, call, o, Hq, d, flags);
}
