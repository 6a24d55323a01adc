// Single-token decode attention over the paged KV arena.
//
// In the paper's PPO stage the actor generates its responses one token at a
// time (Section 2.1); each step reads every cached key and value of every
// sequence once, which makes the step a pure HBM stream.  The token range of a
// sequence is cut into chunks of a whole number of pages; one workgroup handles
// one (sequence, query head, chunk) item with an online softmax and writes an
// un-normalised partial (o, m, l); a second kernel merges the partials of a
// (sequence, head) with the usual log-sum-exp weights.  Chunks are defined on
// logical token positions only, so results do not depend on which physical
// pages a sequence happens to own.
//
// Data path of the split kernel (one wavefront works on one page at a time):
//   K block  [dim/8][16 slots][8 dims]: the wavefront's i-th 16-byte-per-lane
//            load hands lane l the dims 8*(4i + l/16) .. +8 of slot l%16.  Each
//            lane dots them with the matching slice of q (v_dot2), and two
//            cross-row adds finish the 16 scores of the page.
//   V block  [4 slot-quads][dim][4 slots]: the i-th load hands lane l two
//            adjacent dims for four consecutive slots; the four probabilities
//            are wave-uniform (v_readlane), so the lane owns two output dims
//            and needs no cross-lane reduction for P*V.
// All accumulation is fp32; probabilities stay fp32.
//
// Grouped-query heads (several query heads per KV head) turn both products into
// small matrix products, and those go to the matrix cores (attn_split_gqa_kernel):
// the same 1 KiB K load is the A operand of a 16x16x32 MFMA whose B operand is
// the group's q rows, giving S^T[slot][q head]; its result registers, after the
// softmax, are already laid out as the B operand of the 16x16x16 MFMAs that
// multiply V^T (A operand, straight from the V block's 8-byte granules) into
// O^T[dim][q head].  Probabilities are fed as a high and a low 16-bit part so
// that the product keeps fp32-level accuracy.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "common.h"
#include "device_ops.h"

namespace rlhf {
namespace {

constexpr int kPage = RLHF_PAGE_TOKENS;
constexpr int kSplitThreads = 256;
constexpr int kSplitWaves = 4;

struct SplitPlan {
    int pages_per_item;  // chunk length in pages
    int n_chunks;        // chunks that cover max_len
    int max_len;
};

// Chunk length: the longest of 64/32/16/8/4 pages that still yields a few
// thousand items (several per workgroup slot of the 256 compute units).  Every
// item pays a fixed start-up and merge cost of a few microseconds of its slot,
// so long chunks win as long as the slots stay evenly loaded; short caches fall
// back to 4 pages (one per wavefront).  Depends on the call's parameters only.
SplitPlan make_plan(const rlhf_attn_params &p)
{
    SplitPlan plan;
    const int cap = p.max_pages_per_seq * kPage;
    plan.max_len = (p.max_seq_len > 0 && p.max_seq_len < cap) ? p.max_seq_len : cap;
    const int group = p.n_q_heads / p.n_kv_heads;
    // one item covers one query head, or up to 16 heads of a group on the MFMA path
    const int64_t units = group == 1 ? (int64_t)p.batch * p.n_q_heads
                                     : (int64_t)p.batch * p.n_kv_heads * ((group + 15) / 16);
    const int max_pages = (plan.max_len + kPage - 1) / kPage;
    int ppi = 64;
    while (ppi > 4 && units * ((max_pages + ppi - 1) / ppi) < 3072)
        ppi >>= 1;
    plan.pages_per_item = ppi;
    plan.n_chunks = std::max(1, (max_pages + ppi - 1) / ppi);
    return plan;
}

template <int DT, int D>
__global__ __launch_bounds__(kSplitThreads) void attn_split_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, float *__restrict__ partials, int n_q_heads, int n_kv_heads,
    int mpps, int pages_per_item, int n_chunks, int max_len, float scale_log2)
{
    constexpr int NL = D / 32;  // 16-byte loads per lane for one K (or V) block
    __shared__ float s_m[kSplitWaves], s_l[kSplitWaves];
    __shared__ float s_o[kSplitWaves][D];

    const int chunk = blockIdx.x % n_chunks;
    const int unit = blockIdx.x / n_chunks;  // b * Hq + hq
    const int b = unit / n_q_heads;
    const int hq = unit - b * n_q_heads;
    const int hkv = hq / (n_q_heads / n_kv_heads);
    const int L = min(seq_lens[b], max_len);
    const int first_page = chunk * pages_per_item;
    if (first_page * kPage >= L)
        return;
    const int end_page = min(first_page + pages_per_item, (L + kPage - 1) / kPage);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slot = lane & 15;

    // q slices matching the K loads
    uint4 qr[NL];
    const uint16_t *qrow = q + (int64_t)unit * D;
#pragma unroll
    for (int i = 0; i < NL; ++i)
        qr[i] = load16(qrow + (4 * i + (lane >> 4)) * 8);

    const int32_t *table = page_table + (int64_t)b * mpps;
    const int64_t head_off = (int64_t)hkv * (kPage * D);
    const int64_t page_stride = (int64_t)n_kv_heads * (kPage * D);

    float m = -INFINITY, lsum = 0.f, acc0 = 0.f, acc1 = 0.f;

    auto load_page = [&](int page_index, uint4(&kd)[NL], uint4(&vd)[NL]) {
        const int64_t base = (int64_t)table[page_index] * page_stride + head_off + lane * 8;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            kd[i] = load16(k_arena + base + i * 512);
            vd[i] = load16(v_arena + base + i * 512);
        }
    };
    auto process_page = [&](int lp, const uint4(&kb)[NL], uint4(&vb)[NL]) {
        // scores of the page's 16 slots
        float part = 0.f;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            part = dot2<DT>(kb[i].x, qr[i].x, part);
            part = dot2<DT>(kb[i].y, qr[i].y, part);
            part = dot2<DT>(kb[i].z, qr[i].z, part);
            part = dot2<DT>(kb[i].w, qr[i].w, part);
        }
        part += __shfl_xor(part, 16);
        part += __shfl_xor(part, 32);
        const float y = (lp * kPage + slot < L) ? part * scale_log2 : -INFINITY;
        const float m_new = fmaxf(m, row16_max(y));  // finite: the page holds >= 1 live slot
        const float alpha = fast_exp2(m - m_new);
        const float p = fast_exp2(y - m_new);
        lsum = fmaf(lsum, alpha, p);
        acc0 *= alpha;
        acc1 *= alpha;
        m = m_new;
        // Slots past the sequence's end have probability 0, but whatever bits sit
        // there (never written, possibly NaN) must not reach 0 * v: blank them.
        // Only the last page of a sequence can be partial; the branch is uniform.
        const int live = L - lp * kPage;
        if (live < kPage) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int s0 = 4 * ((D == 128) ? i : 2 * i + (lane >> 5));
                const uint32_t m01 = (s0 + 0 < live ? 0x0000ffffu : 0u) | (s0 + 1 < live ? 0xffff0000u : 0u);
                const uint32_t m23 = (s0 + 2 < live ? 0x0000ffffu : 0u) | (s0 + 3 < live ? 0xffff0000u : 0u);
                vb[i].x &= m01;
                vb[i].y &= m23;
                vb[i].z &= m01;
                vb[i].w &= m23;
            }
        }
        // P * V
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            float pj[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (D == 128) {
                    pj[j] = lane_bcast(p, 4 * i + j);
                } else {
                    const float lo = lane_bcast(p, 8 * i + j);
                    const float hi = lane_bcast(p, 8 * i + 4 + j);
                    pj[j] = lane < 32 ? lo : hi;
                }
            }
            acc0 = fmaf(pj[0], unpack_lo<DT>(vb[i].x), acc0);
            acc0 = fmaf(pj[1], unpack_hi<DT>(vb[i].x), acc0);
            acc0 = fmaf(pj[2], unpack_lo<DT>(vb[i].y), acc0);
            acc0 = fmaf(pj[3], unpack_hi<DT>(vb[i].y), acc0);
            acc1 = fmaf(pj[0], unpack_lo<DT>(vb[i].z), acc1);
            acc1 = fmaf(pj[1], unpack_hi<DT>(vb[i].z), acc1);
            acc1 = fmaf(pj[2], unpack_lo<DT>(vb[i].w), acc1);
            acc1 = fmaf(pj[3], unpack_hi<DT>(vb[i].w), acc1);
        }
    };

    // The wavefront's pages, one ahead: the next page's loads are in flight while
    // the current one is consumed.  The last page is peeled off so that the
    // prefetch inside the loop is unconditional (a conditional one would force the
    // wait counters to cover both cases and serialise load and compute).
    int lp = first_page + wave;
    if (lp < end_page) {
        uint4 kb[NL], vb[NL];
        load_page(lp, kb, vb);
        for (int next = lp + kSplitWaves; next < end_page; next += kSplitWaves) {
            uint4 kn[NL], vn[NL];
            load_page(next, kn, vn);
            process_page(lp, kb, vb);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                kb[i] = kn[i];
                vb[i] = vn[i];
            }
            lp = next;
        }
        process_page(lp, kb, vb);
    }

    // wavefront result -> LDS
    const float l_wave = row16_sum(lsum);
    if constexpr (D == 64) {  // lanes l and l+32 hold the two halves of the slot quads
        acc0 += __shfl_xor(acc0, 32);
        acc1 += __shfl_xor(acc1, 32);
    }
    if (lane == 0) {
        s_m[wave] = m;
        s_l[wave] = l_wave;
    }
    if (lane < D / 2) {
        s_o[wave][2 * lane] = acc0;
        s_o[wave][2 * lane + 1] = acc1;
    }
    __syncthreads();
    if (threadIdx.x < D + 2) {
        float M = s_m[0];
#pragma unroll
        for (int w = 1; w < kSplitWaves; ++w)
            M = fmaxf(M, s_m[w]);
        float *dst = partials + ((int64_t)unit * n_chunks + chunk) * (D + 2);
        if (threadIdx.x < D) {
            float o = 0.f;
#pragma unroll
            for (int w = 0; w < kSplitWaves; ++w)
                o = fmaf(s_o[w][threadIdx.x], fast_exp2(s_m[w] - M), o);
            dst[threadIdx.x] = o;
        } else if (threadIdx.x == D) {
            dst[D] = M;
        } else {
            float l = 0.f;
#pragma unroll
            for (int w = 0; w < kSplitWaves; ++w)
                l = fmaf(s_l[w], fast_exp2(s_m[w] - M), l);
            dst[D + 1] = l;
        }
    }
}

// ---- grouped-query variant on the matrix cores --------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// D[16x16] += A[16x32] * B[32x16]; lane l supplies row (A) / column (B) l%16 and
// the 8 contraction entries of group l/16; it receives D[4*(l/16)+j][l%16].
template <int DT>
__device__ __forceinline__ f32x4_t mfma_k32(const uint4 &a, const uint4 &b, f32x4_t c)
{
    if constexpr (DT == RLHF_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// Same with 16 contraction entries, 4 per lane (entries 4*(l/16) .. +3).
template <int DT>
__device__ __forceinline__ f32x4_t mfma_k16(const uint2 &a, const uint2 &b, f32x4_t c)
{
    if constexpr (DT == RLHF_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a),
                                                         __builtin_bit_cast(s16x4_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, a),
                                                     __builtin_bit_cast(f16x4_t, b), c, 0, 0, 0);
}

// Splits two fp32 probabilities into packed 16-bit high parts and packed 16-bit
// remainders: p ~= hi + lo with relative error about 2^-16 (bf16) or better.
template <int DT>
__device__ __forceinline__ void split_pair(float p0, float p1, uint32_t &hi, uint32_t &lo)
{
    if constexpr (DT == RLHF_BF16) {
        const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
        hi = (u0 >> 16) | (u1 & 0xffff0000u);
        const float r0 = p0 - __uint_as_float(u0 & 0xffff0000u);  // exact
        const float r1 = p1 - __uint_as_float(u1 & 0xffff0000u);
        lo = (__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u);
    } else {
        const _Float16 h0 = (_Float16)p0, h1 = (_Float16)p1;
        const _Float16 l0 = (_Float16)(p0 - (float)h0), l1 = (_Float16)(p1 - (float)h1);
        hi = (uint32_t)__builtin_bit_cast(uint16_t, h0) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
        lo = (uint32_t)__builtin_bit_cast(uint16_t, l0) | ((uint32_t)__builtin_bit_cast(uint16_t, l1) << 16);
    }
}

// One workgroup per (sequence, KV head, block of <= 16 query heads of its group,
// chunk).  Lane l = (group g = l/16, column c = l%16): c is a slot when the lane
// feeds K, a query head when it feeds q or holds scores and outputs.
template <int DT, int D>
__global__ __launch_bounds__(kSplitThreads) void attn_split_gqa_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, float *__restrict__ partials, int n_q_heads, int n_kv_heads,
    int mpps, int pages_per_item, int n_chunks, int max_len, float scale_log2)
{
    constexpr int NL = D / 32;      // 16-byte loads per lane for one K (or V) block
    constexpr int LDS_ROW = D + 1;  // padded against bank conflicts
    __shared__ float s_m[kSplitWaves][16], s_l[kSplitWaves][16];
    __shared__ float s_o[kSplitWaves][16][LDS_ROW];

    const int group = n_q_heads / n_kv_heads;
    const int n_qb = (group + 15) >> 4;
    int idx = blockIdx.x;
    const int chunk = idx % n_chunks;
    idx /= n_chunks;
    const int qb = idx % n_qb;
    idx /= n_qb;
    const int hkv = idx % n_kv_heads;
    const int b = idx / n_kv_heads;
    const int L = min(seq_lens[b], max_len);
    const int first_page = chunk * pages_per_item;
    if (first_page * kPage >= L)
        return;
    const int end_page = min(first_page + pages_per_item, (L + kPage - 1) / kPage);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int head0 = hkv * group + qb * 16;     // first query head of this block
    const int n_heads = min(16, group - qb * 16);

    // q as the B operand: column c = head, contraction entries = dims 8*(4i+g) .. +8
    uint4 qr[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        qr[i] = make_uint4(0, 0, 0, 0);
        if (c < n_heads)
            qr[i] = load16(q + ((int64_t)b * n_q_heads + head0 + c) * D + (4 * i + g) * 8);
    }

    const int32_t *table = page_table + (int64_t)b * mpps;
    const int64_t head_off = (int64_t)hkv * (kPage * D);
    const int64_t page_stride = (int64_t)n_kv_heads * (kPage * D);
    const int k_lane = lane * 8;                 // K: granule 64*i + lane
    const int v_lane = (g * D + 2 * c) * 4;      // V: granules (quad g, dims 32*i + 2c, +1)

    float m = -INFINITY, lsum = 0.f;
    f32x4_t o[NL][2];
#pragma unroll
    for (int i = 0; i < NL; ++i)
        o[i][0] = o[i][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    auto load_page = [&](int page_index, uint4(&kd)[NL], uint4(&vd)[NL]) {
        const int64_t base = (int64_t)table[page_index] * page_stride + head_off;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            kd[i] = load16(k_arena + base + k_lane + i * 512);
            vd[i] = load16(v_arena + base + v_lane + i * 128);
        }
    };
    auto process_page = [&](int lp, const uint4(&kb)[NL], uint4(&vb)[NL]) {
        // S^T[slot 4g+j][head c]
        f32x4_t sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NL; ++i)
            sc = mfma_k32<DT>(kb[i], qr[i], sc);
        const int live = L - lp * kPage;
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            y[j] = (4 * g + j < live) ? sc[j] * scale_log2 : -INFINITY;
        float mx = fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));      // finite: slot 0 of the page is live
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2(m - m_new);
        float p[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            p[j] = fast_exp2(y[j] - m_new);
        lsum = fmaf(lsum, alpha, (p[0] + p[1]) + (p[2] + p[3]));
        m = m_new;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            o[i][0] *= alpha;
            o[i][1] *= alpha;
        }
        uint2 ph, pl;
        split_pair<DT>(p[0], p[1], ph.x, pl.x);
        split_pair<DT>(p[2], p[3], ph.y, pl.y);
        if (live < kPage) {  // blank never-written slots: 0 * NaN must not reach the MFMA
            const uint32_t m01 = (4 * g + 0 < live ? 0x0000ffffu : 0u) | (4 * g + 1 < live ? 0xffff0000u : 0u);
            const uint32_t m23 = (4 * g + 2 < live ? 0x0000ffffu : 0u) | (4 * g + 3 < live ? 0xffff0000u : 0u);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                vb[i].x &= m01;
                vb[i].y &= m23;
                vb[i].z &= m01;
                vb[i].w &= m23;
            }
        }
        // O^T[dim][head] += V^T[dim][slot] * P^T[slot][head]
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const uint2 v0 = make_uint2(vb[i].x, vb[i].y);  // dim 32i + 2c
            const uint2 v1 = make_uint2(vb[i].z, vb[i].w);  // dim 32i + 2c + 1
            o[i][0] = mfma_k16<DT>(v0, ph, o[i][0]);
            o[i][0] = mfma_k16<DT>(v0, pl, o[i][0]);
            o[i][1] = mfma_k16<DT>(v1, ph, o[i][1]);
            o[i][1] = mfma_k16<DT>(v1, pl, o[i][1]);
        }
    };

    // one page ahead, last page peeled (see attn_split_kernel)
    int lp = first_page + wave;
    if (lp < end_page) {
        uint4 kb[NL], vb[NL];
        load_page(lp, kb, vb);
        for (int next = lp + kSplitWaves; next < end_page; next += kSplitWaves) {
            uint4 kn[NL], vn[NL];
            load_page(next, kn, vn);
            process_page(lp, kb, vb);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                kb[i] = kn[i];
                vb[i] = vn[i];
            }
            lp = next;
        }
        process_page(lp, kb, vb);
    }

    // wavefront result -> LDS.  o[i][e][j] is row 4g+j of its tile, i.e. dim
    // 32i + 2(4g+j) + e, for head c.
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (g == 0) {
        s_m[wave][c] = m;
        s_l[wave][c] = lsum;
    }
#pragma unroll
    for (int i = 0; i < NL; ++i)
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                s_o[wave][c][32 * i + 2 * (4 * g + j) + e] = o[i][e][j];
    __syncthreads();
    for (int t = threadIdx.x; t < n_heads * (D + 2); t += kSplitThreads) {
        const int h = t / (D + 2), d = t - h * (D + 2);
        float M = s_m[0][h];
#pragma unroll
        for (int w = 1; w < kSplitWaves; ++w)
            M = fmaxf(M, s_m[w][h]);
        float r;
        if (d == D) {
            r = M;
        } else {
            r = 0.f;
#pragma unroll
            for (int w = 0; w < kSplitWaves; ++w)
                r = fmaf(d < D ? s_o[w][h][d] : s_l[w][h], fast_exp2(s_m[w][h] - M), r);
        }
        const int64_t unit = (int64_t)b * n_q_heads + head0 + h;
        partials[(unit * n_chunks + chunk) * (D + 2) + d] = r;
    }
}

// One wavefront per (sequence, query head): out = sum_c w_c o_c / sum_c w_c l_c,
// w_c = 2^(m_c - max m).
template <int ODT, int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(
    const float *__restrict__ partials, const int32_t *__restrict__ seq_lens, void *__restrict__ out,
    int n_units, int n_q_heads, int pages_per_item, int n_chunks, int max_len)
{
    const int lane = threadIdx.x & 63;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= n_units)
        return;
    const int b = unit / n_q_heads;
    const int L = min(seq_lens[b], max_len);
    const int chunk_tokens = pages_per_item * kPage;
    const int n = (L + chunk_tokens - 1) / chunk_tokens;
    const float *src = partials + (int64_t)unit * n_chunks * (D + 2);
    float M = -INFINITY;
    for (int c = 0; c < n; ++c)
        M = fmaxf(M, src[c * (D + 2) + D]);
    constexpr int PER = D / 64;
    float o[PER], l = 0.f;
#pragma unroll
    for (int k = 0; k < PER; ++k)
        o[k] = 0.f;
    for (int c = 0; c < n; ++c) {
        const float *pc = src + c * (D + 2);
        const float w = fast_exp2(pc[D] - M);
        l = fmaf(pc[D + 1], w, l);
#pragma unroll
        for (int k = 0; k < PER; ++k)
            o[k] = fmaf(pc[lane + 64 * k], w, o[k]);
    }
    const float inv = n > 0 ? 1.0f / l : 0.f;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const float r = n > 0 ? o[k] * inv : 0.f;
        const int64_t idx = (int64_t)unit * D + lane + 64 * k;
        if constexpr (ODT == RLHF_F32)
            ((float *)out)[idx] = r;
        else
            ((uint16_t *)out)[idx] = pack16<ODT>(r);
    }
}

int check_params(const rlhf_attn_params *p)
{
    if (!p)
        return fail(RLHF_ERR_INVALID, "NULL params");
    if (p->batch < 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->max_pages_per_seq <= 0 ||
        p->max_seq_len < 0)
        return fail(RLHF_ERR_INVALID, "bad attention shape");
    if (p->n_q_heads % p->n_kv_heads)
        return fail(RLHF_ERR_INVALID, "n_kv_heads %d does not divide n_q_heads %d", p->n_kv_heads, p->n_q_heads);
    if (p->page_tokens != kPage)
        return fail(RLHF_ERR_UNSUPPORTED, "page_tokens must be %d", kPage);
    if (p->head_dim != 64 && p->head_dim != 128)
        return fail(RLHF_ERR_UNSUPPORTED, "head_dim %d (64 or 128)", p->head_dim);
    if (p->qkv_dtype != RLHF_F16 && p->qkv_dtype != RLHF_BF16)
        return fail(RLHF_ERR_UNSUPPORTED, "qkv_dtype %d (f16 or bf16)", p->qkv_dtype);
    if (p->out_dtype != p->qkv_dtype && p->out_dtype != RLHF_F32)
        return fail(RLHF_ERR_UNSUPPORTED, "out_dtype must be the qkv dtype or f32");
    if ((int64_t)p->max_pages_per_seq * kPage > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "max_pages_per_seq too large");
    return RLHF_OK;
}

size_t workspace_bytes(const rlhf_attn_params &p, const SplitPlan &plan)
{
    return (size_t)p.batch * p.n_q_heads * plan.n_chunks * (p.head_dim + 2) * sizeof(float);
}

template <int DT, int D>
int launch(const rlhf_attn_params &p, const SplitPlan &plan, const void *q, const void *k_arena,
           const void *v_arena, const int32_t *page_table, const int32_t *seq_lens, void *out,
           float *partials, hipStream_t s)
{
    const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)D);
    const int64_t units = (int64_t)p.batch * p.n_q_heads;
    const int64_t items = units * plan.n_chunks;
    if (items > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "too many work items for one launch");
    const int group = p.n_q_heads / p.n_kv_heads;
    if (group == 1) {
        hipLaunchKernelGGL((attn_split_kernel<DT, D>), dim3((unsigned)items), dim3(kSplitThreads), 0, s,
                           (const uint16_t *)q, (const uint16_t *)k_arena, (const uint16_t *)v_arena,
                           page_table, seq_lens, partials, p.n_q_heads, p.n_kv_heads, p.max_pages_per_seq,
                           plan.pages_per_item, plan.n_chunks, plan.max_len, scale * kLog2e);
        RLHF_LAUNCH_CHECK("attn_split_kernel");
    } else {
        const int64_t gitems = (int64_t)p.batch * p.n_kv_heads * ((group + 15) / 16) * plan.n_chunks;
        hipLaunchKernelGGL((attn_split_gqa_kernel<DT, D>), dim3((unsigned)gitems), dim3(kSplitThreads), 0, s,
                           (const uint16_t *)q, (const uint16_t *)k_arena, (const uint16_t *)v_arena,
                           page_table, seq_lens, partials, p.n_q_heads, p.n_kv_heads, p.max_pages_per_seq,
                           plan.pages_per_item, plan.n_chunks, plan.max_len, scale * kLog2e);
        RLHF_LAUNCH_CHECK("attn_split_gqa_kernel");
    }
    const dim3 mgrid((unsigned)((units + 3) / 4));
    if (p.out_dtype == RLHF_F32)
        hipLaunchKernelGGL((attn_merge_kernel<RLHF_F32, D>), mgrid, dim3(256), 0, s, partials, seq_lens, out,
                           (int)units, p.n_q_heads, plan.pages_per_item, plan.n_chunks, plan.max_len);
    else
        hipLaunchKernelGGL((attn_merge_kernel<DT, D>), mgrid, dim3(256), 0, s, partials, seq_lens, out,
                           (int)units, p.n_q_heads, plan.pages_per_item, plan.n_chunks, plan.max_len);
    RLHF_LAUNCH_CHECK("attn_merge_kernel");
    return RLHF_OK;
}

}  // namespace
}  // namespace rlhf

using namespace rlhf;

extern "C" int rlhf_decode_attention_workspace_bytes(const rlhf_attn_params *params, size_t *out_bytes)
{
    if (!out_bytes)
        return fail(RLHF_ERR_INVALID, "NULL out_bytes");
    int rc = check_params(params);
    if (rc != RLHF_OK)
        return rc;
    *out_bytes = std::max<size_t>(16, workspace_bytes(*params, make_plan(*params)));
    return RLHF_OK;
}

extern "C" int rlhf_decode_attention(const rlhf_attn_params *params, const void *q, const void *k_arena,
                                     const void *v_arena, const int32_t *page_table, const int32_t *seq_lens,
                                     void *out, void *workspace, size_t workspace_bytes_given, void *stream)
{
    int rc = check_params(params);
    if (rc != RLHF_OK)
        return rc;
    const rlhf_attn_params &p = *params;
    if (p.batch == 0)
        return RLHF_OK;
    if (!q || !k_arena || !v_arena || !page_table || !seq_lens || !out || !workspace)
        return fail(RLHF_ERR_INVALID, "NULL pointer");
    if (((uintptr_t)q | (uintptr_t)k_arena | (uintptr_t)v_arena | (uintptr_t)out | (uintptr_t)workspace) % 16)
        return fail(RLHF_ERR_INVALID, "q, k_arena, v_arena, out and workspace must be 16-byte aligned");
    const SplitPlan plan = make_plan(p);
    const size_t need = workspace_bytes(p, plan);
    if (workspace_bytes_given < need)
        return fail(RLHF_ERR_INVALID, "workspace holds %zu bytes, %zu needed", workspace_bytes_given, need);
    hipStream_t s = (hipStream_t)stream;
    float *partials = (float *)workspace;
    if (p.qkv_dtype == RLHF_BF16) {
        if (p.head_dim == 128)
            return launch<RLHF_BF16, 128>(p, plan, q, k_arena, v_arena, page_table, seq_lens, out, partials, s);
        return launch<RLHF_BF16, 64>(p, plan, q, k_arena, v_arena, page_table, seq_lens, out, partials, s);
    }
    if (p.head_dim == 128)
        return launch<RLHF_F16, 128>(p, plan, q, k_arena, v_arena, page_table, seq_lens, out, partials, s);
    return launch<RLHF_F16, 64>(p, plan, q, k_arena, v_arena, page_table, seq_lens, out, partials, s);
}
