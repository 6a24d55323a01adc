// Causal attention of a block of new tokens per sequence over the paged KV
// arena ("prefill": a prompt, or a chunk of one, entering the cache before the
// one-token-per-step generation of Section 2.1 starts).
//
// Unlike a decode step this is a real contraction -- every key of a sequence
// meets hundreds of query rows -- so both products run on the matrix cores and
// the kernel is bound by them, not by HBM.
//
// Work split.  A workgroup owns one (sequence, KV head) and a block of
// consecutive new positions; its query rows are the pairs (position, head of
// the KV head's group), flattened position-major.  Each of the four wavefronts
// takes NT tiles of 16 such rows and walks the keys 0 .. (its last position) in
// steps of 32 keys = two pages.  Workgroups are numbered so that those of one
// (sequence, KV head) land on the same XCD one after the other (its K/V stays
// in that XCD's L2) and the long, late position blocks start first.
//
// Per step and tile, with lane l = (g = l/16, c = l%16):
//   S^T[key][row]   = K page (A operand, straight from the arena's block
//                     layout) x q rows (B operand, held in registers): lane
//                     (g, c) receives keys 4g..4g+3 of each page for row c;
//   softmax         against a per-row reference exponent that is only moved
//                     (and the accumulators rescaled) when some score exceeds
//                     it by more than 2^kLift -- after the first few steps of
//                     a row that never happens, so the common step has no
//                     cross-lane traffic and no rescaling;
//   O^T[dim][row]  += V^T (A operand: the lane's 4-slot granules of the two
//                     pages side by side form the 8 contraction entries)
//                     x P^T (B operand: exactly the registers S^T arrived in).
// Probabilities go in as a high and a low 16-bit part, so the result keeps
// fp32-level accuracy.  Row sums stay per lane until the end.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "common.h"
#include "device_ops.h"
#include "mfma_ops.h"

namespace rlhf {
namespace {

constexpr int kPage = RLHF_PAGE_TOKENS;
constexpr int kThreads = 256;
constexpr int kWgWaves = 4;
constexpr int kTiles = 4;                          // 16-row tiles per wavefront
constexpr int kRowsPerWg = kWgWaves * kTiles * 16; // (position, head) rows per workgroup
constexpr int kXcds = 8;
constexpr float kLift = 8.0f;  // log2 units a score may exceed the reference before it is moved

__device__ __forceinline__ uint4 load_cached(const uint16_t *p)
{
    return *reinterpret_cast<const uint4 *>(p);
}

template <int DT, int ODT, int D, int NT>
__global__ __launch_bounds__(kThreads) void prefill_attn_kernel(
    const uint16_t *__restrict__ q, const int32_t *__restrict__ cu_q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, void *__restrict__ out, int batch, int n_q_heads, int n_kv_heads,
    int mpps, int max_len, int n_blocks, int pos_per_wg, float scale_log2)
{
    constexpr int NL = D / 32;
    // workgroup -> (unit, position block): units round-robin over the XCDs, the
    // blocks of a unit consecutive on its XCD, last block first
    const int xcd = blockIdx.x % kXcds, seq_no = blockIdx.x / kXcds;
    const int unit = (seq_no / n_blocks) * kXcds + xcd;
    const int pb = n_blocks - 1 - seq_no % n_blocks;
    if (unit >= batch * n_kv_heads)
        return;
    const int b = unit / n_kv_heads, hkv = unit - b * n_kv_heads;
    const int group = n_q_heads / n_kv_heads;
    const int q0 = cu_q[b], n_b = cu_q[b + 1] - q0;
    const int L = min(seq_lens[b], max_len);
    const int i0 = pb * pos_per_wg;
    if (i0 >= n_b || n_b > L)
        return;
    const int first = L - n_b;  // position of the sequence's first query row
    const int rows_wg = pos_per_wg * group;

    const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r_first = wv * NT * 16;
    if (r_first >= rows_wg || i0 + r_first / group >= n_b)
        return;  // nothing for this wavefront (no barriers below)
    const int r_last = min(r_first + NT * 16, rows_wg) - 1;
    const int p_min = first + i0 + r_first / group;
    const int p_max = first + min(n_b - 1, i0 + r_last / group);
    const int n_steps = p_max / 32 + 1;
    const int n_pages = (L + kPage - 1) / kPage;

    // this lane's row of each tile
    int pos[NT];
    bool valid[NT];
    int64_t row_off[NT];  // element offset of the row in q / out
    uint4 qr[NT][NL];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int r_raw = r_first + t * 16 + c;
        const int r = min(r_raw, rows_wg - 1);
        const int il = r / group, hg = r - il * group;
        const int i = min(i0 + il, n_b - 1);
        valid[t] = r_raw < rows_wg && i0 + il < n_b;
        pos[t] = first + i;
        row_off[t] = ((int64_t)(q0 + i) * n_q_heads + hkv * group + hg) * D;
#pragma unroll
        for (int k = 0; k < NL; ++k)
            qr[t][k] = load_cached(q + row_off[t] + (4 * k + g) * 8);
    }

    const int64_t page_stride = (int64_t)n_kv_heads * (kPage * D);
    const int64_t head_off = (int64_t)hkv * (kPage * D);
    const int k_lane = lane * 8;             // K: granule 64*k + lane
    const int v_lane = (g * D + 2 * c) * 4;  // V: granules (quad g, dims 32*k + 2c, +1)
    const int32_t *table = page_table + (int64_t)b * mpps;
    auto load_step = [&](int s, uint4(&ka)[NL], uint4(&kb)[NL], uint4(&va)[NL], uint4(&vb)[NL]) {
        // the second page of the last step may not exist: re-read the last real
        // page instead; its keys lie beyond every position and are masked
        const int pa = table[min(2 * s, n_pages - 1)], pbb = table[min(2 * s + 1, n_pages - 1)];
        const int64_t base_a = (int64_t)pa * page_stride + head_off;
        const int64_t base_b = (int64_t)pbb * page_stride + head_off;
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            ka[k] = load_cached(k_arena + base_a + k_lane + k * 512);
            kb[k] = load_cached(k_arena + base_b + k_lane + k * 512);
            va[k] = load_cached(v_arena + base_a + v_lane + k * 128);
            vb[k] = load_cached(v_arena + base_b + v_lane + k * 128);
        }
    };

    float m_ref[NT], l_part[NT];
    f32x4_t o[NT][NL][2];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        m_ref[t] = -INFINITY;
        l_part[t] = 0.f;
#pragma unroll
        for (int k = 0; k < NL; ++k)
            o[t][k][0] = o[t][k][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    auto process_step = [&](int s, const uint4(&ka)[NL], const uint4(&kb)[NL], const uint4(&va)[NL],
                            const uint4(&vb)[NL]) {
        const int key0 = 32 * s;
        // Keys at or beyond L were never written (or belong to the stand-in page):
        // their probability is 0 but their bits may be NaN, so blank V there.
        uint32_t a01 = ~0u, a23 = ~0u, b01 = ~0u, b23 = ~0u;
        if (key0 + 32 > L) {
            const int ja = key0 + 4 * g, jb = ja + 16;
            a01 = (ja + 0 < L ? 0x0000ffffu : 0u) | (ja + 1 < L ? 0xffff0000u : 0u);
            a23 = (ja + 2 < L ? 0x0000ffffu : 0u) | (ja + 3 < L ? 0xffff0000u : 0u);
            b01 = (jb + 0 < L ? 0x0000ffffu : 0u) | (jb + 1 < L ? 0xffff0000u : 0u);
            b23 = (jb + 2 < L ? 0x0000ffffu : 0u) | (jb + 3 < L ? 0xffff0000u : 0u);
        }
        // V^T operands: the lane's 4-key granules of page a and page b side by side
        uint4 v0[NL], v1[NL];
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            v0[k] = make_uint4(va[k].x & a01, va[k].y & a23, vb[k].x & b01, vb[k].y & b23);  // dim 32k + 2c
            v1[k] = make_uint4(va[k].z & a01, va[k].w & a23, vb[k].z & b01, vb[k].w & b23);  // dim 32k + 2c + 1
        }
        const bool diagonal = key0 + 31 > p_min;  // some key of the step is hidden from some row
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            // S^T: keys 4g+j of page a (sa) and of page b (sb) for row c
            f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                sa = mfma_k32<DT>(ka[k], qr[t][k], sa);
                sb = mfma_k32<DT>(kb[k], qr[t][k], sb);
            }
            float y[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                y[j] = sa[j] * scale_log2;
                y[4 + j] = sb[j] * scale_log2;
            }
            if (diagonal) {
                const int lim = pos[t] - key0 - 4 * g;  // key offset j is visible iff j <= lim
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    y[j] = j <= lim ? y[j] : -INFINITY;
                    y[4 + j] = 16 + j <= lim ? y[4 + j] : -INFINITY;
                }
            }
            const float top = fmaxf(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])),
                                    fmaxf(fmaxf(y[4], y[5]), fmaxf(y[6], y[7])));
            if (__any(top > m_ref[t] + kLift)) {
                // move the reference of every row of the tile to its running maximum
                float cm = fmaxf(top, __shfl_xor(top, 16));
                cm = fmaxf(cm, __shfl_xor(cm, 32));
                const float m_new = fmaxf(m_ref[t], cm);
                const float alpha = fast_exp2(m_ref[t] - m_new);
                m_ref[t] = m_new;
                l_part[t] *= alpha;
#pragma unroll
                for (int k = 0; k < NL; ++k) {
                    o[t][k][0] *= alpha;
                    o[t][k][1] *= alpha;
                }
            }
            float p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                p[j] = fast_exp2(y[j] - m_ref[t]);
            l_part[t] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
            uint4 ph, pl;
            split_pair<DT>(p[0], p[1], ph.x, pl.x);
            split_pair<DT>(p[2], p[3], ph.y, pl.y);
            split_pair<DT>(p[4], p[5], ph.z, pl.z);
            split_pair<DT>(p[6], p[7], ph.w, pl.w);
            // O^T[dim][row] += V^T[dim][key] * P^T[key][row], 32 keys per product
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                o[t][k][0] = mfma_k32<DT>(v0[k], ph, o[t][k][0]);
                o[t][k][0] = mfma_k32<DT>(v0[k], pl, o[t][k][0]);
                o[t][k][1] = mfma_k32<DT>(v1[k], ph, o[t][k][1]);
                o[t][k][1] = mfma_k32<DT>(v1[k], pl, o[t][k][1]);
            }
        }
    };

    // one step ahead; the last step is peeled so that the prefetch in the loop is
    // unconditional
    uint4 ka[NL], kb[NL], va[NL], vb[NL];
    load_step(0, ka, kb, va, vb);
    for (int s = 0; s + 1 < n_steps; ++s) {
        uint4 kan[NL], kbn[NL], van[NL], vbn[NL];
        load_step(s + 1, kan, kbn, van, vbn);
        process_step(s, ka, kb, va, vb);
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            ka[k] = kan[k];
            kb[k] = kbn[k];
            va[k] = van[k];
            vb[k] = vbn[k];
        }
    }
    process_step(n_steps - 1, ka, kb, va, vb);

    // o[t][k][e][j] is dim 32k + 2(4g+j) + e of row c
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float l_all = l_part[t] + __shfl_xor(l_part[t], 16);
        l_all += __shfl_xor(l_all, 32);
        if (!valid[t])
            continue;
        const float inv = 1.0f / l_all;
#pragma unroll
        for (int k = 0; k < NL; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x0 = o[t][k][0][j] * inv, x1 = o[t][k][1][j] * inv;
                const int64_t idx = row_off[t] + 32 * k + 2 * (4 * g + j);
                if constexpr (ODT == RLHF_F32)
                    *(float2 *)((float *)out + idx) = make_float2(x0, x1);
                else
                    *(uint32_t *)((uint16_t *)out + idx) =
                        (uint32_t)pack16<ODT>(x0) | ((uint32_t)pack16<ODT>(x1) << 16);
            }
    }
}

template <int DT, int ODT, int D>
int launch(const rlhf_attn_params &p, const void *q, const int32_t *cu_q, int max_q_len, const void *k_arena,
           const void *v_arena, const int32_t *page_table, const int32_t *seq_lens, void *out, hipStream_t s)
{
    const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)D);
    const int group = p.n_q_heads / p.n_kv_heads;
    const int pos_per_wg = kRowsPerWg / group;
    const int n_blocks = (max_q_len + pos_per_wg - 1) / pos_per_wg;
    const int64_t units = (int64_t)p.batch * p.n_kv_heads;
    const int64_t grid = (units + kXcds - 1) / kXcds * kXcds * n_blocks;
    if (grid > 0x7fffffffLL)
        return fail(RLHF_ERR_UNSUPPORTED, "prefill launch of %lld workgroups: split the call", (long long)grid);
    const int cap = p.max_pages_per_seq * kPage;
    const int max_len = (p.max_seq_len > 0 && p.max_seq_len < cap) ? p.max_seq_len : cap;
    hipLaunchKernelGGL((prefill_attn_kernel<DT, ODT, D, kTiles>), dim3((unsigned)grid), dim3(kThreads), 0, s,
                       (const uint16_t *)q, cu_q, (const uint16_t *)k_arena, (const uint16_t *)v_arena,
                       page_table, seq_lens, out, p.batch, p.n_q_heads, p.n_kv_heads, p.max_pages_per_seq,
                       max_len, n_blocks, pos_per_wg, scale * kLog2e);
    RLHF_LAUNCH_CHECK("prefill_attn_kernel");
    return RLHF_OK;
}

template <int DT, int D>
int launch_out(const rlhf_attn_params &p, const void *q, const int32_t *cu_q, int max_q_len,
               const void *k_arena, const void *v_arena, const int32_t *page_table, const int32_t *seq_lens,
               void *out, hipStream_t s)
{
    if (p.out_dtype == RLHF_F32)
        return launch<DT, RLHF_F32, D>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, s);
    return launch<DT, DT, D>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, s);
}

}  // namespace
}  // namespace rlhf

using namespace rlhf;

extern "C" int rlhf_prefill_attention(const rlhf_attn_params *params, const void *q, const int32_t *cu_q,
                                      int32_t max_q_len, const void *k_arena, const void *v_arena,
                                      const int32_t *page_table, const int32_t *seq_lens, void *out,
                                      void *stream)
{
    if (!params)
        return fail(RLHF_ERR_INVALID, "NULL params");
    const rlhf_attn_params &p = *params;
    if (p.batch < 0 || p.n_q_heads <= 0 || p.n_kv_heads <= 0 || p.max_pages_per_seq <= 0 ||
        p.max_seq_len < 0 || max_q_len < 0)
        return fail(RLHF_ERR_INVALID, "bad attention shape");
    if (p.n_q_heads % p.n_kv_heads)
        return fail(RLHF_ERR_INVALID, "n_kv_heads %d does not divide n_q_heads %d", p.n_kv_heads, p.n_q_heads);
    if (p.page_tokens != kPage)
        return fail(RLHF_ERR_UNSUPPORTED, "page_tokens must be %d", kPage);
    if (p.head_dim != 64 && p.head_dim != 128)
        return fail(RLHF_ERR_UNSUPPORTED, "head_dim %d (64 or 128)", p.head_dim);
    if (p.qkv_dtype != RLHF_F16 && p.qkv_dtype != RLHF_BF16)
        return fail(RLHF_ERR_UNSUPPORTED, "qkv_dtype %d (f16 or bf16)", p.qkv_dtype);
    if (p.out_dtype != p.qkv_dtype && p.out_dtype != RLHF_F32)
        return fail(RLHF_ERR_UNSUPPORTED, "out_dtype must be the qkv dtype or f32");
    if (p.n_q_heads / p.n_kv_heads > kRowsPerWg)
        return fail(RLHF_ERR_UNSUPPORTED, "more than %d query heads per kv head", kRowsPerWg);
    if ((int64_t)p.max_pages_per_seq * kPage > 0x7fffffffLL ||
        (int64_t)p.batch * p.max_pages_per_seq > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "page table too large");
    if (p.batch == 0 || max_q_len == 0)
        return RLHF_OK;
    if (!q || !cu_q || !k_arena || !v_arena || !page_table || !seq_lens || !out)
        return fail(RLHF_ERR_INVALID, "NULL pointer");
    if (((uintptr_t)q | (uintptr_t)k_arena | (uintptr_t)v_arena | (uintptr_t)out) % 16)
        return fail(RLHF_ERR_INVALID, "q, k_arena, v_arena and out must be 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (p.qkv_dtype == RLHF_BF16) {
        if (p.head_dim == 128)
            return launch_out<RLHF_BF16, 128>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens,
                                              out, s);
        return launch_out<RLHF_BF16, 64>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, s);
    }
    if (p.head_dim == 128)
        return launch_out<RLHF_F16, 128>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, s);
    return launch_out<RLHF_F16, 64>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, s);
}
