// Causal attention of a block of new tokens per sequence over the paged KV
// arena ("prefill": a prompt, or a chunk of one, entering the cache before the
// one-token-per-step generation of Section 2.1 starts).
//
// Unlike a decode step this is a real contraction -- every key of a sequence
// meets hundreds of query rows -- so both products run on the matrix cores and
// the kernel is bound by them, not by HBM.
//
// Work split.  A workgroup (8 wavefronts, two per SIMD) owns one (sequence, KV
// head) and a block of consecutive new positions; its 256 query rows are the
// pairs (position, head of the KV head's group), flattened position-major.
// Each wavefront keeps two tiles of 16 rows (q and the output accumulators) in
// registers.  The workgroup walks the keys 0 .. (its last position) in steps of
// 32 keys = two pages; the step's K and V blocks are copied once from the arena
// into LDS (double-buffered, the next step's global loads in flight during the
// current step) and every wavefront takes its matrix operands from there.
// Workgroups are numbered so that those of one (sequence, KV head) land on the
// same XCD one after the other (its K/V stays in that XCD's L2) and the long,
// late position blocks start first.
//
// Per step and tile, with lane l = (g = l/16, c = l%16):
//   S^T[key][row]   = K page (A operand: the arena's K block layout is the
//                     operand layout, lane l reads 16 bytes at granule 64k+l)
//                     x q rows (B operand, registers): lane (g, c) receives
//                     keys 4g..4g+3 of each page for row c;
//   softmax         against a per-row reference exponent that is only moved
//                     (and the accumulators rescaled) when some score exceeds
//                     it by more than 2^kLift -- after the first steps of a row
//                     that never happens, so the common step has no cross-lane
//                     traffic and no rescaling;
//   O^T[dim][row]  += V^T (A operand: in LDS the 4-key granules of the two
//                     pages sit side by side, 16 bytes = the lane's 8
//                     contraction entries) x P^T (B operand: exactly the
//                     registers S^T arrived in).
// Probabilities go in as a high and a low 16-bit part, so the result keeps
// fp32-level accuracy.  Row sums stay per lane until the end.  Steps that lie
// entirely below a wavefront's first position need no mask; only the last few
// ("edge") steps compare key and query positions and blank never-written keys.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <type_traits>

#include "common.h"
#include "device_ops.h"
#include "mfma_ops.h"

namespace rlhf {
namespace {

constexpr int kPage = RLHF_PAGE_TOKENS;
constexpr int kThreads = 512;
constexpr int kWgWaves = kThreads / 64;
constexpr int kTiles = 2;                          // 16-row tiles per wavefront
constexpr int kRowsPerWg = kWgWaves * kTiles * 16; // (position, head) rows per workgroup
constexpr int kStepKeys = 2 * kPage;
constexpr int kXcds = 8;
constexpr float kLift = 8.0f;  // log2 units a score may exceed the reference before it is moved

// Packs the upper 16 bits of two words: `first` into the low half.
__device__ __forceinline__ uint32_t pack_upper(uint32_t first, uint32_t second)
{
    return __builtin_amdgcn_perm(second, first, 0x07060302u);
}

// max(a, b) as median(a, b, +inf): one instruction, and no NaN-quieting move in
// front of it as the generic fmaxf needs for a matrix-core result (scores are
// finite or -inf here).
__device__ __forceinline__ float max2(float a, float b)
{
    return __builtin_amdgcn_fmed3f(a, b, INFINITY);
}

// fp32 pair -> packed high parts and packed remainders (see split_pair); the
// bf16 form truncates, which the remainder absorbs.
template <int DT>
__device__ __forceinline__ void split2(float p0, float p1, uint32_t &hi, uint32_t &lo)
{
    if constexpr (DT == RLHF_BF16) {
        const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
        hi = pack_upper(u0, u1);
        const float r0 = p0 - __uint_as_float(u0 & 0xffff0000u);  // exact
        const float r1 = p1 - __uint_as_float(u1 & 0xffff0000u);
        lo = pack_upper(__float_as_uint(r0), __float_as_uint(r1));
    } else {
        split_pair<DT>(p0, p1, hi, lo);
    }
}

template <int DT, int ODT, int D>
__global__ __launch_bounds__(kThreads) void prefill_attn_kernel(
    const uint16_t *__restrict__ q, const int32_t *__restrict__ cu_q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, void *__restrict__ out, int batch, int n_q_heads, int n_kv_heads,
    int mpps, int max_len, int n_blocks, int pos_per_wg, float scale_log2)
{
    constexpr int NT = kTiles;
    constexpr int NL = D / 32;                 // contraction chunks of q.K
    constexpr int ND = D / 16;                 // 16-dim output tiles
    constexpr int kBlockBytes = kPage * D * 2; // one K (or V) block of a page and head
    constexpr int kStageBytes = 4 * kBlockBytes;
    constexpr int kItems = kBlockBytes / 8;    // 16-byte K items of two pages = V granule pairs
    __shared__ __attribute__((aligned(16))) unsigned char stage[2][kStageBytes];

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
        return;                 // whole workgroup: no barrier has been reached
    const int first = L - n_b;  // position of the sequence's first query row
    const int rows_wg = pos_per_wg * group;
    const int n_steps = (first + min(n_b, i0 + pos_per_wg) - 1) / kStepKeys + 1;  // workgroup-wide
    const int n_pages = (L + kPage - 1) / kPage;

    const int tid = threadIdx.x;
    const int lane = tid & 63, g = lane >> 4, c = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this wavefront's rows; one without rows still copies and synchronises
    const int r_first = wv * NT * 16;
    const bool active = r_first < rows_wg && i0 + r_first / group < n_b;
    const int r_last = min(r_first + NT * 16, rows_wg) - 1;
    const int p_min = first + i0 + r_first / group;
    const int p_max = active ? first + min(n_b - 1, i0 + r_last / group) : -1;
    const int n_plain = active ? (p_min + 1) / kStepKeys : 0;  // steps with every key visible to every row
    const int s_last = p_max >= 0 ? p_max / kStepKeys : -1;    // last step with a visible key

    int pos[NT];
    bool valid[NT];
    int64_t row_off[NT];  // element offset of the lane's row in q / out
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
            qr[t][k] = *reinterpret_cast<const uint4 *>(q + row_off[t] + (4 * k + g) * 8);
    }

    // ---- arena -> LDS copy of one step: thread i < kItems moves 16 bytes of K
    // (page a for the first half of the items, page b for the second) and the
    // V granule i of both pages (8 bytes each), stored side by side
    const int64_t page_stride = (int64_t)n_kv_heads * (kPage * D);
    const int64_t head_off = (int64_t)hkv * (kPage * D);
    const int32_t *table = page_table + (int64_t)b * mpps;
    const bool copier = tid < kItems;
    const int k_sel = tid >= kItems / 2;
    const int k_off = (tid - k_sel * (kItems / 2)) * 8;  // elements inside the K block
    uint4 st_k;
    uint2 st_va, st_vb;
    auto fetch = [&](int s) {
        // the second page of the last step may not exist: re-read the last real
        // page instead; its keys lie beyond every position and are masked
        const int pa = table[min(2 * s, n_pages - 1)], pbb = table[min(2 * s + 1, n_pages - 1)];
        const int64_t base_a = (int64_t)pa * page_stride + head_off;
        const int64_t base_b = (int64_t)pbb * page_stride + head_off;
        if (copier) {
            st_k = *reinterpret_cast<const uint4 *>(k_arena + (k_sel ? base_b : base_a) + k_off);
            st_va = *reinterpret_cast<const uint2 *>(v_arena + base_a + tid * 4);
            st_vb = *reinterpret_cast<const uint2 *>(v_arena + base_b + tid * 4);
        }
    };
    auto deposit = [&](int buf) {
        if (copier) {
            *reinterpret_cast<uint4 *>(&stage[buf][tid * 16]) = st_k;
            *reinterpret_cast<uint4 *>(&stage[buf][2 * kBlockBytes + tid * 16]) =
                make_uint4(st_va.x, st_va.y, st_vb.x, st_vb.y);
        }
    };

    float m_ref[NT], l_part[NT];
    f32x4_t o[NT][ND];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        m_ref[t] = -INFINITY;
        l_part[t] = 0.f;
#pragma unroll
        for (int k = 0; k < ND; ++k)
            o[t][k] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    // One step of one wavefront.  kEdge: the step reaches past some row's
    // position (mask by position) or past L (blank V of never-written keys).
    auto process_step = [&](int s, int buf, auto edge) {
        constexpr bool kEdge = decltype(edge)::value;
        const int key0 = kStepKeys * s;
        const unsigned char *sk = &stage[buf][0];
        const unsigned char *sv = &stage[buf][2 * kBlockBytes];
        // phase 1: scores and probabilities of both tiles (K operands live)
        uint4 ph[NT], pl[NT];
        {
            uint4 ka[NL], kb[NL];
#pragma unroll
            for (int k = 0; k < NL; ++k) {
                ka[k] = *reinterpret_cast<const uint4 *>(sk + (k * 64 + lane) * 16);
                kb[k] = *reinterpret_cast<const uint4 *>(sk + kBlockBytes + (k * 64 + lane) * 16);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                // S^T: keys 4g+j of page a (sa) and of page b (sb) for row c
                f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < NL; ++k) {
                    sa = mfma_k32<DT>(ka[k], qr[t][k], sa);
                    sb = mfma_k32<DT>(kb[k], qr[t][k], sb);
                }
                float x[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[j] = sa[j];
                    x[4 + j] = sb[j];
                }
                if constexpr (kEdge) {
                    const int lim = pos[t] - key0 - 4 * g;  // key offset j is visible iff j <= lim
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        x[j] = j <= lim ? x[j] : -INFINITY;
                        x[4 + j] = kPage + j <= lim ? x[4 + j] : -INFINITY;
                    }
                }
                // scale_log2 > 0: the largest raw score is the largest scaled one
                const float top = scale_log2 * max2(max2(max2(x[0], x[1]), max2(x[2], x[3])),
                                                    max2(max2(x[4], x[5]), max2(x[6], x[7])));
                if (__any(top > m_ref[t] + kLift)) {
                    // move the reference of every row of the tile to its running maximum
                    float cm = fmaxf(top, __shfl_xor(top, 16));
                    cm = fmaxf(cm, __shfl_xor(cm, 32));
                    const float m_new = fmaxf(m_ref[t], cm);
                    const float alpha = fast_exp2(m_ref[t] - m_new);
                    m_ref[t] = m_new;
                    l_part[t] *= alpha;
#pragma unroll
                    for (int k = 0; k < ND; ++k)
                        o[t][k] *= alpha;
                }
                float p[8];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    p[j] = fast_exp2(fmaf(x[j], scale_log2, -m_ref[t]));
                l_part[t] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                split2<DT>(p[0], p[1], ph[t].x, pl[t].x);
                split2<DT>(p[2], p[3], ph[t].y, pl[t].y);
                split2<DT>(p[4], p[5], ph[t].z, pl[t].z);
                split2<DT>(p[6], p[7], ph[t].w, pl[t].w);
            }
        }
        // phase 2: O^T[dim][row] += V^T[dim][key] * P^T[key][row], 32 keys per product.
        // V^T operand k: rows = dims 16k + c, entries = keys 4g..4g+3 of page a, then of page b
        uint32_t a01 = ~0u, a23 = ~0u, b01 = ~0u, b23 = ~0u;
        if constexpr (kEdge) {
            if (key0 + kStepKeys > L) {  // blank never-written keys: 0 * NaN must not reach the product
                const int ja = key0 + 4 * g, jb = ja + kPage;
                a01 = (ja + 0 < L ? 0x0000ffffu : 0u) | (ja + 1 < L ? 0xffff0000u : 0u);
                a23 = (ja + 2 < L ? 0x0000ffffu : 0u) | (ja + 3 < L ? 0xffff0000u : 0u);
                b01 = (jb + 0 < L ? 0x0000ffffu : 0u) | (jb + 1 < L ? 0xffff0000u : 0u);
                b23 = (jb + 2 < L ? 0x0000ffffu : 0u) | (jb + 3 < L ? 0xffff0000u : 0u);
            }
        }
#pragma unroll
        for (int k = 0; k < ND; ++k) {
            uint4 vop = *reinterpret_cast<const uint4 *>(sv + (g * D + 16 * k + c) * 16);
            if constexpr (kEdge)
                vop = make_uint4(vop.x & a01, vop.y & a23, vop.z & b01, vop.w & b23);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                o[t][k] = mfma_k32<DT>(vop, ph[t], o[t][k]);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                o[t][k] = mfma_k32<DT>(vop, pl[t], o[t][k]);
        }
    };
    // Pipeline: while step s is computed out of one LDS buffer, the global loads
    // of step s+1 are in flight; they are written to the other buffer after the
    // computation, and one barrier per step orders both the hand-over of that
    // buffer and the reuse of the current one.  Every wavefront passes the same
    // n_steps - 1 barriers, but spends them in two loops of its own lengths: its
    // mask-free steps first, then its edge steps (and steps past its last
    // position, where it only copies).  The last step is peeled so that the
    // prefetch in the loops is unconditional.
    fetch(0);
    deposit(0);
    // Everything loaded so far (q included) has arrived before the loops start:
    // otherwise the wait counters inside them must allow for q still being in
    // flight, which in steady state means waiting for the prefetch just issued.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int s = 0;
    for (const int s_end = min(n_plain, n_steps - 1); s < s_end; ++s) {
        fetch(s + 1);
        process_step(s, s & 1, std::false_type{});
        deposit((s + 1) & 1);
        __syncthreads();
    }
    for (; s + 1 < n_steps; ++s) {
        fetch(s + 1);
        if (s <= s_last)
            process_step(s, s & 1, std::true_type{});
        deposit((s + 1) & 1);
        __syncthreads();
    }
    if (s <= s_last)
        process_step(s, s & 1, std::true_type{});

    // o[t][k][j] is dim 16k + 4g + j of row c
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float l_all = l_part[t] + __shfl_xor(l_part[t], 16);
        l_all += __shfl_xor(l_all, 32);
        if (!active || !valid[t])
            continue;
        const float inv = 1.0f / l_all;
#pragma unroll
        for (int k = 0; k < ND; ++k) {
            const int64_t idx = row_off[t] + 16 * k + 4 * g;
            const float x0 = o[t][k][0] * inv, x1 = o[t][k][1] * inv, x2 = o[t][k][2] * inv,
                        x3 = o[t][k][3] * inv;
            if constexpr (ODT == RLHF_F32)
                *(float4 *)((float *)out + idx) = make_float4(x0, x1, x2, x3);
            else
                *(uint2 *)((uint16_t *)out + idx) =
                    make_uint2((uint32_t)pack16<ODT>(x0) | ((uint32_t)pack16<ODT>(x1) << 16),
                               (uint32_t)pack16<ODT>(x2) | ((uint32_t)pack16<ODT>(x3) << 16));
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
    hipLaunchKernelGGL((prefill_attn_kernel<DT, ODT, D>), dim3((unsigned)grid), dim3(kThreads), 0, s,
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
    if (p.softmax_scale < 0.f)
        return fail(RLHF_ERR_INVALID, "softmax_scale must not be negative");
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
