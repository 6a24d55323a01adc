// Causal attention of a block of new tokens per sequence over the paged KV
// arena ("prefill": a prompt, or a chunk of one, entering the cache before the
// one-token-per-step generation of Section 2.1 starts).
//
// Unlike a decode step this is a real contraction -- every key of a sequence
// meets hundreds of query rows -- so both products run on the matrix cores and
// the kernel is bound by them, not by HBM.
//
// Work split.  A workgroup (8 or 12 wavefronts: two or three per SIMD) owns one
// (sequence, KV head) and a block of consecutive new positions; its 256 or 384
// query rows are the pairs (position, head of the KV head's group), flattened
// position-major.  Twelve wavefronts hide more of the LDS and barrier latency
// and copy each K/V block for more rows; eight make more, smaller workgroups
// for small calls.
// Each wavefront keeps one tile of 32 rows (q and the output accumulators) in
// registers.  The workgroup walks the keys 0 .. (its last position) in steps of
// 32 keys = two pages; the step's K and V blocks are copied once from the arena
// into LDS (double-buffered, the next step's global loads in flight during the
// current step) and every wavefront takes its matrix operands from there.
// Workgroups are numbered so that those of one (sequence, KV head) land on the
// same XCD one after the other (its K/V stays in that XCD's L2) and the long,
// late position blocks start first.
//
// All products are 32x32x16 matrix-core instructions (the shape one wavefront
// can issue at full rate).  Per step, with lane l = (h = l/32, c = l%32):
//   S^T[key][row]   = K (A operand: in LDS the two pages' K granules are
//                     interleaved to [dim/8][32 keys][8 dims], so lane l reads
//                     16 contiguous bytes at granule 64*i + l) x q rows (B
//                     operand, registers): lane (h, c) receives, for row c, the
//                     16 keys 8*(r/4) + 4h + r%4, r = 0..15;
//   softmax         against a per-row reference exponent that is only moved
//                     (and the accumulators rescaled) when some score exceeds
//                     it by more than 2^kLift -- after the first steps of a row
//                     that never happens, so the common step has no cross-lane
//                     traffic and no rescaling;
//   O^T[dim][row]  += V^T (A operand: in LDS the 4-key granules are paired so
//                     that 16 bytes hold exactly the 8 keys the lane's half h
//                     contributes) x P^T (B operand: the registers S^T arrived
//                     in, first 8 for the first page, last 8 for the second).
// The P.V product runs in fp16 whatever the cache type: weights are rounded to
// fp16 (relative error up to 2^-11 each; a bf16 weight would carry 2^-8, more than the
// result may be off by), kept as 2^kShift * exp(score - reference) so that none
// that matters falls under fp16's normal range, and a bf16 V block is converted
// on its way into LDS (exact for magnitudes from 2^-14 to 65504; larger ones
// become infinity).  Row sums are taken in fp32 from the unrounded weights and
// stay per lane until the end.  Steps that lie
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
// Wavefronts per workgroup: twelve (three per SIMD, which the kernel's 168 registers just allow) when the
// launch has workgroups enough to fill the chip several times over, else eight (smaller blocks of positions).
constexpr int kWavesSmall = 8, kWavesLarge = 12;
constexpr int kTileRows = 32;                      // query rows per wavefront
constexpr int kMaxGroup = kWavesSmall * kTileRows;  // query heads per KV head the smaller workgroup can hold
constexpr int kStepKeys = 2 * kPage;
constexpr int kXcds = 8;
constexpr float kLift = 5.0f;   // log2 units a score may exceed the reference before it is moved
constexpr float kShift = 10.0f;  // weights are kept as 2^kShift * exp(score - reference): at most 2^15 in fp16,
                                 // and what falls under fp16's normal range is below 2^-24 of a row's largest

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// Two fp32 -> packed fp16, round to nearest (v_cvt_pk_f16_f32), `first` in the low half.
__device__ __forceinline__ uint32_t pack_f16(float first, float second)
{
    const float2_t v = {first, second};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, half2_t));
}

// acc + lo + hi of two packed fp16, in fp32 (v_dot2_f32_f16 against (1, 1)).
__device__ __forceinline__ float pair_sum(uint32_t packed, float acc)
{
    const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, packed), ones, acc, false);
}

// Two packed bf16 -> two packed fp16.  Exact for magnitudes in fp16's normal
// range; smaller ones round (absolute error under 2^-25), 65536 and above
// become infinity.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w)
{
    return pack_f16(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}

template <int DT, int ODT, int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void prefill_attn_kernel(
    const uint16_t *__restrict__ q, const int32_t *__restrict__ cu_q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, void *__restrict__ out, int batch, int n_q_heads, int n_kv_heads,
    int mpps, int max_len, int n_blocks, int pos_per_wg, float scale_log2)
{
    constexpr int NC = D / 16;                 // 16-dim contraction chunks of q.K
    constexpr int ND = D / 32;                 // 32-dim output tiles
    constexpr int kBlockBytes = kPage * D * 2; // one K (or V) block of a page and head
    constexpr int kStageBytes = 4 * kBlockBytes;
    constexpr int kItems = kBlockBytes / 8;    // 16-byte copy items of K (two pages) = of V
    constexpr int kThreads = WAVES * 64;
    constexpr int kCopies = (kItems + kThreads - 1) / kThreads;
    // One LDS block: the two K/V stages first (their addresses then fit the 16-bit offset field of
    // the LDS instructions), then a per-wavefront exchange tile (32 rows of up to 256 bytes) for the
    // output: rows leave through it, so that global memory sees whole rows (full cache lines) per
    // store instruction although the accumulators hold the matrix layout (a lane: four dims of one
    // row per register quad).  The 16-byte chunks of a row are XOR-swizzled with the row number to
    // spread both access patterns over the banks.
    constexpr int kXchgRow = 256;
    constexpr int kXchgBytes = kTileRows * kXchgRow;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kStageBytes + WAVES * kXchgBytes];
    unsigned char (*stage)[kStageBytes] = reinterpret_cast<unsigned char (*)[kStageBytes]>(lds);

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
    const int lane = tid & 63, h = lane >> 5, c = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this wavefront's rows; one without rows still copies and synchronises
    const int r_first = wv * kTileRows;
    const bool active = r_first < rows_wg && i0 + r_first / group < n_b;
    const int r_last = min(r_first + kTileRows, rows_wg) - 1;
    const int p_min = first + i0 + r_first / group;
    const int p_max = active ? first + min(n_b - 1, i0 + r_last / group) : -1;
    const int n_plain = active ? (p_min + 1) / kStepKeys : 0;  // steps with every key visible to every row
    const int s_last = p_max >= 0 ? p_max / kStepKeys : -1;    // last step with a visible key

    // the lane's row: q as the B operand of chunk i = dims 16i + 8h .. +8
    const int r_raw = r_first + c;
    const int r = min(r_raw, rows_wg - 1);
    const int il = r / group, hg = r - il * group;
    const int i_row = min(i0 + il, n_b - 1);
    const int pos = first + i_row;
    const int64_t row_off = ((int64_t)(q0 + i_row) * n_q_heads + hkv * group + hg) * D;
    uint4 qr[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i)
        qr[i] = *reinterpret_cast<const uint4 *>(q + row_off + 16 * i + 8 * h);

    // ---- arena -> LDS copy of one step, thread tid moving items tid, tid + kThreads, ...
    // K item: 16 bytes = 8 dims of one key; arena granule (dim/8, slot) of page
    //   a or b goes to granule (dim/8)*32 + 16*page + slot.
    // V item (page, half hh, dim): the arena's 4-key granules of quads hh and
    //   hh + 2 for that dim (8 bytes each) go side by side to granule
    //   (2*page + hh)*D + dim: the 8 keys 4hh..4hh+3, 8+4hh..8+4hh+3 of the page.
    const int64_t page_stride = (int64_t)n_kv_heads * (kPage * D);
    const int64_t head_off = (int64_t)hkv * (kPage * D);
    const int32_t *table = page_table + (int64_t)b * mpps;
    struct Staged {  // one step's copy items in registers, between the global load and the LDS store
        uint4 k[kCopies];
        uint2 v0[kCopies], v1[kCopies];
    };
    // Page ids of a step.  Steps past the end, and the second page of a last
    // step that has only one, stand in the sequence's last real page: its keys
    // lie beyond every position and are masked (or the copy is never used).
    auto page_ids = [&](int s, int &pa, int &pbb) {
        pa = table[min(2 * s, n_pages - 1)];
        pbb = table[min(2 * s + 1, n_pages - 1)];
    };
    auto fetch = [&](Staged &st, int pa, int pbb) {
#pragma unroll
        for (int i = 0; i < kCopies; ++i) {
            // A wavefront's 64 items lie in one page (kItems / 2 is a multiple of 64), so
            // the page and its base address are scalars and the loads take them as such.
            const int item0 = wv * 64 + i * kThreads;
            if (kItems % kThreads == 0 || item0 < kItems) {
                const bool second = item0 >= kItems / 2;  // page b
                const int64_t base = (int64_t)(second ? pbb : pa) * page_stride + head_off;
                const uint16_t *kp = k_arena + base, *vp = v_arena + base;
                const int within = lane + item0 - (second ? kItems / 2 : 0);
                st.k[i] = *reinterpret_cast<const uint4 *>(kp + within * 8);
                const int hh = within / D, dim = within - hh * D;
                st.v0[i] = *reinterpret_cast<const uint2 *>(vp + (hh * D + dim) * 4);
                st.v1[i] = *reinterpret_cast<const uint2 *>(vp + ((hh + 2) * D + dim) * 4);
            }
        }
    };
    auto deposit = [&](const Staged &st, int buf) {
#pragma unroll
        for (int i = 0; i < kCopies; ++i) {
            const int item0 = wv * 64 + i * kThreads;
            if (kItems % kThreads == 0 || item0 < kItems) {
                const int item = item0 + lane;
                const int second = item0 >= kItems / 2;
                const int within = item - second * (kItems / 2);
                const int d8 = within >> 4, slot = within & 15;
                *reinterpret_cast<uint4 *>(&stage[buf][(d8 * 32 + 16 * second + slot) * 16]) = st.k[i];
                uint4 v = make_uint4(st.v0[i].x, st.v0[i].y, st.v1[i].x, st.v1[i].y);
                if constexpr (DT == RLHF_BF16)  // the P.V product runs in fp16
                    v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z),
                                   bf16x2_to_f16x2(v.w));
                *reinterpret_cast<uint4 *>(&stage[buf][2 * kBlockBytes + item * 16]) = v;
            }
        }
    };

    float m_ref = -INFINITY, l_part = 0.f;
    f32x16_t o[ND];
#pragma unroll
    for (int k = 0; k < ND; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            o[k][j] = 0.f;

    // One step of one wavefront.  kEdge: the step reaches past some row's
    // position (mask by position) or past L (blank V of never-written keys).
    auto process_step = [&](int s, int buf, auto edge) {
        constexpr bool kEdge = decltype(edge)::value;
        const int key0 = kStepKeys * s;
        const unsigned char *sk = &stage[buf][0];
        const unsigned char *sv = &stage[buf][2 * kBlockBytes];
        // S^T: register r holds key 8*(r/4) + 4h + r%4 of the step for row c
        f32x16_t sc;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            sc[j] = 0.f;
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const uint4 kop = *reinterpret_cast<const uint4 *>(sk + (64 * i + lane) * 16);
            sc = mfma_32x32<DT>(kop, qr[i], sc);
        }
        float x[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            x[j] = sc[j];
        if constexpr (kEdge) {
            const int lim = pos - key0 - 4 * h;  // key offset 8*(r/4) + r%4 is visible iff <= lim
#pragma unroll
            for (int j = 0; j < 16; ++j)
                x[j] = 8 * (j / 4) + j % 4 <= lim ? x[j] : -INFINITY;
        }
        // Move the reference of the rows up to their running maximum when some
        // score exceeds it by more than 2^kLift (rare after a row's first steps).
        // scale_log2 > 0: the largest raw score is the largest scaled one.
        // three-operand maxima (v_max3_f32): eight instructions for the sixteen scores
        auto max3 = [](float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); };
        float top = max3(max3(max3(x[0], x[1], x[2]), max3(x[3], x[4], x[5]), max3(x[6], x[7], x[8])),
                         max3(max3(x[9], x[10], x[11]), max3(x[12], x[13], x[14]), x[15]), -INFINITY);
        top *= scale_log2;
        if (__any(top > m_ref + (kLift + kShift))) {  // m_ref is the reference minus kShift
            const float cm = fmaxf(top, __shfl_xor(top, 32)) - kShift;
            const float m_new = fmaxf(m_ref, cm);
            const float alpha = fast_exp2(m_ref - m_new);
            m_ref = m_new;
            l_part *= alpha;
#pragma unroll
            for (int k = 0; k < ND; ++k)
                o[k] *= alpha;
        }
        float p[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            p[j] = fast_exp2(fmaf(x[j], scale_log2, -m_ref));
        // P^T as B operands: entries 8h..8h+7 of page a are registers 0..7, of page b 8..15
        uint4 ph[2];
#pragma unroll
        for (int e = 0; e < 2; ++e)
            ph[e] = make_uint4(pack_f16(p[8 * e + 0], p[8 * e + 1]), pack_f16(p[8 * e + 2], p[8 * e + 3]),
                               pack_f16(p[8 * e + 4], p[8 * e + 5]), pack_f16(p[8 * e + 6], p[8 * e + 7]));
        // Row sums from the rounded weights, the very numbers the product below uses
        // (numerator and denominator see the same rounding), two per instruction.
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            l_part = pair_sum(ph[e].x, l_part);
            l_part = pair_sum(ph[e].y, l_part);
            l_part = pair_sum(ph[e].z, l_part);
            l_part = pair_sum(ph[e].w, l_part);
        }
        // O^T[dim][row] += V^T[dim][key] * P^T[key][row], 16 keys (one page) per product
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            uint32_t m01 = ~0u, m23 = ~0u, m45 = ~0u, m67 = ~0u;
            if constexpr (kEdge) {
                if (key0 + kStepKeys > L) {  // blank never-written keys: 0 * NaN must not reach the product
                    const int j0 = key0 + kPage * e + 4 * h, j1 = j0 + 8;
                    m01 = (j0 + 0 < L ? 0x0000ffffu : 0u) | (j0 + 1 < L ? 0xffff0000u : 0u);
                    m23 = (j0 + 2 < L ? 0x0000ffffu : 0u) | (j0 + 3 < L ? 0xffff0000u : 0u);
                    m45 = (j1 + 0 < L ? 0x0000ffffu : 0u) | (j1 + 1 < L ? 0xffff0000u : 0u);
                    m67 = (j1 + 2 < L ? 0x0000ffffu : 0u) | (j1 + 3 < L ? 0xffff0000u : 0u);
                }
            }
#pragma unroll
            for (int k = 0; k < ND; ++k) {
                // rows = dims 32k + c, entries = keys 4h..4h+3 and 8+4h..8+4h+3 of page e
                uint4 vop = *reinterpret_cast<const uint4 *>(sv + ((2 * e + h) * D + 32 * k + c) * 16);
                if constexpr (kEdge)
                    vop = make_uint4(vop.x & m01, vop.y & m23, vop.z & m45, vop.w & m67);
                o[k] = mfma_32x32<RLHF_F16>(vop, ph[e], o[k]);
            }
        }
    };

    // Pipeline.  A step's K/V go arena -> registers -> LDS -> matrix operands.
    // The global loads of step s+2 are issued at the top of step s (their page
    // ids were read a step earlier still) and land in LDS at the end of step
    // s+1, so two steps of computation cover the dependent page-id -> data
    // latency; the LDS buffers alternate, and the one barrier per step orders
    // both the hand-over of the buffer just written and the reuse of the one
    // just read.  The two register sets alternate as well, which is why the
    // loops below take two steps per trip.  Every wavefront passes n_steps
    // barriers, but spends them in two loops of its own lengths: its mask-free
    // steps first (an even number of them), then its edge steps and the steps
    // past its last position, where it only copies.
    Staged set_a, set_b;
    int pa, pbb;
    page_ids(0, pa, pbb);
    fetch(set_a, pa, pbb);
    page_ids(1, pa, pbb);
    fetch(set_b, pa, pbb);
    page_ids(2, pa, pbb);
    deposit(set_a, 0);
    // Everything loaded so far (q included) has arrived before the loops start:
    // otherwise the wait counters inside them must allow for q still being in
    // flight, which in steady state means waiting for the prefetch just issued.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    // one step: `mine` is free (its content went to LDS a step ago) and takes
    // step s+2; `other` holds step s+1 and is written out after the computation
    auto advance = [&](int s, Staged &mine, const Staged &other, auto edge) {
        fetch(mine, pa, pbb);
        page_ids(s + 3, pa, pbb);
        if (!decltype(edge)::value || s <= s_last)
            process_step(s, s & 1, edge);
        deposit(other, (s + 1) & 1);
        __syncthreads();
    };
    int s = 0;
    for (const int s_end = min(n_plain, n_steps) & ~1; s < s_end; s += 2) {
        advance(s, set_a, set_b, std::false_type{});
        advance(s + 1, set_b, set_a, std::false_type{});
    }
    for (; s < n_steps; s += 2) {
        advance(s, set_a, set_b, std::true_type{});
        if (s + 1 < n_steps)
            advance(s + 1, set_b, set_a, std::true_type{});
    }

    // o[k][r] is dim 32k + 8*(r/4) + 4h + r%4 of row c.  The tile goes to the exchange buffer row by
    // row (normalised, in the output type) and leaves it as whole rows: 16 bytes per lane, a row's
    // bytes side by side in one instruction.  Everything the stores need is derived here from the
    // lane number again, so that none of it occupies a register during the steps above.
    const float l_all = l_part + __shfl_xor(l_part, 32);
    const float inv = 1.0f / l_all;
    int ln = threadIdx.x & 63;
    asm volatile("" : "+v"(ln));
    const int c2 = ln & 31, h2 = ln >> 5;
    constexpr int OSZ = ODT == RLHF_F32 ? 4 : 2;
    constexpr int ORB = D * OSZ < kXchgRow ? D * OSZ : kXchgRow;  // row bytes per pass
    constexpr int NP = D * OSZ / ORB;                              // passes
    constexpr int KP = ND / NP;                                    // 32-dim tiles per pass
    constexpr int OCH = ORB / 16, ORPI = 64 / OCH, ON = kTileRows / ORPI;
    const int och = ln % OCH, osub = ln / OCH;
    const float inv_group = 1.0f / (float)group;
    unsigned char *mine = lds + 2 * kStageBytes + wv * kXchgBytes;
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
#pragma unroll
        for (int kk = 0; kk < KP; ++kk) {
            const int k = ps * KP + kk;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const float x0 = o[k][4 * qd] * inv, x1 = o[k][4 * qd + 1] * inv, x2 = o[k][4 * qd + 2] * inv,
                            x3 = o[k][4 * qd + 3] * inv;
                const int off = (32 * kk + 8 * qd + 4 * h2) * OSZ;  // byte offset in the pass's row part
                unsigned char *dst = mine + c2 * ORB + (((off >> 4) ^ (c2 % OCH)) << 4) + (off & 15);
                if constexpr (ODT == RLHF_F32)
                    *(float4 *)dst = make_float4(x0, x1, x2, x3);
                else
                    *(uint2 *)dst = make_uint2(pack16x2<ODT>(x0, x1), pack16x2<ODT>(x2, x3));
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < ON; ++t) {
            const int j = ORPI * t + osub;
            const int rr = r_first + j, rc = min(rr, rows_wg - 1);
            // rc / group without an integer division: rc < 2^9, so the fp32 product is exact enough
            const int ilj = (int)(((float)rc + 0.5f) * inv_group), hgj = rc - ilj * group;
            const bool exists = active && rr < rows_wg && i0 + ilj < n_b;
            const int64_t row = ((int64_t)(q0 + min(i0 + ilj, n_b - 1)) * n_q_heads + hkv * group + hgj) * D;
            const uint4 w = *reinterpret_cast<const uint4 *>(mine + j * ORB + ((och ^ (j % OCH)) << 4));
            if (exists)
                *reinterpret_cast<uint4 *>((unsigned char *)out + row * OSZ + ps * ORB + och * 16) = w;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

template <int DT, int ODT, int D, int WAVES>
int launch_waves(const rlhf_attn_params &p, const void *q, const int32_t *cu_q, int max_q_len, const void *k_arena,
                 const void *v_arena, const int32_t *page_table, const int32_t *seq_lens, void *out, hipStream_t s)
{
    const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)D);
    const int group = p.n_q_heads / p.n_kv_heads;
    const int pos_per_wg = WAVES * kTileRows / group;
    const int n_blocks = (max_q_len + pos_per_wg - 1) / pos_per_wg;
    const int64_t units = (int64_t)p.batch * p.n_kv_heads;
    const int64_t grid = (units + kXcds - 1) / kXcds * kXcds * n_blocks;
    if (grid > max_workgroups(WAVES * 64))
        return fail(RLHF_ERR_UNSUPPORTED, "prefill launch of %lld workgroups: split the call", (long long)grid);
    const int cap = p.max_pages_per_seq * kPage;
    const int max_len = (p.max_seq_len > 0 && p.max_seq_len < cap) ? p.max_seq_len : cap;
    hipLaunchKernelGGL((prefill_attn_kernel<DT, ODT, D, WAVES>), dim3((unsigned)grid), dim3(WAVES * 64), 0, s,
                       (const uint16_t *)q, cu_q, (const uint16_t *)k_arena, (const uint16_t *)v_arena,
                       page_table, seq_lens, out, p.batch, p.n_q_heads, p.n_kv_heads, p.max_pages_per_seq,
                       max_len, n_blocks, pos_per_wg, scale * kLog2e);
    RLHF_LAUNCH_CHECK("prefill_attn_kernel");
    return RLHF_OK;
}

template <int DT, int ODT, int D>
int launch(const rlhf_attn_params &p, const void *q, const int32_t *cu_q, int max_q_len, const void *k_arena,
           const void *v_arena, const int32_t *page_table, const int32_t *seq_lens, void *out, int waves,
           hipStream_t s)
{
    // the larger workgroup when it still leaves about sixteen workgroups per compute unit (256 of them)
    const int group = p.n_q_heads / p.n_kv_heads;
    const int pos_large = kWavesLarge * kTileRows / group;
    const int64_t wgs_large = (int64_t)p.batch * p.n_kv_heads * ((max_q_len + pos_large - 1) / pos_large);
    if (waves == kWavesLarge || (waves == 0 && wgs_large >= 4096))
        return launch_waves<DT, ODT, D, kWavesLarge>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens,
                                                     out, s);
    return launch_waves<DT, ODT, D, kWavesSmall>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out,
                                                 s);
}

template <int DT, int D>
int launch_out(const rlhf_attn_params &p, const void *q, const int32_t *cu_q, int max_q_len,
               const void *k_arena, const void *v_arena, const int32_t *page_table, const int32_t *seq_lens,
               void *out, int waves, hipStream_t s)
{
    if (p.out_dtype == RLHF_F32)
        return launch<DT, RLHF_F32, D>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, waves,
                                       s);
    return launch<DT, DT, D>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, waves, s);
}

}  // namespace
}  // namespace rlhf

using namespace rlhf;

extern "C" int rlhf_prefill_attention(const rlhf_attn_params *params, const void *q, const int32_t *cu_q,
                                      int32_t max_q_len, const void *k_arena, const void *v_arena,
                                      const int32_t *page_table, const int32_t *seq_lens, void *out,
                                      void *stream)
{
    return rlhf_prefill_attention_wg(params, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, 0,
                                     stream);
}

extern "C" int rlhf_prefill_attention_wg(const rlhf_attn_params *params, const void *q, const int32_t *cu_q,
                                         int32_t max_q_len, const void *k_arena, const void *v_arena,
                                         const int32_t *page_table, const int32_t *seq_lens, void *out,
                                         int32_t wavefronts_per_workgroup, void *stream)
{
    const int waves = wavefronts_per_workgroup;
    if (waves != 0 && waves != kWavesSmall && waves != kWavesLarge)
        return fail(RLHF_ERR_INVALID, "wavefronts_per_workgroup %d (0, %d or %d)", waves, kWavesSmall, kWavesLarge);
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
    if (p.n_q_heads / p.n_kv_heads > kMaxGroup)
        return fail(RLHF_ERR_UNSUPPORTED, "more than %d query heads per kv head", kMaxGroup);
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
                                              out, waves, s);
        return launch_out<RLHF_BF16, 64>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, waves,
                                         s);
    }
    if (p.head_dim == 128)
        return launch_out<RLHF_F16, 128>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, waves,
                                         s);
    return launch_out<RLHF_F16, 64>(p, q, cu_q, max_q_len, k_arena, v_arena, page_table, seq_lens, out, waves, s);
}
