// Next-token sampling fused with the vocabulary pass.
//
// In the paper's PPO stage the actor generates its responses token by token
// (Section 2.1); after every decode step one token per sequence is drawn from
// the actor's logits.  One pass over a row yields both the sample and its
// log-probability:
//
//   token = argmax_v ( a_v / T + G_v ),  G_v = -ln(-ln u_v)      (Gumbel-max:
//           an exact draw from softmax(a / T)); T = 0 means greedy argmax
//   logp  = a_token / T - logsumexp(a / T)
//
// The uniforms are counter-based, so no noise is read from memory: u_v comes
// from word v%4 of Philox4x32-10 with counter (v/4, row, offset low, offset
// high) and key = seed (Salmon et al., SC'11; implemented here from the
// published round function).  The top 23 bits are used, centred in their cell,
// so that u and 1-u are exact in fp32.  -ln u is taken with a short series when
// u is within 2^-6 of 1 (where a hardware log loses relative accuracy and where
// the largest Gumbel values, the ones that decide the argmax, come from).
//
// One workgroup (256 or 1024 lanes) owns one row, or, when the caller brings a
// workspace and the rows are too few to occupy the chip, one of up to eight
// segments of a row; a second small kernel then merges the segments' (best
// score, index, sum) records.  Noise depends on (row, index) only, so the split
// changes nothing in the draw.  The pass is bound by the vector ALU (ten Philox
// rounds per four logits plus three transcendentals per logit), not by HBM: a
// decode step reads only batch x vocab logits.
//
// The top-k variant keeps the entries at or above the k-th largest logit of the
// row (ties included) and draws among them with the same per-entry noise; it
// finds that threshold exactly and then needs noise for the survivors only, so
// for the usual k it is cheaper than the plain draw (sample_topk_kernel below).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>

#include "common.h"
#include "device_ops.h"

namespace rlhf {
namespace {

// Lanes per row: 256 when there are rows enough to fill the chip, 1024 when a
// decode step brings only a few hundred rows (then a row's latency matters).
constexpr int kFewRows = 1024;
constexpr float kLift = 40.0f;
constexpr float kNoRef = -1.0e30f;

__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        // one 32x32->64 multiply-add instruction per product instead of a high and a low multiply
        const uint64_t p0 = (uint64_t)M0 * c.x, p1 = (uint64_t)M1 * c.z;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
        k.x += 0x9E3779B9u;
        k.y += 0xBB67AE85u;
    }
    return c;
}

// ln x for normal x > 0 on the hardware log2 (v_log_f32) alone: the library
// form adds range fix-up code for denormals, which u >= 2^-24 and
// e = -ln u >= 2^-24 never are.
__device__ __forceinline__ float fast_ln(float x)
{
    return __builtin_amdgcn_logf(x) * kLn2;
}

// Gumbel noise from one 32-bit word.
__device__ __forceinline__ float gumbel(uint32_t word)
{
    const float u = ((float)(word >> 9) + 0.5f) * (1.0f / 8388608.0f);  // in (0,1), exact
    // e = -ln u is Exp(1).  Near u = 1 it is taken from the series of -ln(1 - c),
    // c = 1 - u (exact), because a hardware log loses relative accuracy there.
    const float c = 1.0f - u;
    const float series = c * (1.0f + c * (0.5f + c * (1.0f / 3.0f + c * 0.25f)));
    const float e = c < 0.015625f ? series : -fast_ln(u);
    return -fast_ln(e);
}

struct Lane {
    float best_z = -INFINITY;
    int best_i = INT_MAX;
    float ref2 = kNoRef * kLog2e;  // reference exponent of the running sum, log2 units
    float lift = kNoRef + kLift;
    float s = 0.f;                 // sum 2^(y*log2e - ref2), y = a / T
};

// LSE = false leaves the running sum of exponentials out (no log-probability asked for).
template <bool NOISE, bool LSE = true>
__device__ __forceinline__ void take(Lane &st, float y, float g, int v)
{
    const float z = NOISE ? y + g : y;
    if (z > st.best_z) {  // strict: a lane sees its indices in increasing order
        st.best_z = z;
        st.best_i = v;
    }
    if constexpr (!LSE)
        return;
    if (y > st.lift) {
        const float ref2 = y * kLog2e;
        st.s *= fast_exp2(st.ref2 - ref2);
        st.ref2 = ref2;
        st.lift = y + kLift;
    }
    st.s += fast_exp2(fmaf(y, kLog2e, -st.ref2));
}

// Four consecutive entries starting at a multiple of four: one Philox block.
template <bool NOISE, bool LSE = true>
__device__ __forceinline__ void take4(Lane &st, const float (&y)[4], int v0, uint32_t row, uint2 off, uint2 key)
{
    uint4 r = make_uint4(0, 0, 0, 0);
    if (NOISE)
        r = philox4x32_10(make_uint4((uint32_t)(v0 >> 2), row, off.x, off.y), key);
    take<NOISE, LSE>(st, y[0], NOISE ? gumbel(r.x) : 0.f, v0);
    take<NOISE, LSE>(st, y[1], NOISE ? gumbel(r.y) : 0.f, v0 + 1);
    take<NOISE, LSE>(st, y[2], NOISE ? gumbel(r.z) : 0.f, v0 + 2);
    take<NOISE, LSE>(st, y[3], NOISE ? gumbel(r.w) : 0.f, v0 + 3);
}

template <bool NOISE, bool LSE = true>
__device__ __forceinline__ void take1(Lane &st, float y, int v, uint32_t row, uint2 off, uint2 key)
{
    float g = 0.f;
    if (NOISE) {
        const uint4 r = philox4x32_10(make_uint4((uint32_t)(v >> 2), row, off.x, off.y), key);
        const uint32_t word = (v & 3) == 0 ? r.x : (v & 3) == 1 ? r.y : (v & 3) == 2 ? r.z : r.w;
        g = gumbel(word);
    }
    take<NOISE, LSE>(st, y, g, v);
}

// Larger score wins; equal scores go to the lower index.
__device__ __forceinline__ void better(float &z, int &i, float oz, int oi)
{
    if (oz > z || (oz == z && oi < i)) {
        z = oz;
        i = oi;
    }
}

// What a segment of a row leaves for the merge.
struct SegmentRecord {
    float best_z;
    int32_t best_i;
    float ref2;  // reference exponent of `s`, log2 units
    float s;
};

// Workgroup (x, y, z) takes segment z of gridDim.z of row y * kRowSlab + x.  With
// one segment it writes the row's results; with more it writes its record to
// `records` [row][segment].
template <int DT, bool VEC, bool NOISE, bool LSE, int kThreads>
__global__ __launch_bounds__(kThreads) void sample_tokens_kernel(
    const void *__restrict__ logits, int32_t *__restrict__ tokens_out, float *__restrict__ logp_out,
    SegmentRecord *__restrict__ records, int64_t n_rows, int vocab, int64_t stride, float inv_t, uint2 key,
    uint2 off)
{
    constexpr int kWaves = kThreads / 64;
    __shared__ float s_f[kWaves];
    __shared__ int s_i[kWaves];
    const int64_t row64 = (int64_t)blockIdx.y * kRowSlab + blockIdx.x;
    if (row64 >= n_rows)  // the last slab of a grid of more than kRowSlab rows
        return;
    const uint32_t row = (uint32_t)row64;
    const int seg = blockIdx.z, n_seg = gridDim.z;
    const int tid = threadIdx.x;
    constexpr int EB = (DT == RLHF_F32) ? 4 : 2;
    const char *base = (const char *)logits + row64 * stride * EB;

    Lane st;
    if constexpr (VEC) {
        constexpr int E = (DT == RLHF_F32) ? 4 : 8;
        const int nvec = vocab / E;
        const uint4 *p = (const uint4 *)base;
        const int i_begin = (int)((int64_t)nvec * seg / n_seg), i_end = (int)((int64_t)nvec * (seg + 1) / n_seg);
        for (int i = i_begin + tid; i < i_end; i += kThreads) {
            const uint4 u = load16(p + i);
            if constexpr (DT == RLHF_F32) {
                const float y[4] = {__uint_as_float(u.x) * inv_t, __uint_as_float(u.y) * inv_t,
                                    __uint_as_float(u.z) * inv_t, __uint_as_float(u.w) * inv_t};
                take4<NOISE, LSE>(st, y, i * 4, row, off, key);
            } else {
                const float y0[4] = {unpack_lo<DT>(u.x) * inv_t, unpack_hi<DT>(u.x) * inv_t,
                                     unpack_lo<DT>(u.y) * inv_t, unpack_hi<DT>(u.y) * inv_t};
                const float y1[4] = {unpack_lo<DT>(u.z) * inv_t, unpack_hi<DT>(u.z) * inv_t,
                                     unpack_lo<DT>(u.w) * inv_t, unpack_hi<DT>(u.w) * inv_t};
                take4<NOISE, LSE>(st, y0, i * 8, row, off, key);
                take4<NOISE, LSE>(st, y1, i * 8 + 4, row, off, key);
            }
        }
        const int done = nvec * E;
        if (seg == n_seg - 1 && tid < vocab - done)
            take1<NOISE, LSE>(st, load_scalar<DT>(base, done + tid) * inv_t, done + tid, row, off, key);
    } else {
        const int v_begin = (int)((int64_t)vocab * seg / n_seg), v_end = (int)((int64_t)vocab * (seg + 1) / n_seg);
        for (int v = v_begin + tid; v < v_end; v += kThreads)
            take1<NOISE, LSE>(st, load_scalar<DT>(base, v) * inv_t, v, row, off, key);
    }

    // best (score, index) of the row: wavefront butterflies, then the four wavefronts
    float z = st.best_z;
    int idx = st.best_i;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1)
        better(z, idx, __shfl_xor(z, d), __shfl_xor(idx, d));
    if ((tid & 63) == 0) {
        s_f[tid >> 6] = z;
        s_i[tid >> 6] = idx;
    }
    __syncthreads();
    z = s_f[0];
    idx = s_i[0];
#pragma unroll
    for (int k = 1; k < kWaves; ++k)
        better(z, idx, s_f[k], s_i[k]);
    if (idx == INT_MAX && n_seg == 1)  // nothing but -inf / NaN in the row
        idx = 0;
    __syncthreads();

    // logsumexp of a / T
    float w = wave_max(st.ref2);
    if ((tid & 63) == 0)
        s_f[tid >> 6] = w;
    __syncthreads();
    float ref2 = s_f[0];
#pragma unroll
    for (int k = 1; k < kWaves; ++k)
        ref2 = fmaxf(ref2, s_f[k]);
    __syncthreads();
    w = wave_sum(st.s * fast_exp2(st.ref2 - ref2));
    if ((tid & 63) == 0)
        s_f[tid >> 6] = w;
    __syncthreads();
    if (tid == 0) {
        float s = s_f[0];
#pragma unroll
        for (int k = 1; k < kWaves; ++k)
            s += s_f[k];
        if (n_seg > 1) {
            records[row64 * n_seg + seg] = SegmentRecord{z, idx, ref2, s};
        } else {
            tokens_out[row64] = idx;
            if (logp_out)
                logp_out[row64] = load_scalar<DT>(base, idx) * inv_t - (ref2 + log2f(s)) * kLn2;
        }
    }
}

// One lane per row: the best of the segments' candidates (ties to the lower
// index) and the sum of their exponentials.
template <int DT>
__global__ __launch_bounds__(256) void sample_merge_kernel(
    const void *__restrict__ logits, const SegmentRecord *__restrict__ records, int32_t *__restrict__ tokens_out,
    float *__restrict__ logp_out, int64_t n_rows, int n_seg, int64_t stride, float inv_t)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= n_rows)
        return;
    const SegmentRecord *rec = records + row * n_seg;
    float z = -INFINITY, ref2 = kNoRef * kLog2e;
    int idx = INT_MAX;
    for (int k = 0; k < n_seg; ++k) {
        better(z, idx, rec[k].best_z, rec[k].best_i);
        ref2 = fmaxf(ref2, rec[k].ref2);
    }
    float s = 0.f;
    for (int k = 0; k < n_seg; ++k)
        s += rec[k].s * fast_exp2(rec[k].ref2 - ref2);
    if (idx == INT_MAX)  // nothing but -inf / NaN in the row
        idx = 0;
    tokens_out[row] = idx;
    if (logp_out) {
        constexpr int EB = (DT == RLHF_F32) ? 4 : 2;
        const char *base = (const char *)logits + row * stride * EB;
        logp_out[row] = load_scalar<DT>(base, idx) * inv_t - (ref2 + log2f(s)) * kLn2;
    }
}

// ---- top-k --------------------------------------------------------------------
// Order-preserving key of a logit: unsigned comparison of keys = comparison of
// the values (-0 is folded into +0 first), so thresholds are found exactly, in
// integers, whatever the storage type.
__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t u = __float_as_uint(x + 0.0f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? key ^ 0x80000000u : ~key);
}

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kTopkCap = 4096;  // candidates kept in LDS for the exact part of the search

// Integer wave reductions on the DPP network (no LDS traffic); wave-uniform results.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = max(v, dpp_move_u<kDppQuadXor1>(v));
    v = max(v, dpp_move_u<kDppQuadXor2>(v));
    v = max(v, dpp_move_u<kDppRowHalfMirror>(v));
    v = max(v, dpp_move_u<kDppRowMirror>(v));
    const uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
    const uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
    return max(max(a, b), max(c, d));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    return ~wave_max_u32(~v);
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    v += dpp_move_u<kDppQuadXor1>(v);
    v += dpp_move_u<kDppQuadXor2>(v);
    v += dpp_move_u<kDppRowHalfMirror>(v);
    v += dpp_move_u<kDppRowMirror>(v);
    const uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
    const uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
    return (a + b) + (c + d);
}

// Hands the entries of a row that this lane owns to f(x, cnt, v0): cnt
// consecutive entries x[0..cnt) starting at index v0 (a whole 16-byte vector,
// or one entry).  Loads go out U at a time before the first is used: a row is a
// few loads per lane, and their latency, not their number, is what a pass costs.
// The vectors land in the caller's u[]: a row of at most U * 1024 vectors (every
// vocabulary the paper's models have) is one such batch, so after the first pass
// it sits in registers, and a later pass with `reuse` set reads nothing at all.
template <int DT, bool VEC, int U, class F>
__device__ __forceinline__ void row_foreach(const char *base, int vocab, int tid, uint4 (&u)[U], bool reuse,
                                            F &&f)
{
    if constexpr (VEC) {
        constexpr int E = (DT == RLHF_F32) ? 4 : 8;
        const int nvec = vocab / E;
        const uint4 *p = (const uint4 *)base;
        const bool keep = reuse && nvec <= U * kTopkThreads;  // u[] still holds the whole row
        for (int i0 = tid; i0 < nvec; i0 += U * kTopkThreads) {
            if (!keep) {  // ordinary loads: a row too long for the registers is read again from L2
#pragma unroll
                for (int j = 0; j < U; ++j)
                    if (i0 + j * kTopkThreads < nvec)
                        u[j] = p[i0 + j * kTopkThreads];
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int i = i0 + j * kTopkThreads;
                if (i < nvec) {
                    float x[E];
                    if constexpr (DT == RLHF_F32) {
                        x[0] = __uint_as_float(u[j].x);
                        x[1] = __uint_as_float(u[j].y);
                        x[2] = __uint_as_float(u[j].z);
                        x[3] = __uint_as_float(u[j].w);
                    } else {
                        x[0] = unpack_lo<DT>(u[j].x);
                        x[1] = unpack_hi<DT>(u[j].x);
                        x[2] = unpack_lo<DT>(u[j].y);
                        x[3] = unpack_hi<DT>(u[j].y);
                        x[4] = unpack_lo<DT>(u[j].z);
                        x[5] = unpack_hi<DT>(u[j].z);
                        x[6] = unpack_lo<DT>(u[j].w);
                        x[7] = unpack_hi<DT>(u[j].w);
                    }
                    f(x, E, E * i);
                }
            }
        }
        const int done = nvec * E;
        if (tid < vocab - done) {
            const float x = load_scalar<DT>(base, done + tid);
            f(&x, 1, done + tid);
        }
    } else {
        for (int v0 = tid; v0 < vocab; v0 += U * kTopkThreads) {
            float x[U];
#pragma unroll
            for (int j = 0; j < U; ++j)
                if (v0 + j * kTopkThreads < vocab)
                    x[j] = load_scalar<DT>(base, v0 + j * kTopkThreads);
#pragma unroll
            for (int j = 0; j < U; ++j)
                if (v0 + j * kTopkThreads < vocab)
                    f(&x[j], 1, v0 + j * kTopkThreads);
        }
    }
}

// Top-k draw, one workgroup of 1024 lanes per row.  The survivors are the
// entries at or above tau, the k-th largest logit; they are found exactly, on
// the order keys (their upper half for bf16, whose lower half carries nothing),
// as a bracket [lo, hi) with count(>= lo) >= k > count(>= hi) that is narrowed
// until count(>= lo) = k (no tie at the k-th value: the entries at or above lo
// are the survivors) or the bracket is one key wide (lo = tau).
//   k <= 1024: the first pass leaves every lane's maximum; a threshold that
//     about k of those 1024 maxima reach is a lower bound of tau with little
//     more than k entries of the row at or above it, so the second pass (the row
//     is in L2 now) already collects the candidates into LDS, and the rest (the
//     bracket, then the draw) runs on that list.
//   larger k: the lower bound comes from stepping down from the row maximum in
//     doubling steps, one pass per step.
//   If more than kTopkCap entries lie at or above lo (large k, or a k-th value
//     tied thousands of times), the bracket is bisected on the row until the
//     candidates fit or the bracket is one key wide; in the second case the
//     draw scans the row.
// Searches on LDS data test sixteen thresholds per round, one per wavefront, on
// keys held in registers.  Passes over the row compare values, not keys (the
// same order for numbers; NaN entries compare false and never survive).  Each
// sweep and search appears once in the code (the control flow is arranged around
// that): the kernel has to stay well inside the instruction cache.
template <int DT, bool VEC, bool NOISE>
__global__ __launch_bounds__(kTopkThreads) void sample_topk_kernel(
    const void *__restrict__ logits, int32_t *__restrict__ tokens_out, float *__restrict__ logp_out,
    int64_t n_rows, int vocab, int64_t stride, int top_k, float inv_t, uint2 key, uint2 off)
{
    __shared__ uint32_t s_key[kTopkCap];
    __shared__ int s_idx[kTopkCap];
    __shared__ uint32_t s_max[kTopkThreads];  // the lanes' maxima: apart from the list, which a fast
                                              // wavefront may start to fill while a slow one still reads these
    __shared__ uint32_t s_top[kTopkWaves], s_low[kTopkWaves], s_cnt[2][kTopkWaves], s_i[kTopkWaves];
    __shared__ float s_f[kTopkWaves], s_r[kTopkWaves], s_s[kTopkWaves], s_y[kTopkWaves];
    __shared__ int s_fill[3];  // the sweeps' candidate counters, one per round in rotation
    const int64_t row64 = (int64_t)blockIdx.y * kRowSlab + blockIdx.x;
    if (row64 >= n_rows)  // the last slab of a grid of more than kRowSlab rows
        return;
    const uint32_t row = (uint32_t)row64;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    constexpr int EB = (DT == RLHF_F32) ? 4 : 2;
    constexpr int SHIFT = (DT == RLHF_BF16) ? 16 : 0;  // a bf16 value's key is constant in its lower half
    const char *base = (const char *)logits + row64 * stride * EB;
    auto skey = [](float x) -> uint32_t { return order_key(x) >> SHIFT; };
    auto skey_value = [](uint32_t sk) -> float {
        uint32_t full = sk << SHIFT;
        if (SHIFT && !(full & 0x80000000u))  // negative value: the dropped half of its key was all ones
            full |= (1u << SHIFT) - 1u;
        return key_value(full);
    };
    const uint32_t key_ninf = skey(-INFINITY);
    // value v with: x >= v  <=>  skey(x) >= t, for every number x
    auto threshold_value = [&](uint32_t t) -> float { return t <= key_ninf ? -INFINITY : skey_value(t); };

    // pass 1: every lane's own maximum (-inf for a lane without entries), the row's, and the least of the lanes'
    const uint32_t k = (uint32_t)min(top_k, vocab);
    const int owners = VEC ? min(kTopkThreads, vocab / (16 / EB)) : min(kTopkThreads, vocab);  // lanes 0 .. owners-1 have entries
    float mine_f = -INFINITY;
    uint4 rowv[16];  // the lane's vectors of the row, kept for the sweeps when the row fits
    row_foreach<DT, VEC, 16>(base, vocab, tid, rowv, false, [&](const float *x, int cnt, int) {
#pragma unroll
        for (int j = 0; j < cnt; ++j)
            mine_f = fmaxf(mine_f, x[j]);
    });
    const uint32_t mine = skey(mine_f);
    s_max[tid] = mine;
    if (tid < 2)
        s_fill[tid] = 0;  // rounds 0 and 1; every round clears the counter of the round after it
    {
        const uint32_t hi_w = wave_max_u32(mine), lo_w = wave_min_u32(tid < owners ? mine : 0xffffffffu);
        if (lane == 0) {
            s_top[wv] = hi_w;
            s_low[wv] = lo_w;
        }
    }
    __syncthreads();
    uint32_t top = 0, low = 0xffffffffu;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
        top = max(top, s_top[w]);
        low = min(low, s_low[w]);
    }
    top = min(top, skey(INFINITY));  // fmaxf skips NaN entries, so this only guards top + 1

    // count(>= lo) >= k: `owners` lane maxima reach `low`; otherwise every number reaches key_ninf
    uint32_t lo = ((uint32_t)owners >= k && low <= top) ? low : min(key_ninf, top), hi = top + 1;
    // Lane maxima at or above a threshold undercount the row's entries there, the
    // more so the closer their number is to all 1024: no slack then.
    uint32_t c_lo = kTopkThreads, slack = min(max(k >> 3, 16u), k < 896u ? 896u - k : 0u);
    int n_list = kTopkThreads;
    bool listed = true;
    const bool count_only = k > (uint32_t)kTopkCap;  // the candidates can never fit the list
    // phase 0 (k <= 1024 only): the search runs on the lane maxima and leaves in
    // lo a threshold that k to k + slack of them reach; phase 1: sweeps of the
    // row until the candidates are in the list, then the search runs on the list.
    for (int phase = (k <= (uint32_t)kTopkThreads) ? 0 : 1; phase < 2; ++phase) {
        if (phase == 1) {
            bool stepping = k > (uint32_t)kTopkThreads;  // no lower bound yet
            float step = 1.0f;
            const float vmax = skey_value(top);
            uint32_t t = stepping ? min(skey(vmax - step), top) : lo;
            listed = false;
            // Ends: stepping reaches -inf (every number counts) within 130
            // doublings and is cut off at 140 rounds; bisection halves the bracket
            // every round.
            for (int round = 0;; ++round) {
                // one sweep: count the entries at or above t, keep the first kTopkCap of them.
                // This round's counter was cleared two barriers ago; the next round's is
                // cleared now (its last readers passed the barrier that ended the round
                // before this one), so a round costs one barrier.
                int *const fill = &s_fill[round % 3];
                if (tid == 0)
                    s_fill[(round + 1) % 3] = 0;
                const float tv = threshold_value(t);
                uint32_t local = 0;
                row_foreach<DT, VEC, 16>(base, vocab, tid, rowv, true, [&](const float *x, int cnt, int v0) {
                    if (count_only) {
#pragma unroll
                        for (int j = 0; j < cnt; ++j)
                            local += x[j] >= tv;
                        return;
                    }
                    float m = x[0];
#pragma unroll
                    for (int j = 1; j < cnt; ++j)
                        m = fmaxf(m, x[j]);
                    if (__ballot(m >= tv) == 0)  // nearly always: candidates are few
                        return;
                    uint32_t mask = 0;
#pragma unroll
                    for (int j = 0; j < cnt; ++j)
                        mask |= (uint32_t)(x[j] >= tv) << j;
                    // One counter update per wavefront and vector: the lanes' candidate
                    // counts (at most 8 each) are summed and prefix-summed bit by bit with
                    // ballots, and the first active lane claims the slots for all.
                    const uint32_t n = (uint32_t)__popc(mask);
                    uint32_t before = 0, total = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const uint64_t bal = __ballot((n >> b) & 1u);
                        before += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u)) << b;
                        total += (uint32_t)__popcll(bal) << b;
                    }
                    const uint64_t active = __ballot(true);
                    int first = 0;
                    if (__builtin_amdgcn_mbcnt_hi((uint32_t)(active >> 32),
                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)active, 0u)) == 0)
                        first = atomicAdd(fill, (int)total);
                    int at = __builtin_amdgcn_readfirstlane(first) + (int)before;
                    while (mask) {
                        const int e = __ffs(mask) - 1;
                        mask &= mask - 1;
                        float sel = x[0];
#pragma unroll
                        for (int j = 1; j < cnt; ++j)
                            sel = (e == j) ? x[j] : sel;
                        if (at < kTopkCap) {
                            s_key[at] = skey(sel);
                            s_idx[at] = v0 + e;
                        }
                        ++at;
                    }
                });
                if (count_only) {
                    local = wave_sum_u32(local);
                    if (lane == 0)
                        atomicAdd(fill, (int)local);
                }
                __syncthreads();
                const uint32_t c = (uint32_t)*fill;
                if (c >= k) {
                    lo = t;
                    c_lo = c;
                    stepping = false;
                    if (c <= (uint32_t)kTopkCap) {
                        listed = true;
                        n_list = (int)c;
                        break;
                    }
                } else {
                    hi = t;
                }
                if (hi <= key_ninf) {  // fewer than k numbers in the row (the rest is NaN): all of them survive
                    lo = 0;
                    break;
                }
                if (stepping && round < 140) {
                    step *= 2.0f;
                    t = skey(vmax - step);
                    if (t >= hi)  // the step vanished in rounding (huge |vmax|): go down one key
                        t = hi - 1;
                } else if (stepping) {  // a row of infinities: count every number once, then bisect
                    stepping = false;
                    lo = 0;
                    t = key_ninf;
                } else {
                    if (hi - lo <= 1)
                        break;
                    t = lo + (hi - lo) / 2;
                }
            }
            if (!listed)
                break;
            slack = 0;
        }
        // Narrows [lo, hi) on the n_list keys until count(>= lo), kept in c_lo, is
        // within `slack` of k or the bracket is one key wide.  Every wavefront holds
        // the first 1024 keys in registers (sixteen per lane).  Up to 1024 keys, each
        // wavefront runs the whole bisection on its own: a probe is sixteen compares
        // and scalar population counts, so the search needs no LDS traffic and no
        // barrier, and all wavefronts arrive at the same bracket.
        const uint32_t *keys = phase == 0 ? s_max : s_key;
        uint32_t held[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            held[j] = (lane + 64 * j < n_list) ? keys[lane + 64 * j] : 0u;  // thresholds are above lo >= 0
        if (n_list <= kTopkThreads) {
            while (hi - lo > 1 && c_lo > k + slack) {
                const uint32_t t = lo + (hi - lo) / 2;  // strictly inside the bracket
                uint32_t c = 0;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    c += (uint32_t)__popcll(__ballot(held[j] >= t));
                if (c >= k) {
                    lo = t;
                    c_lo = c;
                } else {
                    hi = t;
                }
            }
        } else {
            // A list of more than 1024 keys (k near or above 1024): the part beyond the
            // registers is read from LDS at every probe, so the wavefronts share the
            // work instead -- wavefront w counts the keys at or above a threshold of its
            // own, the bracket cut in seventeen; the first wavefront's threshold lies
            // strictly inside the bracket whenever it is two keys wide or more, so every
            // round shrinks it.  A round's counts go to the half of s_cnt the previous
            // round did not use: one barrier per round.
            int parity = 0;
            while (hi - lo > 1 && c_lo > k + slack) {
                const uint32_t span = hi - lo, part = span / (kTopkWaves + 1), rest = span - part * (kTopkWaves + 1);
                const uint32_t my_t = lo + part * (uint32_t)(wv + 1) + min((uint32_t)(wv + 1), rest);
                uint32_t c = 0;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    c += (uint32_t)__popcll(__ballot(held[j] >= my_t));
                for (int i = 1024 + lane; i < n_list; i += 64)
                    c += (uint32_t)__popcll(__ballot(s_key[i] >= my_t));  // complete in lane 0, which goes round longest
                if (lane == 0)
                    s_cnt[parity][wv] = c;
                __syncthreads();
                uint32_t nlo = lo, nhi = hi, nc = c_lo;
#pragma unroll
                for (int w = 0; w < kTopkWaves; ++w) {  // thresholds rise with w, counts fall
                    const uint32_t tw = lo + part * (uint32_t)(w + 1) + min((uint32_t)(w + 1), rest);
                    const uint32_t cw = s_cnt[parity][w];
                    if (cw >= k) {
                        nlo = tw;
                        nc = cw;
                    } else {
                        nhi = min(nhi, tw);
                    }
                }
                lo = nlo;
                hi = nhi;
                c_lo = nc;
                parity ^= 1;
            }
        }
        if (phase == 0)
            hi = top + 1;  // lo bounds tau from below; the row's bracket is open above again
    }
    const uint32_t tau = lo;  // the survivors are the entries at or above it

    // the draw over the survivors
    Lane st;
    if (listed) {
        for (int i = tid; i < n_list; i += kTopkThreads)
            if (s_key[i] >= tau)
                take1<NOISE>(st, skey_value(s_key[i]) * inv_t, s_idx[i], row, off, key);
    } else {
        // survivors are many: the plain draw's sweep, removed entries at -inf
        // (no weight in the sum, never the maximum)
        const float tv = threshold_value(tau);
        uint4 one[1];
        row_foreach<DT, VEC, 1>(base, vocab, tid, one, false, [&](const float *x, int cnt, int v0) {
            if (cnt == 1) {
                if (x[0] >= tv)
                    take1<NOISE>(st, x[0] * inv_t, v0, row, off, key);
            } else {
#pragma unroll
                for (int q = 0; q < cnt; q += 4) {
                    float y[4];
                    bool any = false;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bool in = x[q + j] >= tv;
                        y[j] = in ? x[q + j] * inv_t : -INFINITY;
                        any |= in;
                    }
                    if (any)
                        take4<NOISE>(st, y, v0 + q, row, off, key);
                }
            }
        });
    }
    // best score (ties to the lowest index), then the sum over the survivors.  Each
    // wavefront fetches the logit of its own best entry before the barrier, so that
    // the load's latency is not paid once more after the workgroup's winner is known.
    const float zw = wave_max(st.best_z);
    const uint32_t iw = wave_min_u32(st.best_z == zw ? (uint32_t)st.best_i : (uint32_t)INT_MAX);
    const float rw = wave_max(st.ref2);
    const float sw = wave_sum(st.s * fast_exp2(st.ref2 - rw));
    if (lane == 0) {
        s_f[wv] = zw;
        s_i[wv] = iw;
        s_r[wv] = rw;
        s_s[wv] = sw;
        s_y[wv] = (logp_out && iw != (uint32_t)INT_MAX) ? load_scalar<DT>(base, (int)iw) : 0.f;
    }
    __syncthreads();
    if (tid == 0) {
        float z = s_f[0];
        int idx = (int)s_i[0];
        float ref2 = s_r[0];
#pragma unroll
        for (int w = 1; w < kTopkWaves; ++w) {
            better(z, idx, s_f[w], (int)s_i[w]);
            ref2 = fmaxf(ref2, s_r[w]);
        }
        float sum = 0.f, y = 0.f;
        bool have = false;
#pragma unroll
        for (int w = 0; w < kTopkWaves; ++w) {
            sum += s_s[w] * fast_exp2(s_r[w] - ref2);
            if (idx != INT_MAX && (int)s_i[w] == idx) {  // the wavefront that proposed the winner holds its logit
                y = s_y[w];
                have = true;
            }
        }
        if (idx == INT_MAX)
            idx = 0;
        tokens_out[row64] = idx;
        if (logp_out) {
            if (!have)  // no entry was drawn from (a row without numbers): token 0
                y = load_scalar<DT>(base, idx);
            logp_out[row64] = y * inv_t - (ref2 + log2f(sum)) * kLn2;
        }
    }
}

template <int DT>
int launch_topk(const void *logits, int32_t *tokens, float *logp, int64_t n, int vocab, int64_t stride, bool vec,
                float temperature, int top_k, uint64_t seed, uint64_t offset, hipStream_t s)
{
    const uint2 key = make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
    const uint2 off = make_uint2((uint32_t)offset, (uint32_t)(offset >> 32));
    const bool noise = temperature > 0.f;
    const float inv_t = noise ? 1.0f / temperature : 1.0f;
    const dim3 grid = row_grid(n), block(kTopkThreads);
#define RLHF_TOPK_LAUNCH(V, N)                                                                          \
    hipLaunchKernelGGL((sample_topk_kernel<DT, V, N>), grid, block, 0, s, logits, tokens, logp, n, vocab, \
                       stride, top_k, inv_t, key, off)
    if (vec && noise)
        RLHF_TOPK_LAUNCH(true, true);
    else if (vec)
        RLHF_TOPK_LAUNCH(true, false);
    else if (noise)
        RLHF_TOPK_LAUNCH(false, true);
    else
        RLHF_TOPK_LAUNCH(false, false);
#undef RLHF_TOPK_LAUNCH
    RLHF_LAUNCH_CHECK("sample_topk_kernel");
    return RLHF_OK;
}

// Segments per row: enough workgroups of 1024 lanes for two per compute unit,
// at most kMaxSegments, none shorter than 8192 entries; 1 without a workspace.
constexpr int kMaxSegments = 8;
constexpr int kTargetGroups = 512;

int segments(int64_t n_rows, int vocab, bool have_workspace)
{
    if (!have_workspace || n_rows <= 0 || n_rows >= kTargetGroups)
        return 1;
    const int64_t want = (kTargetGroups + n_rows - 1) / n_rows;
    const int64_t fit = std::max<int64_t>(vocab / 8192, 1);
    return (int)std::min<int64_t>(std::min<int64_t>(want, fit), kMaxSegments);
}

template <int DT>
int launch(const void *logits, int32_t *tokens, float *logp, int64_t n, int vocab, int64_t stride, bool vec,
           float temperature, uint64_t seed, uint64_t offset, void *workspace, hipStream_t s)
{
    const int n_seg = segments(n, vocab, workspace != nullptr);
    SegmentRecord *records = (SegmentRecord *)workspace;
    const dim3 grid = row_grid(n, (unsigned)n_seg);
    const uint2 key = make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
    const uint2 off = make_uint2((uint32_t)offset, (uint32_t)(offset >> 32));
    const bool noise = temperature > 0.f;
    const bool wide = n < kFewRows;
    const float inv_t = noise ? 1.0f / temperature : 1.0f;
    const bool lse = logp != nullptr;  // the sum of exponentials is only needed for the log-probability
#define RLHF_SAMPLE_LAUNCH(V, N, T)                                                                            \
    do {                                                                                                       \
        if (lse)                                                                                               \
            hipLaunchKernelGGL((sample_tokens_kernel<DT, V, N, true, T>), grid, dim3(T), 0, s, logits, tokens, \
                               logp, records, n, vocab, stride, inv_t, key, off);                              \
        else                                                                                                   \
            hipLaunchKernelGGL((sample_tokens_kernel<DT, V, N, false, T>), grid, dim3(T), 0, s, logits, tokens, \
                               logp, records, n, vocab, stride, inv_t, key, off);                              \
    } while (0)
#define RLHF_SAMPLE_PICK(V, N)          \
    do {                                \
        if (wide)                       \
            RLHF_SAMPLE_LAUNCH(V, N, 1024); \
        else                            \
            RLHF_SAMPLE_LAUNCH(V, N, 256);  \
    } while (0)
    if (vec && noise)
        RLHF_SAMPLE_PICK(true, true);
    else if (vec)
        RLHF_SAMPLE_PICK(true, false);
    else if (noise)
        RLHF_SAMPLE_PICK(false, true);
    else
        RLHF_SAMPLE_PICK(false, false);
#undef RLHF_SAMPLE_PICK
#undef RLHF_SAMPLE_LAUNCH
    RLHF_LAUNCH_CHECK("sample_tokens_kernel");
    if (n_seg > 1) {
        hipLaunchKernelGGL((sample_merge_kernel<DT>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, logits,
                           records, tokens, logp, n, n_seg, stride, inv_t);
        RLHF_LAUNCH_CHECK("sample_merge_kernel");
    }
    return RLHF_OK;
}

}  // namespace
}  // namespace rlhf

static int sample_tokens_impl(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                              int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype, float temperature,
                              uint64_t seed, uint64_t offset, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    using namespace rlhf;
    if (n_rows < 0 || vocab <= 0 || !(temperature >= 0.f))
        return fail(RLHF_ERR_INVALID, "n_rows=%lld vocab=%d temperature=%g", (long long)n_rows, vocab,
                    (double)temperature);
    if (n_rows > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "n_rows above 2^31-1: split the call");
    if (row_stride_elems == 0)
        row_stride_elems = vocab;
    if (row_stride_elems < vocab)
        return fail(RLHF_ERR_INVALID, "row stride %lld below vocab %d", (long long)row_stride_elems, vocab);
    if (logits_dtype != RLHF_F16 && logits_dtype != RLHF_BF16 && logits_dtype != RLHF_F32)
        return fail(RLHF_ERR_UNSUPPORTED, "logits dtype %d", logits_dtype);
    if (n_rows == 0)
        return RLHF_OK;
    if (!logits || !tokens_out)
        return fail(RLHF_ERR_INVALID, "NULL pointer");
    const int eb = elem_bytes(logits_dtype);
    if ((uintptr_t)logits % eb)
        return fail(RLHF_ERR_INVALID, "logits not aligned to their element size");
    if (workspace) {
        const size_t need = (size_t)n_rows * segments(n_rows, vocab, true) * sizeof(SegmentRecord);
        if ((uintptr_t)workspace % 16)
            return fail(RLHF_ERR_INVALID, "workspace must be 16-byte aligned");
        if (workspace_bytes < need)
            return fail(RLHF_ERR_INVALID, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    }
    const bool vec = ((uintptr_t)logits % 16 == 0) && ((row_stride_elems * eb) % 16 == 0);
    hipStream_t s = (hipStream_t)stream;
    switch (logits_dtype) {
    case RLHF_F16:
        return launch<RLHF_F16>(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, vec, temperature,
                                seed, offset, workspace, s);
    case RLHF_BF16:
        return launch<RLHF_BF16>(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, vec,
                                 temperature, seed, offset, workspace, s);
    default:
        return launch<RLHF_F32>(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, vec, temperature,
                                seed, offset, workspace, s);
    }
}

extern "C" int rlhf_sample_tokens(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                                  int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype,
                                  float temperature, uint64_t seed, uint64_t offset, void *stream)
{
    return sample_tokens_impl(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, logits_dtype,
                              temperature, seed, offset, nullptr, 0, stream);
}

extern "C" int rlhf_sample_tokens_workspace_bytes(int64_t n_rows, int32_t vocab, size_t *out_bytes)
{
    using namespace rlhf;
    if (!out_bytes)
        return fail(RLHF_ERR_INVALID, "NULL out_bytes");
    if (n_rows < 0 || vocab <= 0)
        return fail(RLHF_ERR_INVALID, "n_rows=%lld vocab=%d", (long long)n_rows, vocab);
    // at least one record, so that a caller can always allocate what is asked for
    *out_bytes = (size_t)std::max<int64_t>(n_rows, 1) * segments(n_rows, vocab, true) * sizeof(SegmentRecord);
    return RLHF_OK;
}

extern "C" int rlhf_sample_tokens_split(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                                        int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype,
                                        float temperature, uint64_t seed, uint64_t offset, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    if (!workspace)
        return rlhf::fail(RLHF_ERR_INVALID, "NULL workspace");
    return sample_tokens_impl(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, logits_dtype,
                              temperature, seed, offset, workspace, workspace_bytes, stream);
}

extern "C" int rlhf_sample_tokens_topk(const void *logits, int32_t *tokens_out, float *logp_out, int64_t n_rows,
                                       int32_t vocab, int64_t row_stride_elems, int32_t logits_dtype,
                                       float temperature, int32_t top_k, uint64_t seed, uint64_t offset,
                                       void *stream)
{
    using namespace rlhf;
    if (top_k < 1)
        return fail(RLHF_ERR_INVALID, "top_k %d (at least 1)", top_k);
    if (vocab > 0 && top_k >= vocab)  // nothing is removed: the plain draw
        return sample_tokens_impl(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, logits_dtype,
                                  temperature, seed, offset, nullptr, 0, stream);
    if (n_rows < 0 || vocab <= 0 || !(temperature >= 0.f))
        return fail(RLHF_ERR_INVALID, "n_rows=%lld vocab=%d temperature=%g", (long long)n_rows, vocab,
                    (double)temperature);
    if (n_rows > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "n_rows above 2^31-1: split the call");
    if (row_stride_elems == 0)
        row_stride_elems = vocab;
    if (row_stride_elems < vocab)
        return fail(RLHF_ERR_INVALID, "row stride %lld below vocab %d", (long long)row_stride_elems, vocab);
    if (logits_dtype != RLHF_F16 && logits_dtype != RLHF_BF16 && logits_dtype != RLHF_F32)
        return fail(RLHF_ERR_UNSUPPORTED, "logits dtype %d", logits_dtype);
    if (n_rows == 0)
        return RLHF_OK;
    if (!logits || !tokens_out)
        return fail(RLHF_ERR_INVALID, "NULL pointer");
    const int eb = elem_bytes(logits_dtype);
    if ((uintptr_t)logits % eb)
        return fail(RLHF_ERR_INVALID, "logits not aligned to their element size");
    const bool vec = ((uintptr_t)logits % 16 == 0) && ((row_stride_elems * eb) % 16 == 0);
    hipStream_t s = (hipStream_t)stream;
    switch (logits_dtype) {
    case RLHF_F16:
        return launch_topk<RLHF_F16>(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, vec,
                                     temperature, top_k, seed, offset, s);
    case RLHF_BF16:
        return launch_topk<RLHF_BF16>(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, vec,
                                      temperature, top_k, seed, offset, s);
    default:
        return launch_topk<RLHF_F32>(logits, tokens_out, logp_out, n_rows, vocab, row_stride_elems, vec,
                                     temperature, top_k, seed, offset, s);
    }
}
