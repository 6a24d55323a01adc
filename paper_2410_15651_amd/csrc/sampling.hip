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
        const uint32_t hi0 = __umulhi(M0, c.x), lo0 = M0 * c.x;
        const uint32_t hi1 = __umulhi(M1, c.z), lo1 = M1 * c.z;
        c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
        k.x += 0x9E3779B9u;
        k.y += 0xBB67AE85u;
    }
    return c;
}

// Gumbel noise from one 32-bit word.
__device__ __forceinline__ float gumbel(uint32_t word)
{
    const float u = ((float)(word >> 9) + 0.5f) * (1.0f / 8388608.0f);  // in (0,1), exact
    // e = -ln u is Exp(1).  Near u = 1 it is taken from the series of -ln(1 - c),
    // c = 1 - u (exact), because a hardware log loses relative accuracy there.
    const float c = 1.0f - u;
    const float series = c * (1.0f + c * (0.5f + c * (1.0f / 3.0f + c * 0.25f)));
    const float e = c < 0.015625f ? series : -__logf(u);
    return -__logf(e);
}

struct Lane {
    float best_z = -INFINITY;
    int best_i = INT_MAX;
    float ref2 = kNoRef * kLog2e;  // reference exponent of the running sum, log2 units
    float lift = kNoRef + kLift;
    float s = 0.f;                 // sum 2^(y*log2e - ref2), y = a / T
};

template <bool NOISE>
__device__ __forceinline__ void take(Lane &st, float y, float g, int v)
{
    const float z = NOISE ? y + g : y;
    if (z > st.best_z) {  // strict: a lane sees its indices in increasing order
        st.best_z = z;
        st.best_i = v;
    }
    if (y > st.lift) {
        const float ref2 = y * kLog2e;
        st.s *= fast_exp2(st.ref2 - ref2);
        st.ref2 = ref2;
        st.lift = y + kLift;
    }
    st.s += fast_exp2(fmaf(y, kLog2e, -st.ref2));
}

// Four consecutive entries starting at a multiple of four: one Philox block.
template <bool NOISE>
__device__ __forceinline__ void take4(Lane &st, const float (&y)[4], int v0, uint32_t row, uint2 off, uint2 key)
{
    uint4 r = make_uint4(0, 0, 0, 0);
    if (NOISE)
        r = philox4x32_10(make_uint4((uint32_t)(v0 >> 2), row, off.x, off.y), key);
    take<NOISE>(st, y[0], NOISE ? gumbel(r.x) : 0.f, v0);
    take<NOISE>(st, y[1], NOISE ? gumbel(r.y) : 0.f, v0 + 1);
    take<NOISE>(st, y[2], NOISE ? gumbel(r.z) : 0.f, v0 + 2);
    take<NOISE>(st, y[3], NOISE ? gumbel(r.w) : 0.f, v0 + 3);
}

template <bool NOISE>
__device__ __forceinline__ void take1(Lane &st, float y, int v, uint32_t row, uint2 off, uint2 key)
{
    float g = 0.f;
    if (NOISE) {
        const uint4 r = philox4x32_10(make_uint4((uint32_t)(v >> 2), row, off.x, off.y), key);
        const uint32_t word = (v & 3) == 0 ? r.x : (v & 3) == 1 ? r.y : (v & 3) == 2 ? r.z : r.w;
        g = gumbel(word);
    }
    take<NOISE>(st, y, g, v);
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

// Workgroup (x, y) takes segment y of gridDim.y of row x.  With one segment it
// writes the row's results; with more it writes its record to `records`
// [row][segment].
template <int DT, bool VEC, bool NOISE, int kThreads>
__global__ __launch_bounds__(kThreads) void sample_tokens_kernel(
    const void *__restrict__ logits, int32_t *__restrict__ tokens_out, float *__restrict__ logp_out,
    SegmentRecord *__restrict__ records, int vocab, int64_t stride, float inv_t, uint2 key, uint2 off)
{
    constexpr int kWaves = kThreads / 64;
    __shared__ float s_f[kWaves];
    __shared__ int s_i[kWaves];
    const int64_t row64 = blockIdx.x;
    const uint32_t row = (uint32_t)row64;
    const int seg = blockIdx.y, n_seg = gridDim.y;
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
                take4<NOISE>(st, y, i * 4, row, off, key);
            } else {
                const float y0[4] = {unpack_lo<DT>(u.x) * inv_t, unpack_hi<DT>(u.x) * inv_t,
                                     unpack_lo<DT>(u.y) * inv_t, unpack_hi<DT>(u.y) * inv_t};
                const float y1[4] = {unpack_lo<DT>(u.z) * inv_t, unpack_hi<DT>(u.z) * inv_t,
                                     unpack_lo<DT>(u.w) * inv_t, unpack_hi<DT>(u.w) * inv_t};
                take4<NOISE>(st, y0, i * 8, row, off, key);
                take4<NOISE>(st, y1, i * 8 + 4, row, off, key);
            }
        }
        const int done = nvec * E;
        if (seg == n_seg - 1 && tid < vocab - done)
            take1<NOISE>(st, load_scalar<DT>(base, done + tid) * inv_t, done + tid, row, off, key);
    } else {
        const int v_begin = (int)((int64_t)vocab * seg / n_seg), v_end = (int)((int64_t)vocab * (seg + 1) / n_seg);
        for (int v = v_begin + tid; v < v_end; v += kThreads)
            take1<NOISE>(st, load_scalar<DT>(base, v) * inv_t, v, row, off, key);
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
    const dim3 grid((unsigned)n, (unsigned)n_seg);
    const uint2 key = make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
    const uint2 off = make_uint2((uint32_t)offset, (uint32_t)(offset >> 32));
    const bool noise = temperature > 0.f;
    const bool wide = n < kFewRows;
    const float inv_t = noise ? 1.0f / temperature : 1.0f;
#define RLHF_SAMPLE_LAUNCH(V, N, T)                                                                       \
    hipLaunchKernelGGL((sample_tokens_kernel<DT, V, N, T>), grid, dim3(T), 0, s, logits, tokens, logp, records, \
                       vocab, stride, inv_t, key, off)
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
