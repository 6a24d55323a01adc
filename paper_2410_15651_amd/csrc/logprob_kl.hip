// Fused token log-probability and actor-vs-reference KL over the vocabulary.
//
// The paper's PPO stage (Section 2.1) scores every generated position with the
// actor and the reference model; what the trainer needs from the two logit rows
// of a position is the actor's log-probability of the sampled token and the
// divergence of the actor's distribution from the reference's.  Both follow
// from five running sums over the row, so each logit is read from HBM exactly
// once:
//
//   S_a = sum_v 2^(a_v*log2e - M_a)      S_r = sum_v 2^(r_v*log2e - M_r)
//   T   = sum_v 2^(a_v*log2e - M_a) * (a_v - r_v)
//   lse_a = (M_a + log2 S_a) ln2,  lse_r likewise
//   logp  = a_tok - lse_a
//   KL    = T / S_a + (lse_r - lse_a)      ( = sum_v p_v (log p_v - log q_v) )
//
// One workgroup of 256 lanes owns one row.  Each lane keeps its own reference
// exponent M and moves it only when a later logit exceeds it by more than
// kLift, so the usual per-element running-max update of an online softmax
// becomes one compare per 16-byte load; sums may grow to 2^58 relative to the
// reference, which fp32 holds without loss of relative precision.  Lanes are
// merged at the end of the row with DPP row reductions and one LDS exchange
// between the four wavefronts.
//
// The kernel is bound by HBM reads for fp32 logits and sits close to the
// vector-ALU limit for 16-bit logits (two v_exp_f32 per actor/reference pair),
// hence the care about instruction count per element.
#include <hip/hip_runtime.h>

#include "common.h"
#include "device_ops.h"

namespace rlhf {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 4;
// A lane re-bases its sums when a logit exceeds its reference by this much
// (natural-log units): terms stay below 2^(40*log2e) ~ 2^57.7.
constexpr float kLift = 40.0f;
constexpr float kNoRef = -1.0e30f;  // "no element seen yet"

template <int DT>
struct Logit {
    static constexpr int kPerVec = (DT == RLHF_F32) ? 4 : 8;
};

template <int DT>
__device__ __forceinline__ void unpack_vec(const uint4 &u, float (&f)[Logit<DT>::kPerVec])
{
    if constexpr (DT == RLHF_F32) {
        f[0] = __uint_as_float(u.x);
        f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z);
        f[3] = __uint_as_float(u.w);
    } else {
        f[0] = unpack_lo<DT>(u.x);
        f[1] = unpack_hi<DT>(u.x);
        f[2] = unpack_lo<DT>(u.y);
        f[3] = unpack_hi<DT>(u.y);
        f[4] = unpack_lo<DT>(u.z);
        f[5] = unpack_hi<DT>(u.z);
        f[6] = unpack_lo<DT>(u.w);
        f[7] = unpack_hi<DT>(u.w);
    }
}

// Per-lane running state of one row.
struct RowSums {
    float a_ref2 = kNoRef * kLog2e;  // actor reference exponent, log2 units
    float a_lift = kNoRef + kLift;   // re-base when an actor logit exceeds this
    float sa = 0.f;                  // sum 2^(a*log2e - a_ref2)
    float t = 0.f;                   // sum 2^(a*log2e - a_ref2) * (a - r)
    float r_ref2 = kNoRef * kLog2e;
    float r_lift = kNoRef + kLift;
    float sr = 0.f;
};

template <int N>
__device__ __forceinline__ void accumulate(RowSums &st, const float (&a)[N], const float (&r)[N])
{
    float ca = a[0], cr = r[0];
#pragma unroll
    for (int i = 1; i < N; ++i) {
        ca = fmaxf(ca, a[i]);
        cr = fmaxf(cr, r[i]);
    }
    if (ca > st.a_lift) {  // rare after the first load of a lane
        const float ref2 = ca * kLog2e;
        const float sc = fast_exp2(st.a_ref2 - ref2);
        st.sa *= sc;
        st.t *= sc;
        st.a_ref2 = ref2;
        st.a_lift = ca + kLift;
    }
    if (cr > st.r_lift) {
        const float ref2 = cr * kLog2e;
        st.sr *= fast_exp2(st.r_ref2 - ref2);
        st.r_ref2 = ref2;
        st.r_lift = cr + kLift;
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const float ea = fast_exp2(fmaf(a[i], kLog2e, -st.a_ref2));
        const float er = fast_exp2(fmaf(r[i], kLog2e, -st.r_ref2));
        // a = -inf gives ea = 0 and a - r = -inf (or NaN when r = -inf too); the
        // clamp turns that product into 0 instead of NaN.  fmaxf drops a NaN operand.
        const float d = fmaxf(a[i] - r[i], -FLT_MAX);
        st.sa += ea;
        st.sr += er;
        st.t = fmaf(ea, d, st.t);
    }
}

// Maxima of two values and sums of three over the workgroup, one barrier each
// (a row's five reductions cost two barriers instead of ten: with a workgroup per
// row nothing is in flight while a row is being finished, so that time is lost
// bandwidth).  Every thread gets the results; the four wavefronts' partial
// results are combined in wavefront order by everybody, so all threads agree.
__device__ __forceinline__ void block_max2(float &a, float &b, float *lds)
{
    const float wa = wave_max(a), wb = wave_max(b);
    if ((threadIdx.x & 63) == 0) {
        lds[threadIdx.x >> 6] = wa;
        lds[kWaves + (threadIdx.x >> 6)] = wb;
    }
    __syncthreads();
    a = lds[0];
    b = lds[kWaves];
#pragma unroll
    for (int k = 1; k < kWaves; ++k) {
        a = fmaxf(a, lds[k]);
        b = fmaxf(b, lds[kWaves + k]);
    }
}

__device__ __forceinline__ void block_sum3(float &a, float &b, float &c, float *lds)
{
    const float wa = wave_sum(a), wb = wave_sum(b), wc = wave_sum(c);
    if ((threadIdx.x & 63) == 0) {
        lds[threadIdx.x >> 6] = wa;
        lds[kWaves + (threadIdx.x >> 6)] = wb;
        lds[2 * kWaves + (threadIdx.x >> 6)] = wc;
    }
    __syncthreads();
    a = lds[0];
    b = lds[kWaves];
    c = lds[2 * kWaves];
#pragma unroll
    for (int k = 1; k < kWaves; ++k) {
        a += lds[k];
        b += lds[kWaves + k];
        c += lds[2 * kWaves + k];
    }
}

// Optional per-token reward shaping done by the lane that writes the row's
// results (all pointers may be null).
struct Shaping {
    float *ref_logp_out;
    float *reward_out;
    const float *terminal;
    float kl_coef;
    int sampled;
    int32_t *token_error_flag;  // set to 1, never cleared here, when a token id is >= vocab
};

// VEC: rows start 16-byte aligned and are read with 128-bit loads; otherwise
// every lane reads single elements.
template <int DT, bool VEC>
__global__ __launch_bounds__(kThreads) void logprob_kl_kernel(
    const void *__restrict__ actor, const void *__restrict__ ref, const int32_t *__restrict__ tokens,
    float *__restrict__ logp_out, float *__restrict__ kl_out, int64_t n_rows, int vocab, int64_t stride,
    Shaping sh)
{
    __shared__ float lds_max[2 * kWaves], lds_sum[3 * kWaves];
    const int64_t row = (int64_t)blockIdx.y * kRowSlab + blockIdx.x;
    if (row >= n_rows)  // the last slab of a grid of more than kRowSlab rows
        return;
    const int tid = threadIdx.x;
    constexpr int E = Logit<DT>::kPerVec;
    constexpr int EB = (DT == RLHF_F32) ? 4 : 2;
    const char *arow = (const char *)actor + row * stride * EB;
    const char *rrow = (const char *)ref + row * stride * EB;

    // The row's first loads go out before anything else is waited for: a workgroup
    // owns one row, so whatever precedes its first load (the token id, its check)
    // is time in which its share of the memory system idles.  A padded row pays
    // for loads it does not use.
    const int nvec = VEC ? vocab / E : 0;
    // Rows whose byte length is not a multiple of 128 start off a 128-byte line
    // every other row; then each wavefront's 1 KB load would straddle nine lines
    // instead of eight.  The vectors before the first line boundary are taken
    // by the first lanes, and the streaming loop starts on the boundary.
    const int head = VEC ? min((int)(((128u - (uint32_t)((uintptr_t)arow & 127u)) & 127u) >> 4), nvec) : 0;
    const uint4 *pa = (const uint4 *)arow;
    const uint4 *pr = (const uint4 *)rrow;
    int i = head + tid;
    uint4 va[kUnroll], vr[kUnroll];
    bool more = VEC && i + (kUnroll - 1) * kThreads < nvec;
    if (more) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            va[u] = load16(pa + i + u * kThreads);
            vr[u] = load16(pr + i + u * kThreads);
        }
    }

    const int tok = tokens[row];
    if (tok < 0 || tok >= vocab) {  // padded position: uniform across the block
        if (tid == 0) {
            if (tok >= vocab && sh.token_error_flag)  // not padding by convention: tell the caller
                *sh.token_error_flag = 1;
            logp_out[row] = 0.f;
            kl_out[row] = 0.f;
            if (sh.ref_logp_out)
                sh.ref_logp_out[row] = 0.f;
            if (sh.reward_out)
                sh.reward_out[row] = 0.f;
        }
        return;
    }

    // the gather of the sampled token's logit, issued before the long stream
    float a_tok = 0.f, r_tok = 0.f, terminal = 0.f;
    if (tid == 0) {
        a_tok = load_scalar<DT>(arow, tok);
        if (sh.ref_logp_out || sh.reward_out)
            r_tok = load_scalar<DT>(rrow, tok);
        if (sh.reward_out && sh.terminal)
            terminal = sh.terminal[row];
    }

    RowSums st;
    if constexpr (VEC) {
        // each batch is loaded while the one before it is still being summed
        while (more) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float fa[E], fr[E];
                unpack_vec<DT>(va[u], fa);
                unpack_vec<DT>(vr[u], fr);
                accumulate<E>(st, fa, fr);
            }
            i += kUnroll * kThreads;
            more = i + (kUnroll - 1) * kThreads < nvec;
            if (more) {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    va[u] = load16(pa + i + u * kThreads);
                    vr[u] = load16(pr + i + u * kThreads);
                }
            }
        }
        for (; i < nvec; i += kThreads) {
            float fa[E], fr[E];
            unpack_vec<DT>(load16(pa + i), fa);
            unpack_vec<DT>(load16(pr + i), fr);
            accumulate<E>(st, fa, fr);
        }
        if (tid < head) {
            float fa[E], fr[E];
            unpack_vec<DT>(load16((const uint4 *)arow + tid), fa);
            unpack_vec<DT>(load16((const uint4 *)rrow + tid), fr);
            accumulate<E>(st, fa, fr);
        }
        const int done = nvec * E;
        if (tid < vocab - done) {
            float fa[1] = {load_scalar<DT>(arow, done + tid)};
            float fr[1] = {load_scalar<DT>(rrow, done + tid)};
            accumulate<1>(st, fa, fr);
        }
    } else {
        for (int j = tid; j < vocab; j += kThreads) {
            float fa[1] = {load_scalar<DT>(arow, j)};
            float fr[1] = {load_scalar<DT>(rrow, j)};
            accumulate<1>(st, fa, fr);
        }
    }

    // Merge the lanes.  Actor and reference go through the same sequence of
    // operations, so identical rows give identical lse values and KL == 0 exactly.
    float a_ref2 = st.a_ref2, r_ref2 = st.r_ref2;
    block_max2(a_ref2, r_ref2, lds_max);
    const float sca = fast_exp2(st.a_ref2 - a_ref2);
    const float scr = fast_exp2(st.r_ref2 - r_ref2);
    float sa = st.sa * sca, sr = st.sr * scr, t = st.t * sca;
    block_sum3(sa, sr, t, lds_sum);
    if (tid == 0) {
        // lse_r - lse_a is formed in log2 units before the single multiply, so
        // that no fused multiply-add can see one side rounded and the other not.
        const float la = log2f(sa), lr = log2f(sr);
        const float lse_a = (a_ref2 + la) * kLn2;
        const float diff2 = (r_ref2 - a_ref2) + (lr - la);
        const float kl = t / sa + diff2 * kLn2;
        logp_out[row] = a_tok - lse_a;
        kl_out[row] = kl;
        if (sh.ref_logp_out)
            sh.ref_logp_out[row] = r_tok - (r_ref2 + lr) * kLn2;
        if (sh.reward_out) {
            // sampled estimate logp_a(tok) - logp_r(tok) = (a_tok - r_tok) + (lse_r - lse_a)
            const float penalty = sh.sampled ? (a_tok - r_tok) + diff2 * kLn2 : kl;
            sh.reward_out[row] = fmaf(-sh.kl_coef, penalty, terminal);
        }
    }
}

template <int DT>
int launch(const void *actor, const void *ref, const int32_t *tokens, float *logp, float *kl,
           int64_t n, int vocab, int64_t stride, bool vec, const Shaping &sh, hipStream_t s)
{
    const dim3 grid = row_grid(n), block(kThreads);
    if (vec)
        hipLaunchKernelGGL((logprob_kl_kernel<DT, true>), grid, block, 0, s, actor, ref, tokens, logp,
                           kl, n, vocab, stride, sh);
    else
        hipLaunchKernelGGL((logprob_kl_kernel<DT, false>), grid, block, 0, s, actor, ref, tokens, logp,
                           kl, n, vocab, stride, sh);
    RLHF_LAUNCH_CHECK("logprob_kl_kernel");
    return RLHF_OK;
}

}  // namespace
}  // namespace rlhf

static int logprobs_kl_impl(const void *actor_logits, const void *ref_logits, const int32_t *tokens,
                            float *logp_out, float *kl_out, int64_t n_positions, int32_t vocab,
                            int64_t row_stride_elems, int32_t logits_dtype, const rlhf::Shaping &sh,
                            void *stream)
{
    using namespace rlhf;
    if (n_positions < 0 || vocab <= 0)
        return fail(RLHF_ERR_INVALID, "n_positions=%lld vocab=%d", (long long)n_positions, vocab);
    if (n_positions > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "n_positions above 2^31-1: split the call");
    if (row_stride_elems == 0)
        row_stride_elems = vocab;
    if (row_stride_elems < vocab)
        return fail(RLHF_ERR_INVALID, "row stride %lld below vocab %d", (long long)row_stride_elems, vocab);
    if (logits_dtype != RLHF_F16 && logits_dtype != RLHF_BF16 && logits_dtype != RLHF_F32)
        return fail(RLHF_ERR_UNSUPPORTED, "logits dtype %d", logits_dtype);
    if (n_positions == 0)
        return RLHF_OK;
    if (!actor_logits || !ref_logits || !tokens || !logp_out || !kl_out)
        return fail(RLHF_ERR_INVALID, "NULL pointer");
    const int eb = elem_bytes(logits_dtype);
    if (((uintptr_t)actor_logits | (uintptr_t)ref_logits) % eb)
        return fail(RLHF_ERR_INVALID, "logits not aligned to their element size");
    const bool vec = ((uintptr_t)actor_logits % 16 == 0) && ((uintptr_t)ref_logits % 16 == 0) &&
                     ((row_stride_elems * eb) % 16 == 0);
    hipStream_t s = (hipStream_t)stream;
    switch (logits_dtype) {
    case RLHF_F16:
        return launch<RLHF_F16>(actor_logits, ref_logits, tokens, logp_out, kl_out, n_positions, vocab,
                                row_stride_elems, vec, sh, s);
    case RLHF_BF16:
        return launch<RLHF_BF16>(actor_logits, ref_logits, tokens, logp_out, kl_out, n_positions, vocab,
                                 row_stride_elems, vec, sh, s);
    default:
        return launch<RLHF_F32>(actor_logits, ref_logits, tokens, logp_out, kl_out, n_positions, vocab,
                                row_stride_elems, vec, sh, s);
    }
}

extern "C" int rlhf_token_logprobs_kl(const void *actor_logits, const void *ref_logits,
                                      const int32_t *tokens, float *logp_out, float *kl_out,
                                      int64_t n_positions, int32_t vocab, int64_t row_stride_elems,
                                      int32_t logits_dtype, void *stream)
{
    const rlhf::Shaping none = {nullptr, nullptr, nullptr, 0.f, 0, nullptr};
    return logprobs_kl_impl(actor_logits, ref_logits, tokens, logp_out, kl_out, n_positions, vocab,
                            row_stride_elems, logits_dtype, none, stream);
}

extern "C" int rlhf_token_logprobs_kl_rewards(const void *actor_logits, const void *ref_logits,
                                              const int32_t *tokens, float *logp_out, float *kl_out,
                                              int64_t n_positions, int32_t vocab, int64_t row_stride_elems,
                                              int32_t logits_dtype, const rlhf_reward_shaping *shaping,
                                              void *stream)
{
    if (!shaping)
        return rlhf::fail(RLHF_ERR_INVALID, "NULL shaping");
    if (shaping->penalty != RLHF_PENALTY_FULL_KL && shaping->penalty != RLHF_PENALTY_SAMPLED)
        return rlhf::fail(RLHF_ERR_INVALID, "penalty %d", shaping->penalty);
    const rlhf::Shaping sh = {shaping->ref_logp_out, shaping->reward_out, shaping->terminal_scores,
                              shaping->kl_coef, shaping->penalty == RLHF_PENALTY_SAMPLED,
                              shaping->token_error_flag};
    return logprobs_kl_impl(actor_logits, ref_logits, tokens, logp_out, kl_out, n_positions, vocab,
                            row_stride_elems, logits_dtype, sh, stream);
}
