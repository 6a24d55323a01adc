// Single-token decode attention over the paged KV arena.
//
// In the paper's PPO stage the actor generates its responses one token at a
// time (Section 2.1); each step reads every cached key and value of every
// sequence once, which makes the step a pure HBM stream.  The work is laid out
// on one axis of "page steps": sequence after sequence, KV head after KV head,
// logical page after logical page.  That axis is cut into equal contiguous
// ranges, one per wavefront, for exactly as many wavefronts as the chip holds
// at once.  A wavefront streams the pages of its range with an online softmax,
// and whenever its range leaves a (sequence, head) unit -- or ends -- it writes
// that unit's un-normalised partial (o, m, l).  Every wavefront gets the same
// number of pages whatever the mix of cache lengths, pays its start-up latency
// once per call instead of once per chunk, and never waits for another
// wavefront.  Ranges are defined on logical positions only, so results do not
// depend on which physical pages a sequence owns.
//
// The partials of a unit are merged with log-sum-exp weights, in one of two
// ways.  One launch: a wavefront whose range holds a whole unit normalises and
// stores it at once; otherwise it stores its partial, waits until the stores
// have landed and adds one to the unit's arrival counter, and the wavefront
// that brings the counter to the number of ranges touching the unit -- known
// from the page-count prefix alone -- sets the counter back to zero and merges
// the unit's partials in range order, whoever it is, so the arithmetic does not
// depend on the order of arrival.  Nobody waits.  Partials travel between
// wavefronts through memory, around the per-XCD caches (see store_pair_device).  The counters are device
// memory of the library's own (zero when the module is loaded, zero again after
// every call), one set per stream that calls, because two calls running at once
// must not share them.  Two launches: a second kernel with one wavefront per
// (sequence, query head) does the merge; this needs no state at all and is what
// runs for grouped-query heads, while the stream is being captured into a
// graph, for streams beyond the table, for calls with more units than a counter
// set holds, and for calls with so few units that one wavefront would merge
// dozens of partials.
//
// Partial slots need no bookkeeping: along the axis both the wavefront index w
// and the unit index u only grow, and each new segment raises w + u by at least
// one, so segment (w, u) simply owns slot w + u.
//
// Data path (a wavefront works on one page-head block at a time, the next
// block's loads already in flight):
//   K block  [dim/8][16 slots][8 dims]: the i-th 16-byte-per-lane load hands
//            lane l the dims 8*(4i + l/16) .. +8 of slot l%16.
//   V block  [4 slot-quads][dim][4 slots] in 8-byte granules.
//   One query head per KV head (attn_stream_kernel): each lane dots its K
//   granules with the matching slice of q (v_dot2) and two cross-row adds
//   finish the page's 16 scores; the V loads hand a lane two adjacent dims for
//   four consecutive slots whose probabilities are wave-uniform (v_readlane),
//   so a lane owns two output dims and P*V needs no cross-lane reduction.
//   Probabilities stay fp32.
//   Grouped-query heads (attn_stream_gqa_kernel) make both products small
//   matrix products, and those go to the matrix cores: the same 1 KiB K load is
//   the A operand of a 16x16x32 MFMA whose B operand is the group's q rows,
//   giving S^T[slot][q head]; its result registers, after the softmax, are
//   already laid out as the B operand of the 16x16x16 MFMAs that multiply V^T
//   (A operand, straight from the V block's granules) into O^T[dim][q head].
//   Probabilities are fed as a high and a low 16-bit part so that the product
//   keeps fp32-level accuracy.
// All accumulation is fp32.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <vector>

#include "common.h"
#include "device_ops.h"
#include "mfma_ops.h"

namespace rlhf {
namespace {

constexpr int kPage = RLHF_PAGE_TOKENS;
constexpr int kThreads = 256;
constexpr int kWgWaves = 4;
constexpr int kMaxBatch = 8192;  // the per-workgroup page-count prefix lives in LDS

// Wavefronts launched = compute units x wavefronts per unit; sizes the partial
// buffer.  The launch uses fewer if the device reports less room.  Fewer than
// would fit on purpose: with one block ahead a wavefront keeps 8-16 KB in
// flight, two (one query head per KV head) or one (grouped heads) per SIMD
// already saturate HBM, and under a saturated HBM wavefronts are served at
// visibly unequal rates, so the fewer and faster they are, the shorter the
// stretch at the end of the call in which only the slowest still run (measured
// on the largest workloads: 255 instead of 266 us, 310 instead of 313 us).
constexpr int kComputeUnits = 256;
constexpr int kWavesPerCuMha = 8;
constexpr int kWavesPerCuGqa = 4;

// Arrival counters of the one-launch path: kCounterSets sets, one per calling
// stream (the last one belongs to the entry point that works in the library's
// own scratch), each with room for kMaxFusedUnits (sequence, unit) pairs.
constexpr int kStreamSets = 8;
constexpr int kCounterSets = kStreamSets + 1;
constexpr int kMaxFusedUnits = 1 << 15;
// The one-launch path is for one query head per KV head, while a wavefront merges
// at most about this many partials per unit on average (ranges / units).  Above
// that, and for grouped heads (a unit's partial is up to sixteen rows, and one
// wavefront merging them all loses to the merge kernel's wavefront per query
// head: measured 27 against 26 us, 21 against 17 us on small calls, even at 262 us),
// the merge kernel is the better tool.
constexpr int kFusedMaxAvgPartials = 8;
constexpr int64_t kSmallCallBytes = (int64_t)8 << 20;  // see make_shape

// Device memory owned by the library.  Host code never uses these names as
// addresses: the per-device addresses come from hipGetSymbolAddress.
static __device__ unsigned int g_arrivals[kCounterSets * kMaxFusedUnits];
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char g_scratch[kStaticScratchBytes];

struct Shape {
    int batch, n_q_heads, n_kv_heads, group;
    int heads_per_unit;   // query heads one unit covers: 1, or up to 16 of a group
    int units_per_seq;    // units per sequence
    int mpps, max_len;
    int n_waves;          // upper bound used for sizing
};

Shape make_shape(const rlhf_attn_params &p)
{
    Shape s;
    s.batch = p.batch;
    s.n_q_heads = p.n_q_heads;
    s.n_kv_heads = p.n_kv_heads;
    s.group = p.n_q_heads / p.n_kv_heads;
    s.heads_per_unit = std::min(s.group, 16);
    s.units_per_seq = s.group == 1 ? p.n_q_heads : p.n_kv_heads * ((s.group + 15) / 16);
    s.mpps = p.max_pages_per_seq;
    const int cap = p.max_pages_per_seq * kPage;
    s.max_len = (p.max_seq_len > 0 && p.max_seq_len < cap) ? p.max_seq_len : cap;
    s.n_waves = kComputeUnits * (s.group == 1 ? kWavesPerCuMha : kWavesPerCuGqa);
    // A call that can read only a few megabytes is a chain of latencies, not a stream: with no more
    // ranges than one wavefront per unit can merge, it needs one launch instead of two, which is
    // worth more there than the extra wavefronts (measured: 8.6 against 11.3 us on 48 units of 3 MB).
    const int64_t n_units = (int64_t)s.batch * s.units_per_seq;
    const int64_t most_bytes = n_units * s.max_len * p.head_dim * 4;  // K and V of every unit at full length
    if (s.group == 1 && most_bytes <= kSmallCallBytes) {
        const int64_t few = std::max<int64_t>((kFusedMaxAvgPartials * n_units + kWgWaves - 1) / kWgWaves * kWgWaves,
                                              kWgWaves);
        s.n_waves = (int)std::min<int64_t>(s.n_waves, few);
    }
    return s;
}

// Workspace: [0, prefix_bytes) page-count prefix P[0..batch] (int32), then the
// partial rows of D+2 floats.
size_t prefix_bytes(const Shape &s)
{
    return (((size_t)s.batch + 2) * sizeof(int32_t) + 255) / 256 * 256;
}
size_t partial_rows(const Shape &s)
{
    return ((size_t)s.n_waves + (size_t)s.batch * s.units_per_seq) * s.heads_per_unit;
}

// ---- position on the page-step axis -----------------------------------------
// Step s of the axis is page `page` of unit (b, h): s = U * P[b] + h * np + page,
// where U = units per sequence, P = exclusive prefix of pages per sequence and
// np = pages of sequence b.
struct Cursor {
    int b, h, page, np, len;
};

__device__ __forceinline__ int pages_of(int len, int max_len)
{
    return (min(max(len, 0), max_len) + kPage - 1) / kPage;
}

// Builds P[0..batch] in LDS from the device lengths; every thread of the
// workgroup must call it.  Returns the total number of pages.
__device__ __forceinline__ int build_prefix(const int32_t *__restrict__ seq_lens, int batch, int max_len,
                                            int *s_prefix, int *s_scan)
{
    const int tid = threadIdx.x;
    const int per = (batch + kThreads - 1) / kThreads;
    const int lo = min(tid * per, batch), hi = min(lo + per, batch);
    int sum = 0;
    for (int b = lo; b < hi; ++b)
        sum += pages_of(seq_lens[b], max_len);
    s_scan[tid] = sum;
    __syncthreads();
    // exclusive scan of the 256 segment sums by one wavefront, four per lane
    if (tid < 64) {
        const int a0 = s_scan[4 * tid], a1 = s_scan[4 * tid + 1], a2 = s_scan[4 * tid + 2],
                  a3 = s_scan[4 * tid + 3];
        const int t = a0 + a1 + a2 + a3;
        int incl = t;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d);
            if (tid >= d)
                incl += o;
        }
        const int excl = incl - t;
        s_scan[4 * tid] = excl;
        s_scan[4 * tid + 1] = excl + a0;
        s_scan[4 * tid + 2] = excl + a0 + a1;
        s_scan[4 * tid + 3] = excl + a0 + a1 + a2;
        if (tid == 63)
            s_prefix[batch] = incl;
    }
    __syncthreads();
    int run = s_scan[tid];
    for (int b = lo; b < hi; ++b) {
        s_prefix[b] = run;
        run += pages_of(seq_lens[b], max_len);
    }
    __syncthreads();
    return s_prefix[batch];
}

// Cursor for step s (0 <= s < units * total pages).
__device__ __forceinline__ Cursor locate(int64_t s, const int *s_prefix, const int32_t *__restrict__ seq_lens,
                                         int batch, int units, int max_len)
{
    // largest b with units * P[b] <= s: sequences without pages share their
    // successor's P and are skipped by taking the largest
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)units * s_prefix[mid] <= s)
            lo = mid;
        else
            hi = mid - 1;
    }
    Cursor c;
    c.b = lo;
    c.np = s_prefix[lo + 1] - s_prefix[lo];
    const int r = (int)(s - (int64_t)units * s_prefix[lo]);
    c.h = r / c.np;
    c.page = r - c.h * c.np;
    c.len = min(seq_lens[lo], max_len);
    return c;
}

// Cursor of the next step.  Only called when a next step exists inside the
// wavefront's range, so a following sequence with pages exists when needed.
__device__ __forceinline__ Cursor advance(Cursor c, const int *s_prefix, const int32_t *__restrict__ seq_lens,
                                          int batch, int units, int max_len)
{
    if (++c.page < c.np)
        return c;
    c.page = 0;
    if (++c.h < units)
        return c;
    c.h = 0;
    do {
        ++c.b;
    } while (c.b < batch - 1 && s_prefix[c.b + 1] == s_prefix[c.b]);
    c.np = s_prefix[c.b + 1] - s_prefix[c.b];
    c.len = min(seq_lens[c.b], max_len);
    return c;
}

__device__ __forceinline__ Cursor uniform(Cursor c)
{
    c.b = __builtin_amdgcn_readfirstlane(c.b);
    c.h = __builtin_amdgcn_readfirstlane(c.h);
    c.page = __builtin_amdgcn_readfirstlane(c.page);
    c.np = __builtin_amdgcn_readfirstlane(c.np);
    c.len = __builtin_amdgcn_readfirstlane(c.len);
    return c;
}

// Range w of n owns steps [w*S/n, (w+1)*S/n); with n <= S no range is empty.
__device__ __forceinline__ int64_t range_begin(int64_t w, int64_t total, int n)
{
    return w * total / n;
}

// Wavefront that owns step s when `total` steps are cut into n ranges: the
// largest w with w*total/n <= s (every range is non-empty).
__device__ __forceinline__ int64_t range_owner(int64_t s, int64_t total, int64_t n)
{
    return ((s + 1) * n + total - 1) / total - 1;
}

// Two adjacent output elements (idx even), in fp32 or in the 16-bit type DT.
template <int DT>
__device__ __forceinline__ void store_pair(void *out, int64_t idx, float a, float b, bool as_f32)
{
    if (as_f32)
        *(float2 *)((float *)out + idx) = make_float2(a, b);
    else
        *(uint32_t *)((uint16_t *)out + idx) = pack16x2<DT>(a, b);
}

// Log-sum-exp merge of a unit's partials, one partial at a time in range
// order: (M, L) are the running reference exponent and sum; the caller then does
// acc = fmaf(acc, alpha, e * v) for every element v of the partial's row.  Both
// forms of the call (one launch, two launches) merge through this, in the same
// order, so their outputs are bit-identical.
__device__ __forceinline__ void merge_step(float &M, float &L, float m_i, float l_i, float &alpha, float &e)
{
    const float Mn = fmaxf(M, m_i);
    alpha = fast_exp2(M - Mn);  // 0 for the first partial (M = -inf)
    e = fast_exp2(m_i - Mn);
    L = fmaf(L, alpha, e * l_i);
    M = Mn;
}

// Partials cross between wavefronts on different XCDs, whose L2 caches are not
// kept coherent with each other inside a kernel.  A device-wide release/acquire
// fence would do, but it writes back and invalidates a whole L2, and with a
// thousand wavefronts doing that the call takes twice as long (measured).  So
// the partial rows themselves go around the caches instead: stored and loaded as
// relaxed device-scope atomics (write-through stores, loads that do not trust a
// cached line), 8 bytes at a time, and the only ordering needed is that a
// wavefront's stores have been acknowledged before it counts itself in.
__device__ __forceinline__ void store_pair_device(float *p, float a, float b)
{
    const uint64_t bits = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
    __hip_atomic_store((uint64_t *)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float2 load_pair_device(const float *p)
{
    const uint64_t bits = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32)));
}

// One arrival at a unit's counter, after this wavefront's partial (written with
// store_pair_device by all lanes) has reached memory.  True for the wavefront
// that completes the unit: it has put the counter back to zero and may read
// every partial of the unit with load_pair_device.
__device__ __forceinline__ bool arrive_last(unsigned int *counter, int count, int lane)
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);  // the compiler keeps the order below
    __builtin_amdgcn_s_waitcnt(0);            // every store of this wavefront acknowledged
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    unsigned int old = 0;
    if (lane == 0)
        old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);  // no load of a partial moves above the count
    if (old != (unsigned int)(count - 1))
        return false;
    if (lane == 0)
        __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// One-launch path: sequences without a cached token get zeros.  The launch's
// wavefronts share the sequences out; w < n_waves for every wavefront launched.
__device__ __forceinline__ void zero_empty_rows(const int *s_prefix, void *out, int out_f32, int batch,
                                                int n_q_heads, int head_dim, int w, int n_waves, int lane)
{
    const int64_t n = (int64_t)n_q_heads * head_dim;  // elements of a sequence's output, even
    for (int b = w; b < batch; b += n_waves) {
        if (s_prefix[b + 1] != s_prefix[b])
            continue;
        for (int64_t i = 2 * lane; i < n; i += 128)
            store_pair<RLHF_F16>(out, (int64_t)b * n + i, 0.f, 0.f, out_f32 != 0);  // 16-bit zero is type-independent
    }
}

// ---- one query head per KV head: vector ALU ----------------------------------
template <int DT, int D>
__global__ __launch_bounds__(kThreads) void attn_stream_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, int32_t *__restrict__ prefix_out, float *__restrict__ partials,
    unsigned int *__restrict__ arrivals, void *__restrict__ out, int out_f32,
    int batch, int n_heads, int mpps, int max_len, int n_waves, float scale_log2)
{
    constexpr int NL = D / 32;  // 16-byte loads per lane for one K (or V) block
    extern __shared__ int s_dyn[];
    int *s_prefix = s_dyn;            // [batch + 1]
    int *s_scan = s_dyn + batch + 1;  // [256]
    const int total_pages = build_prefix(seq_lens, batch, max_len, s_prefix, s_scan);
    const bool one_launch = arrivals != nullptr;
    if (blockIdx.x == 0 && !one_launch)  // the merge kernel's copy of the prefix
        for (int i = threadIdx.x; i <= batch; i += kThreads)
            prefix_out[i] = s_prefix[i];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWgWaves + (threadIdx.x >> 6));
    const int64_t total = (int64_t)total_pages * n_heads;
    const int n_ranges = (int)min((int64_t)n_waves, total);  // never more wavefronts than steps
    if (one_launch)
        zero_empty_rows(s_prefix, out, out_f32, batch, n_heads, D, w, n_waves, lane);
    if (w >= n_ranges)
        return;
    const int64_t s0 = range_begin(w, total, n_ranges), s1 = range_begin(w + 1, total, n_ranges);
    const int slot = lane & 15;
    const int64_t page_stride = (int64_t)n_heads * (kPage * D);

    Cursor cur = uniform(locate(s0, s_prefix, seq_lens, batch, n_heads, max_len));
    uint4 qr[NL];
    auto load_q = [&](const Cursor &c) {
        const uint16_t *qrow = q + ((int64_t)c.b * n_heads + c.h) * D;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            qr[i] = load16(qrow + (4 * i + (lane >> 4)) * 8);
    };
    auto load_page = [&](const Cursor &c, uint4(&kd)[NL], uint4(&vd)[NL]) {
        const int page = page_table[(int64_t)c.b * mpps + c.page];
        const int64_t base = (int64_t)page * page_stride + (int64_t)c.h * (kPage * D) + lane * 8;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            kd[i] = load16(k_arena + base + i * 512);
            vd[i] = load16(v_arena + base + i * 512);
        }
    };

    float m = -INFINITY, lsum = 0.f, acc0 = 0.f, acc1 = 0.f;
    auto process_page = [&](const Cursor &c, const uint4(&kb)[NL], uint4(&vb)[NL]) {
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
        const int live = c.len - c.page * kPage;  // >= 1
        const float y = (slot < live) ? part * scale_log2 : -INFINITY;
        const float m_new = fmaxf(m, row16_max(y));  // finite: slot 0 is live
        const float alpha = fast_exp2(m - m_new);
        const float p = fast_exp2(y - m_new);
        lsum = fmaf(lsum, alpha, p);
        acc0 *= alpha;
        acc1 *= alpha;
        m = m_new;
        // Slots past the sequence's end have probability 0, but whatever bits sit
        // there (never written, possibly NaN) must not reach 0 * v: blank them.
        // Only the last page of a sequence can be partial; the branch is uniform.
        if (live < kPage) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int q0 = 4 * ((D == 128) ? i : 2 * i + (lane >> 5));
                const uint32_t m01 = (q0 + 0 < live ? 0x0000ffffu : 0u) | (q0 + 1 < live ? 0xffff0000u : 0u);
                const uint32_t m23 = (q0 + 2 < live ? 0x0000ffffu : 0u) | (q0 + 3 < live ? 0xffff0000u : 0u);
                vb[i].x &= m01;
                vb[i].y &= m23;
                vb[i].z &= m01;
                vb[i].w &= m23;
            }
        }
        // P * V: load i holds slot quad i (D = 128) or quads 2i, 2i+1 in the two
        // halves of the wavefront (D = 64); lane l owns dims 2l, 2l+1 (mod D)
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
    // Ends this wavefront's segment of unit (b, h) and clears the state.  Two
    // launches: the partial goes to slot w + unit.  One launch: a segment that is
    // the whole unit is normalised and stored; otherwise the partial is stored and
    // counted, and the last of the unit's wavefronts to arrive merges them all.
    int seg_page0 = cur.page;  // page of the unit at which this segment began
    auto flush = [&](const Cursor &c) {
        const float l_all = row16_sum(lsum);
        float o0 = acc0, o1 = acc1;
        if constexpr (D == 64) {  // lanes l and l+32 hold the two halves of the slot quads
            o0 += __shfl_xor(o0, 32);
            o1 += __shfl_xor(o1, 32);
        }
        const int64_t unit = (int64_t)c.b * n_heads + c.h;
        if (one_launch && seg_page0 == 0 && c.page == c.np - 1) {
            const float inv = 1.0f / l_all;
            if (lane < D / 2)
                store_pair<DT>(out, unit * D + 2 * lane, o0 * inv, o1 * inv, out_f32 != 0);
        } else {
            float *dst = partials + ((int64_t)w + unit) * (D + 2);
            if (lane < D / 2)
                store_pair_device(dst + 2 * lane, o0, o1);
            if (lane == 0)
                store_pair_device(dst + D, m, l_all);
            if (one_launch) {
                const int64_t first = (int64_t)n_heads * s_prefix[c.b] + (int64_t)c.h * c.np;
                const int64_t w_first = seg_page0 == 0 ? w : range_owner(first, total, n_ranges);
                const int64_t w_last = c.page == c.np - 1 ? w : range_owner(first + c.np - 1, total, n_ranges);
                const int count = (int)(w_last - w_first + 1);
                if (arrive_last(arrivals + unit, count, lane)) {
                    // partials w_first .. w_last of this unit, always in that order
                    const float *src = partials + (w_first + unit) * (D + 2);
                    const int dl = lane < D / 2 ? 2 * lane : 0;
                    float M = -INFINITY, L = 0.f, a0 = 0.f, a1 = 0.f;
                    for (int i0 = 0; i0 < count; i0 += 8) {
                        float2 ml[8], ov[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {  // eight rows in flight; past the end: the last row again, unused
                            const float *row = src + (int64_t)min(i0 + u, count - 1) * (D + 2);
                            ml[u] = load_pair_device(row + D);
                            ov[u] = load_pair_device(row + dl);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            if (i0 + u < count) {
                                float alpha, e;
                                merge_step(M, L, ml[u].x, ml[u].y, alpha, e);
                                a0 = fmaf(a0, alpha, e * ov[u].x);
                                a1 = fmaf(a1, alpha, e * ov[u].y);
                            }
                    }
                    const float inv = 1.0f / L;
                    if (lane < D / 2)
                        store_pair<DT>(out, unit * D + 2 * lane, a0 * inv, a1 * inv, out_f32 != 0);
                }
            }
        }
        m = -INFINITY;
        lsum = acc0 = acc1 = 0.f;
        seg_page0 = 0;
    };

    // One page ahead: the next block's loads are in flight while the current one
    // is consumed.  The last step is peeled off so that the prefetch inside the
    // loop is unconditional (a conditional one would force the wait counters to
    // cover both cases and serialise load and compute).
    uint4 kb[NL], vb[NL];
    load_q(cur);
    load_page(cur, kb, vb);
    for (int64_t s = s0 + 1; s < s1; ++s) {
        const Cursor nxt = uniform(advance(cur, s_prefix, seq_lens, batch, n_heads, max_len));
        uint4 kn[NL], vn[NL];
        load_page(nxt, kn, vn);
        process_page(cur, kb, vb);
        if (nxt.page == 0) {  // the range moves on to another unit
            flush(cur);
            load_q(nxt);
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            kb[i] = kn[i];
            vb[i] = vn[i];
        }
        cur = nxt;
    }
    process_page(cur, kb, vb);
    flush(cur);
}

// ---- grouped-query variant on the matrix cores --------------------------------
// A unit is (sequence, KV head, block of <= 16 query heads of its group): unit
// index h of a sequence = kv head * blocks per group + block.  Lane l = (group
// g = l/16, column c = l%16): c is a slot when the lane feeds K, a query head
// when it feeds q or holds scores and outputs.
template <int DT, int D>
__global__ __launch_bounds__(kThreads) void attn_stream_gqa_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_arena,
    const uint16_t *__restrict__ v_arena, const int32_t *__restrict__ page_table,
    const int32_t *__restrict__ seq_lens, int32_t *__restrict__ prefix_out, float *__restrict__ partials,
    int batch, int n_q_heads, int n_kv_heads, int mpps, int max_len, int n_waves, float scale_log2)
{
    constexpr int NL = D / 32;
    extern __shared__ int s_dyn[];
    int *s_prefix = s_dyn;
    int *s_scan = s_dyn + batch + 1;
    const int total_pages = build_prefix(seq_lens, batch, max_len, s_prefix, s_scan);
    if (blockIdx.x == 0)  // the merge kernel's copy of the prefix
        for (int i = threadIdx.x; i <= batch; i += kThreads)
            prefix_out[i] = s_prefix[i];

    const int group = n_q_heads / n_kv_heads;
    const int n_qb = (group + 15) >> 4;
    const int units = n_kv_heads * n_qb;  // per sequence
    const int rows_per_unit = min(group, 16);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWgWaves + (threadIdx.x >> 6));
    const int64_t total = (int64_t)total_pages * units;
    const int n_ranges = (int)min((int64_t)n_waves, total);  // never more wavefronts than steps
    if (w >= n_ranges)
        return;
    const int64_t s0 = range_begin(w, total, n_ranges), s1 = range_begin(w + 1, total, n_ranges);
    const int g = lane >> 4, c = lane & 15;
    const int64_t page_stride = (int64_t)n_kv_heads * (kPage * D);
    const int k_lane = lane * 8;             // K: granule 64*i + lane
    const int v_lane = (g * D + 2 * c) * 4;  // V: granules (quad g, dims 32*i + 2c, +1)

    Cursor cur = uniform(locate(s0, s_prefix, seq_lens, batch, units, max_len));
    // q as the B operand: column c = head, contraction entries = dims 8*(4i+g) .. +8
    uint4 qr[NL];
    int n_heads_here = 0;
    auto load_q = [&](const Cursor &cu) {
        const int hkv = cu.h / n_qb, qb = cu.h - hkv * n_qb;
        const int head0 = hkv * group + qb * 16;
        n_heads_here = min(16, group - qb * 16);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            qr[i] = make_uint4(0, 0, 0, 0);
            if (c < n_heads_here)
                qr[i] = load16(q + ((int64_t)cu.b * n_q_heads + head0 + c) * D + (4 * i + g) * 8);
        }
    };
    auto load_page = [&](const Cursor &cu, uint4(&kd)[NL], uint4(&vd)[NL]) {
        const int page = page_table[(int64_t)cu.b * mpps + cu.page];
        const int64_t base = (int64_t)page * page_stride + (int64_t)(cu.h / n_qb) * (kPage * D);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            kd[i] = load16(k_arena + base + k_lane + i * 512);
            vd[i] = load16(v_arena + base + v_lane + i * 128);
        }
    };

    float m = -INFINITY, lsum = 0.f;
    f32x4_t o[NL][2];
#pragma unroll
    for (int i = 0; i < NL; ++i)
        o[i][0] = o[i][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    auto process_page = [&](const Cursor &cu, const uint4(&kb)[NL], uint4(&vb)[NL]) {
        // S^T[slot 4g+j][head c]
        f32x4_t sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NL; ++i)
            sc = mfma_k32<DT>(kb[i], qr[i], sc);
        const int live = cu.len - cu.page * kPage;
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            y[j] = (4 * g + j < live) ? sc[j] * scale_log2 : -INFINITY;
        float mx = fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));  // finite: slot 0 of the page is live
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
    // o[i][e][j] is row 4g+j of its tile, i.e. dim 32i + 2(4g+j) + e, for head c.
    // A unit's partial is one row per query head of the unit, at slot w + unit.
    auto flush = [&](const Cursor &cu) {
        float l_all = lsum + __shfl_xor(lsum, 16);
        l_all += __shfl_xor(l_all, 32);
        if (c < n_heads_here) {
            float *dst = partials +
                         (((int64_t)w + (int64_t)cu.b * units + cu.h) * rows_per_unit + c) * (D + 2);
#pragma unroll
            for (int i = 0; i < NL; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *(float2 *)(dst + 32 * i + 2 * (4 * g + j)) = make_float2(o[i][0][j], o[i][1][j]);
            if (g == 0)
                *(float2 *)(dst + D) = make_float2(m, l_all);
        }
        m = -INFINITY;
        lsum = 0.f;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            o[i][0] = o[i][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    };

    // one page ahead, last step peeled (see attn_stream_kernel)
    uint4 kb[NL], vb[NL];
    load_q(cur);
    load_page(cur, kb, vb);
    for (int64_t s = s0 + 1; s < s1; ++s) {
        const Cursor nxt = uniform(advance(cur, s_prefix, seq_lens, batch, units, max_len));
        uint4 kn[NL], vn[NL];
        load_page(nxt, kn, vn);
        process_page(cur, kb, vb);
        if (nxt.page == 0) {
            flush(cur);
            load_q(nxt);
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            kb[i] = kn[i];
            vb[i] = vn[i];
        }
        cur = nxt;
    }
    process_page(cur, kb, vb);
    flush(cur);
}

// One wavefront per (sequence, query head): finds the wavefronts whose ranges
// touched the head's unit, then out = sum_w e_w o_w / sum_w e_w l_w with
// e_w = 2^(m_w - max m).
template <int ODT, int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(
    const float *__restrict__ partials, const int32_t *__restrict__ prefix, void *__restrict__ out,
    int batch, int n_q_heads, int n_kv_heads, int n_waves)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // b * Hq + hq
    if (row >= (int64_t)batch * n_q_heads)
        return;
    const int b = (int)(row / n_q_heads);
    const int hq = (int)(row - (int64_t)b * n_q_heads);
    const int group = n_q_heads / n_kv_heads;
    int units, h, col, rows_per_unit;
    if (group == 1) {
        units = n_q_heads;
        h = hq;
        col = 0;
        rows_per_unit = 1;
    } else {
        const int n_qb = (group + 15) >> 4;
        const int hkv = hq / group, qi = hq - hkv * group;
        units = n_kv_heads * n_qb;
        h = hkv * n_qb + (qi >> 4);
        col = qi & 15;
        rows_per_unit = min(group, 16);
    }
    const int np = prefix[b + 1] - prefix[b];
    const int64_t total = (int64_t)prefix[batch] * units;
    constexpr int PER = D / 64;
    float o[PER], l = 0.f;
#pragma unroll
    for (int k = 0; k < PER; ++k)
        o[k] = 0.f;
    if (np > 0) {
        const int64_t first = (int64_t)units * prefix[b] + (int64_t)h * np, last = first + np - 1;
        const int64_t n = min((int64_t)n_waves, total);  // ranges the stream kernel used
        const int64_t w_first = range_owner(first, total, n), w_last = range_owner(last, total, n);
        const int count = (int)(w_last - w_first + 1);
        const int64_t row_stride = (int64_t)rows_per_unit * (D + 2);
        const float *base = partials + ((w_first + (int64_t)b * units + h) * rows_per_unit + col) * (D + 2);
        // partials w_first .. w_last in that order, four rows in flight
        float M = -INFINITY;
        for (int i0 = 0; i0 < count; i0 += 4) {
            float2 ml[4];
            float v[4][PER];
#pragma unroll
            for (int u = 0; u < 4; ++u) {  // past the end: the last row again, unused
                const float *r = base + (int64_t)min(i0 + u, count - 1) * row_stride;
                ml[u] = *(const float2 *)(r + D);
#pragma unroll
                for (int k = 0; k < PER; ++k)
                    v[u][k] = r[lane + 64 * k];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u < count) {
                    float alpha, e;
                    merge_step(M, l, ml[u].x, ml[u].y, alpha, e);
#pragma unroll
                    for (int k = 0; k < PER; ++k)
                        o[k] = fmaf(o[k], alpha, e * v[u][k]);
                }
        }
    }
    const float inv = np > 0 ? 1.0f / l : 0.f;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const float r = np > 0 ? o[k] * inv : 0.f;
        const int64_t idx = row * D + lane + 64 * k;
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
    if (p->batch > kMaxBatch)
        return fail(RLHF_ERR_UNSUPPORTED, "batch %d above %d: split the call", p->batch, kMaxBatch);
    if ((int64_t)p->max_pages_per_seq * kPage > 0x7fffffffLL ||
        (int64_t)p->batch * p->max_pages_per_seq > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "page table too large");
    if ((int64_t)p->batch * p->n_q_heads > 4 * max_workgroups(256))  // merge: one wavefront per (sequence, head)
        return fail(RLHF_ERR_UNSUPPORTED, "batch x n_q_heads too large for one launch: split the call");
    return RLHF_OK;
}

// Per-device addresses of the library's own device memory and the table that
// gives each calling stream a counter set of its own.  Filled on the first call
// on a device, with that device current.
constexpr int kMaxDevices = 64;
struct DeviceState {
    bool ready = false;
    int compute_units = 0;
    unsigned int *arrivals = nullptr;   // g_arrivals on this device
    unsigned char *scratch = nullptr;   // g_scratch on this device
    int n_streams = 0;
    hipStream_t streams[kStreamSets] = {};
};
std::mutex g_device_mutex;
DeviceState g_devices[kMaxDevices];

int device_state(DeviceState **out)
{
    int dev = 0;
    RLHF_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(RLHF_ERR_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lock(g_device_mutex);
    DeviceState &d = g_devices[dev];
    if (!d.ready) {
        RLHF_HIP_TRY(hipDeviceGetAttribute(&d.compute_units, hipDeviceAttributeMultiprocessorCount, dev));
        RLHF_HIP_TRY(hipGetSymbolAddress((void **)&d.arrivals, HIP_SYMBOL(g_arrivals)));
        RLHF_HIP_TRY(hipGetSymbolAddress((void **)&d.scratch, HIP_SYMBOL(g_scratch)));
        d.ready = true;
    }
    *out = &d;
    return RLHF_OK;
}

// Counter set of a stream on this device, or -1 when the table is full.  Calls
// on one stream run one after the other, so they can share a set; a stream keeps
// its set for the life of the process.
int counter_set_of(DeviceState *d, hipStream_t s)
{
    std::lock_guard<std::mutex> lock(g_device_mutex);
    for (int i = 0; i < d->n_streams; ++i)
        if (d->streams[i] == s)
            return i;
    if (d->n_streams == kStreamSets)
        return -1;
    d->streams[d->n_streams] = s;
    return d->n_streams++;
}

// Whether kernels launched on s now are being recorded rather than run.  A
// failing query counts as "yes": the stateless path is always right.
bool being_captured(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return true;
    }
    return st != hipStreamCaptureStatusNone;
}

enum class Scratch { Caller, Library };

template <int DT, int D>
int launch(const rlhf_attn_params &p, const Shape &sh, const void *q, const void *k_arena,
           const void *v_arena, const int32_t *page_table, const int32_t *seq_lens, void *out,
           void *workspace, Scratch where, hipStream_t s)
{
    const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)D);
    const size_t lds = ((size_t)p.batch + 1 + kThreads) * sizeof(int);
    const int64_t n_units = (int64_t)p.batch * sh.units_per_seq;
    const int waves_per_cu = sh.group == 1 ? kWavesPerCuMha : kWavesPerCuGqa;

    // One launch or two (see the top of the file).
    unsigned int *arrivals = nullptr;
    int n_waves = sh.n_waves;
    const bool capturing = being_captured(s);
    if (!capturing || where == Scratch::Library) {
        DeviceState *d = nullptr;
        const int rc = device_state(&d);
        if (rc != RLHF_OK)
            return rc;
        n_waves = std::min(sh.n_waves, std::max(d->compute_units, 1) * waves_per_cu);
        if (where == Scratch::Library)
            workspace = d->scratch;
        // ranges the kernel will cut the axis into, at most: wavefronts, or page steps if fewer
        const int64_t ranges = std::min<int64_t>(n_waves, n_units * ((sh.max_len + kPage - 1) / kPage));
        if (!capturing && sh.group == 1 && n_units <= kMaxFusedUnits && ranges <= kFusedMaxAvgPartials * n_units) {
            const int set = where == Scratch::Library ? kStreamSets : counter_set_of(d, s);
            if (set >= 0)
                arrivals = d->arrivals + (size_t)set * kMaxFusedUnits;
        }
    }
    int32_t *prefix = (int32_t *)workspace;
    float *partials = (float *)((char *)workspace + prefix_bytes(sh));
    const int out_f32 = p.out_dtype == RLHF_F32;

    if (sh.group == 1) {
        hipLaunchKernelGGL((attn_stream_kernel<DT, D>), dim3(n_waves / kWgWaves), dim3(kThreads), lds, s,
                           (const uint16_t *)q, (const uint16_t *)k_arena, (const uint16_t *)v_arena,
                           page_table, seq_lens, prefix, partials, arrivals, out, out_f32, p.batch,
                           p.n_q_heads, p.max_pages_per_seq, sh.max_len, n_waves, scale * kLog2e);
        RLHF_LAUNCH_CHECK("attn_stream_kernel");
    } else {
        hipLaunchKernelGGL((attn_stream_gqa_kernel<DT, D>), dim3(n_waves / kWgWaves), dim3(kThreads), lds, s,
                           (const uint16_t *)q, (const uint16_t *)k_arena, (const uint16_t *)v_arena,
                           page_table, seq_lens, prefix, partials, p.batch, p.n_q_heads, p.n_kv_heads,
                           p.max_pages_per_seq, sh.max_len, n_waves, scale * kLog2e);
        RLHF_LAUNCH_CHECK("attn_stream_gqa_kernel");
    }
    if (arrivals != nullptr)
        return RLHF_OK;
    const int64_t rows = (int64_t)p.batch * p.n_q_heads;
    const dim3 mgrid((unsigned)((rows + 3) / 4));
    if (p.out_dtype == RLHF_F32)
        hipLaunchKernelGGL((attn_merge_kernel<RLHF_F32, D>), mgrid, dim3(256), 0, s, partials, prefix, out,
                           p.batch, p.n_q_heads, p.n_kv_heads, n_waves);
    else
        hipLaunchKernelGGL((attn_merge_kernel<DT, D>), mgrid, dim3(256), 0, s, partials, prefix, out, p.batch,
                           p.n_q_heads, p.n_kv_heads, n_waves);
    RLHF_LAUNCH_CHECK("attn_merge_kernel");
    return RLHF_OK;
}

size_t workspace_need(const rlhf_attn_params &p, const Shape &sh)
{
    return prefix_bytes(sh) + partial_rows(sh) * (p.head_dim + 2) * sizeof(float);
}

int decode_attention(const rlhf_attn_params *params, const void *q, const void *k_arena, const void *v_arena,
                     const int32_t *page_table, const int32_t *seq_lens, void *out, void *workspace,
                     size_t workspace_bytes_given, Scratch where, void *stream)
{
    int rc = check_params(params);
    if (rc != RLHF_OK)
        return rc;
    const rlhf_attn_params &p = *params;
    if (p.batch == 0)
        return RLHF_OK;
    if (!q || !k_arena || !v_arena || !page_table || !seq_lens || !out ||
        (where == Scratch::Caller && !workspace))
        return fail(RLHF_ERR_INVALID, "NULL pointer");
    if (((uintptr_t)q | (uintptr_t)k_arena | (uintptr_t)v_arena | (uintptr_t)out | (uintptr_t)workspace) % 16)
        return fail(RLHF_ERR_INVALID, "q, k_arena, v_arena, out and workspace must be 16-byte aligned");
    const Shape sh = make_shape(p);
    const size_t need = workspace_need(p, sh);
    if (where == Scratch::Caller && workspace_bytes_given < need)
        return fail(RLHF_ERR_INVALID, "workspace holds %zu bytes, %zu needed", workspace_bytes_given, need);
    if (where == Scratch::Library && need > kStaticScratchBytes)
        return fail(RLHF_ERR_UNSUPPORTED,
                    "this shape needs %zu bytes of scratch, the library's own holds %zu: use "
                    "rlhf_decode_attention with a workspace", need, kStaticScratchBytes);
    hipStream_t s = (hipStream_t)stream;
    if (p.qkv_dtype == RLHF_BF16) {
        if (p.head_dim == 128)
            return launch<RLHF_BF16, 128>(p, sh, q, k_arena, v_arena, page_table, seq_lens, out, workspace, where, s);
        return launch<RLHF_BF16, 64>(p, sh, q, k_arena, v_arena, page_table, seq_lens, out, workspace, where, s);
    }
    if (p.head_dim == 128)
        return launch<RLHF_F16, 128>(p, sh, q, k_arena, v_arena, page_table, seq_lens, out, workspace, where, s);
    return launch<RLHF_F16, 64>(p, sh, q, k_arena, v_arena, page_table, seq_lens, out, workspace, where, s);
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
    *out_bytes = workspace_need(*params, make_shape(*params));
    return RLHF_OK;
}

extern "C" int rlhf_decode_attention(const rlhf_attn_params *params, const void *q, const void *k_arena,
                                     const void *v_arena, const int32_t *page_table, const int32_t *seq_lens,
                                     void *out, void *workspace, size_t workspace_bytes_given, void *stream)
{
    return decode_attention(params, q, k_arena, v_arena, page_table, seq_lens, out, workspace,
                            workspace_bytes_given, Scratch::Caller, stream);
}

extern "C" int rlhf_decode_attention_static(const rlhf_attn_params *params, const void *q, const void *k_arena,
                                            const void *v_arena, const int32_t *page_table,
                                            const int32_t *seq_lens, void *out, void *stream)
{
    return decode_attention(params, q, k_arena, v_arena, page_table, seq_lens, out, nullptr, 0,
                            Scratch::Library, stream);
}
