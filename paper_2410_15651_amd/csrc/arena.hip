// KV arena: one allocation cut into 16-token pages, with the page table and the
// sequence lengths mirrored on the device.
//
// Why an arena: the paper traces the extra memory of RLHF to the allocator
// rather than to live tensors -- the inference phases leave cached blocks of
// assorted sizes that later requests cannot reuse (Section 3.1, Appendix A),
// and generation is the phase with the largest footprint (Appendix B).  Here
// the cache is reserved once and handed out in equal pages, so "reserved" is a
// constant and a page freed by one sequence fits any other.
//
// Host bookkeeping lives in ArenaBook (arena_book.hpp).  This file adds the
// device mirrors and a few small kernels:
//   arena_apply_kernel    applies one call's page-table / length changes, read
//                         straight from a pinned command slot
//   kv_scatter_kernel /   write new K/V rows into their pages in block layout
//   kv_scatter_pages_kernel   (token by token / a whole page at a time)
//   kv_append_step_kernel both of the above in one launch for the call a decode
//                         step makes (one new token per listed sequence)
//   kv_gather_kernel      reads rows back in plain [token][head][dim] order
#include <hip/hip_runtime.h>

#include <cstring>
#include <memory>
#include <new>
#include <vector>

#include "arena_book.hpp"
#include "common.h"
#include "device_ops.h"

namespace rlhf {
namespace {

constexpr int kRingSlots = 4;
constexpr int kPage = RLHF_PAGE_TOKENS;
constexpr int kDescWords = 8;

// Command slot layout (int32 words):
//   [0] n_desc  [1] n_table  [2] n_lens  [3] unused
//   desc [n_desc][8]  = token_offset, seq, start_len, n_new, whole pages before this entry,
//                       edge tokens before this entry, physical page of the first new
//                       token, unused                            (non-empty sequences only)
//   table[n_table][2] = table_index, page (or -1)
//   lens [n_lens][2]  = seq, new_len
__global__ void arena_apply_kernel(const int32_t *__restrict__ cmd, int32_t *__restrict__ table,
                                   int32_t *__restrict__ lens, int32_t *__restrict__ desc)
{
    const int n_desc = cmd[0], n_table = cmd[1], n_lens = cmd[2];
    const int32_t *c_desc = cmd + 4;
    const int32_t *c_table = c_desc + kDescWords * n_desc;
    const int32_t *c_lens = c_table + 2 * n_table;
    const int stride = gridDim.x * blockDim.x;
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    for (int i = tid; i < kDescWords * n_desc; i += stride)
        desc[i] = c_desc[i];
    for (int i = tid; i < n_table; i += stride)
        table[c_table[2 * i]] = c_table[2 * i + 1];
    for (int i = tid; i < n_lens; i += stride)
        lens[c_lens[2 * i]] = c_lens[2 * i + 1];
}

__global__ void fill_i32_kernel(int32_t *__restrict__ p, int64_t n, int32_t value)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        p[i] = value;
}

// Offsets inside a (page, head) block, in elements.
__device__ __forceinline__ int k_block_offset(int slot, int d)
{
    return ((d >> 3) * kPage + slot) * 8 + (d & 7);
}
__device__ __forceinline__ int v_block_offset(int slot, int d, int head_dim)
{
    return ((slot >> 2) * head_dim + d) * 4 + (slot & 3);
}

// An append splits each sequence's new tokens into the pages they fill
// completely and the "edge" tokens before and after those (a decode step is all
// edge tokens, a prompt nearly all whole pages).
//
// Last descriptor whose word `field` is <= x.
__device__ __forceinline__ int find_desc(const int32_t *__restrict__ desc, int n_desc, int field, int64_t x)
{
    int lo = 0, hi = n_desc - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (desc[kDescWords * mid + field] <= x)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// Edge tokens: one wavefront per (token, kv head); K goes in 16-byte granules,
// V element by element into its transposed granules.
__global__ __launch_bounds__(256) void kv_scatter_kernel(
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new,
    uint16_t *__restrict__ k_arena, uint16_t *__restrict__ v_arena,
    const int32_t *__restrict__ table, const int32_t *__restrict__ desc, int n_desc,
    int64_t edge_tokens, int n_kv_heads, int head_dim, int mpps)
{
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= edge_tokens * n_kv_heads)
        return;
    const int64_t e = item / n_kv_heads;
    const int h = (int)(item - e * n_kv_heads);
    const int32_t *d = desc + kDescWords * find_desc(desc, n_desc, 5, e);
    const int start = d[2], n_new = d[3];
    const int first_whole = (start + kPage - 1) / kPage * kPage;         // position where whole pages begin
    const int head_count = min(first_whole - start, n_new);              // edge tokens in front of them
    const int whole_end = head_count < n_new ? (start + n_new) / kPage * kPage : first_whole;
    const int e_local = (int)(e - d[5]);
    const int pos = e_local < head_count ? start + e_local : max(whole_end, first_whole) + (e_local - head_count);
    const int64_t t = (int64_t)d[0] + (pos - start);
    const int page = table[(int64_t)d[1] * mpps + pos / kPage];
    const int slot = pos % kPage;
    const int64_t block = ((int64_t)page * n_kv_heads + h) * (kPage * head_dim);
    const int64_t src = (t * n_kv_heads + h) * head_dim;
    if (lane < head_dim / 8) {
        const uint4 g = *(const uint4 *)(k_new + src + lane * 8);
        *(uint4 *)(k_arena + block + k_block_offset(slot, lane * 8)) = g;
    }
    if (lane < head_dim / 2) {
        const uint32_t w = *(const uint32_t *)(v_new + src + lane * 2);
        v_arena[block + v_block_offset(slot, lane * 2, head_dim)] = (uint16_t)(w & 0xffffu);
        v_arena[block + v_block_offset(slot, lane * 2 + 1, head_dim)] = (uint16_t)(w >> 16);
    }
}

// A decode step's append -- exactly one new token for each listed sequence -- in
// one launch: one wavefront per (sequence, kv head) places the row, and the
// grid's first threads apply the call's page-table and length changes.  The
// row's page comes with the descriptor (the host has just chosen it), so the
// kernel does not depend on its own table update; everything is read straight
// from the pinned command slot.
__global__ __launch_bounds__(256) void kv_append_step_kernel(
    const int32_t *__restrict__ cmd, int32_t *__restrict__ table, int32_t *__restrict__ lens,
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new,
    uint16_t *__restrict__ k_arena, uint16_t *__restrict__ v_arena, int n_desc, int n_table,
    int n_kv_heads, int head_dim)
{
    const int32_t *c_desc = cmd + 4;
    const int32_t *c_table = c_desc + kDescWords * n_desc;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gtid < n_table)
        table[c_table[2 * gtid]] = c_table[2 * gtid + 1];
    if (gtid < n_desc)
        lens[c_desc[kDescWords * gtid + 1]] = c_desc[kDescWords * gtid + 2] + 1;

    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= (int64_t)n_desc * n_kv_heads)
        return;
    const int e = (int)(item / n_kv_heads);
    const int h = (int)(item - (int64_t)e * n_kv_heads);
    const int4 d0 = *(const int4 *)(c_desc + kDescWords * e);      // token_offset, seq, start_len, n_new
    const int4 d1 = *(const int4 *)(c_desc + kDescWords * e + 4);  // .., .., page, ..
    const int slot = d0.z % kPage;
    const int64_t block = ((int64_t)d1.z * n_kv_heads + h) * (kPage * head_dim);
    const int64_t src = ((int64_t)d0.x * n_kv_heads + h) * head_dim;
    if (lane < head_dim / 8) {
        const uint4 g = *(const uint4 *)(k_new + src + lane * 8);
        *(uint4 *)(k_arena + block + k_block_offset(slot, lane * 8)) = g;
    }
    if (lane < head_dim / 2) {
        const uint32_t w = *(const uint32_t *)(v_new + src + lane * 2);
        v_arena[block + v_block_offset(slot, lane * 2, head_dim)] = (uint16_t)(w & 0xffffu);
        v_arena[block + v_block_offset(slot, lane * 2 + 1, head_dim)] = (uint16_t)(w >> 16);
    }
}

// Whole pages: one wavefront per (page, kv head) writes the 16 tokens' K block
// and V block with full 16-byte stores.  K: a block granule is 8 dims of one
// token, copied as it is.  V: a lane takes two adjacent dims of the four tokens
// of a slot quad (four coalesced 4-byte loads) and writes the two transposed
// granules side by side.
__global__ __launch_bounds__(256) void kv_scatter_pages_kernel(
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new,
    uint16_t *__restrict__ k_arena, uint16_t *__restrict__ v_arena,
    const int32_t *__restrict__ table, const int32_t *__restrict__ desc, int n_desc,
    int64_t whole_pages, int n_kv_heads, int head_dim, int mpps)
{
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= whole_pages * n_kv_heads)
        return;
    const int64_t pg = item / n_kv_heads;
    const int h = (int)(item - pg * n_kv_heads);
    const int32_t *d = desc + kDescWords * find_desc(desc, n_desc, 4, pg);
    const int start = d[2];
    const int lp = (start + kPage - 1) / kPage + (int)(pg - d[4]);      // logical page of the sequence
    const int64_t t0 = (int64_t)d[0] + ((int64_t)lp * kPage - start);    // its first token in k_new / v_new
    const int page = table[(int64_t)d[1] * mpps + lp];
    const int64_t block = ((int64_t)page * n_kv_heads + h) * (kPage * head_dim);
    const int64_t row = (int64_t)n_kv_heads * head_dim;                  // elements between two tokens
    const int64_t src = (t0 * n_kv_heads + h) * head_dim;
    // K: granule g = (dim/8)*16 + slot
    for (int g = lane; g < 2 * head_dim; g += 64) {
        const int slot = g & 15, d8 = g >> 4;
        *(uint4 *)(k_arena + block + g * 8) = *(const uint4 *)(k_new + src + slot * row + d8 * 8);
    }
    // V: lane = pair of dims; granules (quad, dim) and (quad, dim+1) are adjacent
    if (lane < head_dim / 2) {
#pragma unroll
        for (int quad = 0; quad < 4; ++quad) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                w[j] = *(const uint32_t *)(v_new + src + (4 * quad + j) * row + lane * 2);
            uint4 out;
            out.x = (w[0] & 0xffffu) | (w[1] << 16);
            out.y = (w[2] & 0xffffu) | (w[3] << 16);
            out.z = (w[0] >> 16) | (w[1] & 0xffff0000u);
            out.w = (w[2] >> 16) | (w[3] & 0xffff0000u);
            *(uint4 *)(v_arena + block + (quad * head_dim + lane * 2) * 4) = out;
        }
    }
}

// One wavefront per (token, kv head) of the requested range.
__global__ __launch_bounds__(256) void kv_gather_kernel(
    const uint16_t *__restrict__ k_arena, const uint16_t *__restrict__ v_arena,
    uint16_t *__restrict__ k_out, uint16_t *__restrict__ v_out, const int32_t *__restrict__ table_row,
    int start, int n, int n_kv_heads, int head_dim)
{
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= (int64_t)n * n_kv_heads)
        return;
    const int i = (int)(item / n_kv_heads);
    const int h = (int)(item - (int64_t)i * n_kv_heads);
    const int pos = start + i;
    const int page = table_row[pos / kPage];
    const int slot = pos % kPage;
    const int64_t block = ((int64_t)page * n_kv_heads + h) * (kPage * head_dim);
    const int64_t dst = ((int64_t)i * n_kv_heads + h) * head_dim;
    if (lane < head_dim / 8)
        *(uint4 *)(k_out + dst + lane * 8) = *(const uint4 *)(k_arena + block + k_block_offset(slot, lane * 8));
    if (lane < head_dim / 2) {
        const uint32_t lo = v_arena[block + v_block_offset(slot, lane * 2, head_dim)];
        const uint32_t hi = v_arena[block + v_block_offset(slot, lane * 2 + 1, head_dim)];
        *(uint32_t *)(v_out + dst + lane * 2) = lo | (hi << 16);
    }
}

struct CommandSlot {
    int32_t *host = nullptr;  // pinned, device-readable
    hipEvent_t done = nullptr;
    bool in_flight = false;
};

}  // namespace
}  // namespace rlhf

struct rlhf_kv_arena {
    rlhf_kv_arena_desc desc;
    std::unique_ptr<rlhf::ArenaBook> book;
    bool host_only = false;
    bool owns_buffer = false;
    int device = -1;
    char *kv = nullptr;            // K half then V half
    size_t half_bytes = 0;
    int32_t *d_table = nullptr;
    int32_t *d_lens = nullptr;
    int32_t *d_desc = nullptr;
    size_t slot_words = 0;
    rlhf::CommandSlot ring[rlhf::kRingSlots];
    int next_slot = 0;
    rlhf::AppendPlan plan;
    rlhf::FreePlan free_plan;
    int fail_next = 0;  // testing aid: this many submissions are treated as refused by the device
    bool broken = false;  // a device error struck after part of a call had been enqueued
};

namespace rlhf {
namespace {

int validate_desc(const rlhf_kv_arena_desc *d, size_t *bytes)
{
    if (!d)
        return fail(RLHF_ERR_INVALID, "NULL arena description");
    if (d->max_seqs <= 0 || d->n_kv_heads <= 0 || d->n_pages <= 0 || d->max_pages_per_seq <= 0)
        return fail(RLHF_ERR_INVALID, "non-positive arena dimension");
    if (d->page_tokens != kPage)
        return fail(RLHF_ERR_UNSUPPORTED, "page_tokens must be %d", kPage);
    if (d->head_dim != 64 && d->head_dim != 128)
        return fail(RLHF_ERR_UNSUPPORTED, "head_dim %d (64 or 128)", d->head_dim);
    if (d->kv_dtype != RLHF_F16 && d->kv_dtype != RLHF_BF16)
        return fail(RLHF_ERR_UNSUPPORTED, "kv_dtype %d (f16 or bf16)", d->kv_dtype);
    if ((int64_t)d->max_seqs * d->max_pages_per_seq > 0x7fffffffLL)
        return fail(RLHF_ERR_INVALID, "page table too large");
    const uint64_t page_half = (uint64_t)d->n_kv_heads * kPage * d->head_dim * 2;
    *bytes = (size_t)(2 * page_half * (uint64_t)d->n_pages);
    return RLHF_OK;
}

void release(rlhf_kv_arena *a)
{
    if (!a->host_only) {
        for (auto &s : a->ring) {
            if (s.done)
                (void)hipEventDestroy(s.done);
            if (s.host)
                (void)hipHostFree(s.host);
        }
        if (a->d_table)
            (void)hipFree(a->d_table);
        if (a->d_lens)
            (void)hipFree(a->d_lens);
        if (a->d_desc)
            (void)hipFree(a->d_desc);
        if (a->owns_buffer && a->kv)
            (void)hipFree(a->kv);
    }
    delete a;
}

// The next command slot, once its previous use (the call kRingSlots calls ago)
// has left the device.  This is the one wait an append or a free can run into,
// and it comes before anything is changed.  The slot is not taken yet.
int wait_for_slot(rlhf_kv_arena *a, CommandSlot **out)
{
    CommandSlot &s = a->ring[a->next_slot];
    if (s.in_flight) {
        RLHF_HIP_TRY(hipEventSynchronize(s.done));
        s.in_flight = false;
    }
    *out = &s;
    return RLHF_OK;
}

void take_slot(rlhf_kv_arena *a)
{
    a->next_slot = (a->next_slot + 1) % kRingSlots;
}

// After the kernel that reads the slot has been enqueued.  A failure here cannot
// be undone (the kernel will run): the arena is marked broken.
int mark_slot_in_flight(rlhf_kv_arena *a, CommandSlot *s, hipStream_t stream)
{
    const hipError_t e = hipEventRecord(s->done, stream);
    if (e != hipSuccess) {
        a->broken = true;
        return fail(RLHF_ERR_DEVICE, "hipEventRecord failed after the update was enqueued: %s; the arena "
                    "is unusable until rlhf_kv_arena_reset", hipGetErrorString(e));
    }
    s->in_flight = true;
    return RLHF_OK;
}

// Launches the kernel that applies the slot's table / length changes.  When the
// launch itself is refused nothing has been enqueued and the caller can undo its
// bookkeeping.
int submit_slot(rlhf_kv_arena *a, CommandSlot *s, int work_items, hipStream_t stream, bool *enqueued)
{
    *enqueued = false;
    const int blocks = std::min(64, std::max(1, (work_items + 255) / 256));
    hipLaunchKernelGGL(arena_apply_kernel, dim3(blocks), dim3(256), 0, stream, s->host, a->d_table,
                       a->d_lens, a->d_desc);
    RLHF_LAUNCH_CHECK("arena_apply_kernel");
    *enqueued = true;
    return mark_slot_in_flight(a, s, stream);
}

int broken_arena()
{
    return fail(RLHF_ERR_DEVICE, "an earlier device error left this arena's device mirrors behind its host "
                "bookkeeping: call rlhf_kv_arena_reset (or destroy it)");
}

int fill_i32(int32_t *p, int64_t n, int32_t value, hipStream_t stream)
{
    const int blocks = (int)std::min<int64_t>(1024, (n + 255) / 256);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(std::max(blocks, 1)), dim3(256), 0, stream, p, n, value);
    RLHF_LAUNCH_CHECK("fill_i32_kernel");
    return RLHF_OK;
}

}  // namespace
}  // namespace rlhf

using namespace rlhf;

extern "C" int rlhf_kv_arena_bytes_required(const rlhf_kv_arena_desc *desc, size_t *out_bytes)
{
    if (!out_bytes)
        return fail(RLHF_ERR_INVALID, "NULL out_bytes");
    return validate_desc(desc, out_bytes);
}

extern "C" int rlhf_kv_arena_create(const rlhf_kv_arena_desc *desc, rlhf_kv_arena **out)
{
    if (!out)
        return fail(RLHF_ERR_INVALID, "NULL out");
    *out = nullptr;
    size_t bytes = 0;
    int rc = validate_desc(desc, &bytes);
    if (rc != RLHF_OK)
        return rc;
    if (desc->initial_free_order && !ArenaBook::is_permutation(desc->initial_free_order, desc->n_pages))
        return fail(RLHF_ERR_INVALID, "initial_free_order is not a permutation of 0..n_pages-1");

    rlhf_kv_arena *a = new (std::nothrow) rlhf_kv_arena();
    if (!a)
        return fail(RLHF_ERR_INVALID, "out of host memory");
    a->desc = *desc;
    a->desc.initial_free_order = nullptr;  // copied into the book; the caller's array is not kept
    a->host_only = (desc->flags & RLHF_ARENA_HOST_ONLY) != 0;
    a->half_bytes = bytes / 2;
    const uint64_t page_bytes_kv = bytes / (uint64_t)desc->n_pages;
    const uint64_t token_bytes_kv = 2ull * desc->n_kv_heads * desc->head_dim * 2;
    a->book.reset(new ArenaBook(desc->max_seqs, desc->n_pages, desc->max_pages_per_seq, kPage,
                                page_bytes_kv, token_bytes_kv, desc->initial_free_order));
    if (a->host_only) {
        *out = a;
        return RLHF_OK;
    }

#define ARENA_TRY(expr)                                                                        \
    do {                                                                                       \
        hipError_t _e = (expr);                                                                \
        if (_e != hipSuccess) {                                                                \
            release(a);                                                                        \
            return fail(RLHF_ERR_DEVICE, "%s failed: %s", #expr, hipGetErrorString(_e));       \
        }                                                                                      \
    } while (0)

    ARENA_TRY(hipGetDevice(&a->device));
    if (desc->device_buffer) {
        if ((uintptr_t)desc->device_buffer % 256 || desc->device_buffer_bytes < bytes) {
            release(a);
            return fail(RLHF_ERR_INVALID, "device_buffer must be 256-byte aligned and hold %zu bytes", bytes);
        }
        a->kv = (char *)desc->device_buffer;
    } else {
        ARENA_TRY(hipMalloc((void **)&a->kv, bytes));
        a->owns_buffer = true;
    }
    const size_t table_elems = (size_t)desc->max_seqs * desc->max_pages_per_seq;
    ARENA_TRY(hipMalloc((void **)&a->d_table, table_elems * sizeof(int32_t)));
    ARENA_TRY(hipMalloc((void **)&a->d_lens, (size_t)desc->max_seqs * sizeof(int32_t)));
    ARENA_TRY(hipMalloc((void **)&a->d_desc, (size_t)desc->max_seqs * kDescWords * sizeof(int32_t)));
    a->slot_words = 4 + (kDescWords + 2) * (size_t)desc->max_seqs + 2 * (size_t)desc->n_pages;
    for (auto &s : a->ring) {
        ARENA_TRY(hipHostMalloc((void **)&s.host, a->slot_words * sizeof(int32_t), hipHostMallocDefault));
        ARENA_TRY(hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
    }
    rc = fill_i32(a->d_table, (int64_t)table_elems, -1, nullptr);
    if (rc == RLHF_OK)
        rc = fill_i32(a->d_lens, desc->max_seqs, 0, nullptr);
    if (rc != RLHF_OK) {
        release(a);
        return rc;
    }
    ARENA_TRY(hipDeviceSynchronize());
#undef ARENA_TRY
    *out = a;
    return RLHF_OK;
}

extern "C" int rlhf_kv_arena_destroy(rlhf_kv_arena *arena)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    if (!arena->host_only)
        (void)hipDeviceSynchronize();
    release(arena);
    return RLHF_OK;
}

extern "C" int rlhf_kv_arena_append(rlhf_kv_arena *arena, const int32_t *seq_ids, const int32_t *n_new,
                                    int32_t n_seqs, const void *k_new, const void *v_new, void *stream)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    if (n_seqs > arena->desc.max_seqs)
        return fail(RLHF_ERR_INVALID, "n_seqs %d above max_seqs", n_seqs);
    if (!arena->host_only) {
        // reject pointer problems before any state changes
        int64_t total = 0;
        for (int32_t i = 0; i < n_seqs && seq_ids && n_new; ++i)
            total += n_new[i] > 0 ? n_new[i] : 0;
        if (total > 0 && (!k_new || !v_new))
            return fail(RLHF_ERR_INVALID, "NULL k_new / v_new");
        if (((uintptr_t)k_new | (uintptr_t)v_new) % 16)
            return fail(RLHF_ERR_INVALID, "k_new / v_new must be 16-byte aligned");
        // every copy kernel below takes one wavefront per (token or page, head):
        // tokens x heads bounds all three grids
        if ((total * arena->desc.n_kv_heads + 3) / 4 > max_workgroups(256))
            return fail(RLHF_ERR_UNSUPPORTED, "append of %lld tokens x %d heads is too large for one launch: split the call",
                        (long long)total, arena->desc.n_kv_heads);
    }
    if (arena->broken)
        return broken_arena();
    // The one step that can wait or fail before any kernel is launched comes first,
    // so that a failure there finds the bookkeeping untouched.
    CommandSlot *slot = nullptr;
    if (!arena->host_only) {
        const int rc = wait_for_slot(arena, &slot);
        if (rc != RLHF_OK)
            return rc;
    }
    const ArenaBook::Result r = arena->book->append(seq_ids, n_new, n_seqs, &arena->plan);
    if (r == ArenaBook::kOom)
        return fail(RLHF_ERR_OOM, "arena has %d free pages, the call needs more", arena->book->pages_free());
    if (r != ArenaBook::kOk)
        return fail(RLHF_ERR_INVALID, "bad or repeated sequence id, negative count, or sequence past max_pages_per_seq");
    if (arena->fail_next > 0) {  // as if the device had refused the call's first kernel
        --arena->fail_next;
        arena->book->undo_append(arena->plan);
        return fail(RLHF_ERR_DEVICE, "simulated device failure: nothing has changed");
    }
    if (arena->host_only || arena->plan.total_tokens == 0)
        return RLHF_OK;

    hipStream_t s = (hipStream_t)stream;
    take_slot(arena);
    const AppendPlan &plan = arena->plan;
    int32_t *w = slot->host;
    int n_desc = 0;
    int32_t *w_desc = w + 4;
    int64_t whole_pages = 0, edge_tokens = 0;
    for (const auto &e : plan.seqs) {
        if (e.n_new == 0)
            continue;
        int32_t *d = w_desc + kDescWords * n_desc;
        d[0] = e.token_offset;
        d[1] = e.seq;
        d[2] = e.start_len;
        d[3] = e.n_new;
        d[4] = (int32_t)whole_pages;
        d[5] = (int32_t)edge_tokens;
        d[6] = arena->book->table()[(size_t)e.seq * arena->desc.max_pages_per_seq + e.start_len / kPage];
        d[7] = 0;
        const int first_whole = (e.start_len + kPage - 1) / kPage;      // first page the entry may fill alone
        const int end_whole = (e.start_len + e.n_new) / kPage;           // one past the last it fills
        const int n_whole = std::max(0, end_whole - first_whole);
        whole_pages += n_whole;
        edge_tokens += e.n_new - n_whole * kPage;
        ++n_desc;
    }
    int32_t *w_table = w_desc + kDescWords * n_desc;
    for (size_t i = 0; i < plan.new_pages.size(); ++i) {
        w_table[2 * i] = plan.new_pages[i].table_index;
        w_table[2 * i + 1] = plan.new_pages[i].page;
    }
    int32_t *w_lens = w_table + 2 * plan.new_pages.size();
    for (int i = 0; i < n_desc; ++i) {
        w_lens[2 * i] = w_desc[kDescWords * i + 1];
        w_lens[2 * i + 1] = w_desc[kDescWords * i + 2] + w_desc[kDescWords * i + 3];
    }
    w[0] = n_desc;
    w[1] = (int32_t)plan.new_pages.size();
    w[2] = n_desc;
    w[3] = 0;
    const int64_t heads = arena->desc.n_kv_heads;
    if (whole_pages == 0 && edge_tokens == n_desc) {
        // a decode step: one token per sequence, placed and booked by one launch
        // (a sequence gets at most one new page, so the grid covers the table changes)
        hipLaunchKernelGGL(kv_append_step_kernel, dim3((unsigned)(((int64_t)n_desc * heads + 3) / 4)), dim3(256),
                           0, s, slot->host, arena->d_table, arena->d_lens, (const uint16_t *)k_new,
                           (const uint16_t *)v_new, (uint16_t *)arena->kv,
                           (uint16_t *)(arena->kv + arena->half_bytes), n_desc, (int)plan.new_pages.size(),
                           arena->desc.n_kv_heads, arena->desc.head_dim);
        if (hipGetLastError() != hipSuccess) {  // refused: nothing was enqueued
            arena->book->undo_append(arena->plan);
            return fail(RLHF_ERR_DEVICE, "launch of kv_append_step_kernel failed; nothing has changed");
        }
        return mark_slot_in_flight(arena, slot, s);
    }
    bool enqueued = false;
    int rc = submit_slot(arena, slot, std::max<int>(kDescWords * n_desc, (int)plan.new_pages.size()), s, &enqueued);
    if (rc != RLHF_OK) {
        if (!enqueued)
            arena->book->undo_append(arena->plan);
        return rc;
    }
    // From here on the device mirrors carry the update: a refused launch of a copy
    // kernel leaves rows unwritten that both mirrors count as present.
    auto copy_launched = [&](const char *name) {
        const hipError_t e = hipGetLastError();
        if (e == hipSuccess)
            return (int)RLHF_OK;
        arena->broken = true;
        return fail(RLHF_ERR_DEVICE, "launch of %s failed after the page table had been updated: %s; the "
                    "arena is unusable until rlhf_kv_arena_reset", name, hipGetErrorString(e));
    };

    if (whole_pages > 0) {
        hipLaunchKernelGGL(kv_scatter_pages_kernel, dim3((unsigned)((whole_pages * heads + 3) / 4)), dim3(256), 0, s,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, (uint16_t *)arena->kv,
                           (uint16_t *)(arena->kv + arena->half_bytes), arena->d_table, arena->d_desc, n_desc,
                           whole_pages, arena->desc.n_kv_heads, arena->desc.head_dim,
                           arena->desc.max_pages_per_seq);
        rc = copy_launched("kv_scatter_pages_kernel");
        if (rc != RLHF_OK)
            return rc;
    }
    if (edge_tokens > 0)
        hipLaunchKernelGGL(kv_scatter_kernel, dim3((unsigned)((edge_tokens * heads + 3) / 4)), dim3(256), 0, s,
                           (const uint16_t *)k_new, (const uint16_t *)v_new, (uint16_t *)arena->kv,
                           (uint16_t *)(arena->kv + arena->half_bytes), arena->d_table, arena->d_desc, n_desc,
                           edge_tokens, arena->desc.n_kv_heads, arena->desc.head_dim,
                           arena->desc.max_pages_per_seq);
    return copy_launched("kv_scatter_kernel");
}

extern "C" int rlhf_kv_arena_free_seq(rlhf_kv_arena *arena, int32_t seq_id, void *stream)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    if (seq_id < 0 || seq_id >= arena->desc.max_seqs)
        return fail(RLHF_ERR_INVALID, "sequence id %d out of range", seq_id);
    if (arena->broken)
        return broken_arena();
    CommandSlot *slot = nullptr;
    if (!arena->host_only) {
        const int rc = wait_for_slot(arena, &slot);  // before anything changes
        if (rc != RLHF_OK)
            return rc;
    }
    const int mpps = arena->desc.max_pages_per_seq;
    const int had = (arena->book->len(seq_id) + kPage - 1) / kPage;
    arena->book->free_seq(seq_id, &arena->free_plan);
    if (arena->fail_next > 0) {
        --arena->fail_next;
        arena->book->undo_free_seq(arena->free_plan);
        return fail(RLHF_ERR_DEVICE, "simulated device failure: nothing has changed");
    }
    if (arena->host_only)
        return RLHF_OK;
    take_slot(arena);
    int32_t *w = slot->host;
    w[0] = 0;
    w[1] = had;
    w[2] = 1;
    w[3] = 0;
    for (int lp = 0; lp < had; ++lp) {
        w[4 + 2 * lp] = seq_id * mpps + lp;
        w[4 + 2 * lp + 1] = -1;
    }
    w[4 + 2 * had] = seq_id;
    w[4 + 2 * had + 1] = 0;
    bool enqueued = false;
    const int rc = submit_slot(arena, slot, std::max(had, 1), (hipStream_t)stream, &enqueued);
    if (rc != RLHF_OK && !enqueued)
        arena->book->undo_free_seq(arena->free_plan);
    return rc;
}

extern "C" int rlhf_kv_arena_fail_next_submissions(rlhf_kv_arena *arena, int32_t n_calls)
{
    if (!arena || n_calls < 0)
        return fail(RLHF_ERR_INVALID, "NULL arena or negative count");
    arena->fail_next = n_calls;
    return RLHF_OK;
}

extern "C" int rlhf_kv_arena_reset(rlhf_kv_arena *arena, void *stream)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    arena->book->reset();
    if (arena->host_only)
        return RLHF_OK;
    arena->broken = false;  // both mirrors are rewritten below
    hipStream_t s = (hipStream_t)stream;
    int rc = fill_i32(arena->d_table, (int64_t)arena->desc.max_seqs * arena->desc.max_pages_per_seq, -1, s);
    if (rc != RLHF_OK)
        return rc;
    return fill_i32(arena->d_lens, arena->desc.max_seqs, 0, s);
}

extern "C" int rlhf_kv_arena_stats(const rlhf_kv_arena *arena, rlhf_kv_arena_stats_t *out)
{
    if (!arena || !out)
        return fail(RLHF_ERR_INVALID, "NULL argument");
    const ArenaBook &b = *arena->book;
    out->reserved_bytes = b.reserved_bytes();
    out->allocated_bytes = b.allocated_bytes();
    out->live_token_bytes = b.live_token_bytes();
    out->driver_allocations = arena->owns_buffer ? 1 : 0;
    out->pages_free = b.pages_free();
    out->pages_in_use = b.pages_in_use();
    out->peak_pages_in_use = b.peak_pages_in_use();
    out->live_seqs = b.live_seqs();
    return RLHF_OK;
}

extern "C" int rlhf_kv_arena_views(const rlhf_kv_arena *arena, const void **k_arena, const void **v_arena,
                                   const int32_t **page_table, const int32_t **seq_lens)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    if (arena->host_only)
        return fail(RLHF_ERR_INVALID, "a host-only arena has no device views");
    if (k_arena)
        *k_arena = arena->kv;
    if (v_arena)
        *v_arena = arena->kv + arena->half_bytes;
    if (page_table)
        *page_table = arena->d_table;
    if (seq_lens)
        *seq_lens = arena->d_lens;
    return RLHF_OK;
}

extern "C" int rlhf_kv_arena_host_state(const rlhf_kv_arena *arena, const int32_t **page_table,
                                        const int32_t **seq_lens, const int32_t **free_list,
                                        int32_t *free_count)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    if (page_table)
        *page_table = arena->book->table();
    if (seq_lens)
        *seq_lens = arena->book->lens();
    if (free_list)
        *free_list = arena->book->free_list_snapshot();
    if (free_count)
        *free_count = arena->book->pages_free();
    return RLHF_OK;
}

extern "C" int rlhf_kv_arena_gather(const rlhf_kv_arena *arena, int32_t seq_id, int32_t start, int32_t n,
                                    void *k_out, void *v_out, void *stream)
{
    if (!arena)
        return fail(RLHF_ERR_INVALID, "NULL arena");
    if (arena->host_only)
        return fail(RLHF_ERR_INVALID, "a host-only arena holds no data");
    if (seq_id < 0 || seq_id >= arena->desc.max_seqs)
        return fail(RLHF_ERR_INVALID, "sequence id %d out of range", seq_id);
    if (start < 0 || n < 0 || (int64_t)start + n > arena->book->len(seq_id))
        return fail(RLHF_ERR_INVALID, "range [%d, %d) outside the sequence's %d tokens", start, start + n,
                    arena->book->len(seq_id));
    if (n == 0)
        return RLHF_OK;
    if (!k_out || !v_out || ((uintptr_t)k_out | (uintptr_t)v_out) % 16)
        return fail(RLHF_ERR_INVALID, "k_out / v_out must be non-NULL and 16-byte aligned");
    const int64_t items = (int64_t)n * arena->desc.n_kv_heads;
    if ((items + 3) / 4 > max_workgroups(256))
        return fail(RLHF_ERR_UNSUPPORTED, "gather of %d tokens x %d heads is too large for one launch: split the call",
                    n, arena->desc.n_kv_heads);
    hipLaunchKernelGGL(kv_gather_kernel, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t *)arena->kv, (const uint16_t *)(arena->kv + arena->half_bytes),
                       (uint16_t *)k_out, (uint16_t *)v_out,
                       arena->d_table + (size_t)seq_id * arena->desc.max_pages_per_seq, start, n,
                       arena->desc.n_kv_heads, arena->desc.head_dim);
    RLHF_LAUNCH_CHECK("kv_gather_kernel");
    return RLHF_OK;
}
