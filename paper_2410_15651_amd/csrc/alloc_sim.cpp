// Host-side simulator of a caching device allocator (see rlhf_memtrace.h for
// the policy and the passages of the paper it serves).  Segments keep their
// blocks in an offset-ordered map; each pool keeps its free blocks in a set
// ordered by (size, segment, offset), so best fit is one lower_bound.
#include <cstdint>
#include <map>
#include <memory>
#include <set>
#include <tuple>
#include <unordered_map>
#include <vector>

#include "common.h"
#include "rlhf_memtrace.h"

namespace {

constexpr uint64_t kMiB = 1ull << 20;
constexpr uint64_t kRound = 512;
constexpr uint64_t kSmallLimit = kMiB;
constexpr uint64_t kSmallSegment = 2 * kMiB;
constexpr uint64_t kLargeSegment = 20 * kMiB;
constexpr uint64_t kLargeDirect = 10 * kMiB;
constexpr uint64_t kLargeRound = 2 * kMiB;

struct Block {
    uint64_t size;
    bool free;
};

struct Segment {
    bool small;
    bool released = false;
    uint64_t size;
    std::map<uint64_t, Block> blocks;  // by offset
};

using FreeKey = std::tuple<uint64_t, uint32_t, uint64_t>;  // size, segment, offset

}  // namespace

struct rlhf_alloc_sim {
    std::vector<Segment> segments;
    std::set<FreeKey> free_blocks[2];  // [0] large pool, [1] small pool
    std::unordered_map<uint64_t, std::pair<uint32_t, uint64_t>> live;  // handle -> segment, offset
    uint64_t next_handle = 1;
    rlhf_alloc_sim_stats_t st{};
};

using namespace rlhf;

extern "C" int rlhf_alloc_sim_create(rlhf_alloc_sim **out)
{
    if (!out)
        return fail(RLHF_ERR_INVALID, "NULL out");
    *out = new rlhf_alloc_sim();
    return RLHF_OK;
}

extern "C" int rlhf_alloc_sim_destroy(rlhf_alloc_sim *sim)
{
    delete sim;
    return RLHF_OK;
}

extern "C" int rlhf_alloc_sim_malloc(rlhf_alloc_sim *sim, uint64_t bytes, uint64_t *handle_out)
{
    if (!sim || !handle_out)
        return fail(RLHF_ERR_INVALID, "NULL argument");
    if (bytes == 0 || bytes > (1ull << 60))
        return fail(RLHF_ERR_INVALID, "request of %llu bytes", (unsigned long long)bytes);
    const uint64_t size = (bytes + kRound - 1) / kRound * kRound;
    const bool small = size <= kSmallLimit;
    auto &pool = sim->free_blocks[small];
    auto it = pool.lower_bound(FreeKey{size, 0, 0});
    uint32_t seg_index;
    uint64_t offset;
    if (it == pool.end()) {
        const uint64_t seg_size = small ? kSmallSegment
                                  : size < kLargeDirect ? kLargeSegment
                                                        : (size + kLargeRound - 1) / kLargeRound * kLargeRound;
        const uint64_t frag = sim->st.reserved_bytes - sim->st.allocated_bytes;
        sim->st.last_fragmentation_bytes = frag;
        if (frag > sim->st.peak_fragmentation_bytes)
            sim->st.peak_fragmentation_bytes = frag;
        sim->st.reserved_bytes += seg_size;
        sim->st.driver_allocations += 1;
        if (sim->st.reserved_bytes > sim->st.peak_reserved_bytes) {
            sim->st.peak_reserved_bytes = sim->st.reserved_bytes;
            sim->st.fragmentation_at_peak_reserved_bytes = frag;
        }
        Segment seg;
        seg.small = small;
        seg.size = seg_size;
        seg.blocks[0] = Block{seg_size, true};
        sim->segments.push_back(std::move(seg));
        seg_index = (uint32_t)sim->segments.size() - 1;
        offset = 0;
        sim->st.n_segments += 1;
        sim->st.n_free_blocks += 1;
    } else {
        seg_index = std::get<1>(*it);
        offset = std::get<2>(*it);
        pool.erase(it);
    }
    Segment &seg = sim->segments[seg_index];
    Block &blk = seg.blocks[offset];
    const uint64_t rest = blk.size - size;
    if (small ? rest >= kRound : rest > kMiB) {
        blk.size = size;
        seg.blocks[offset + size] = Block{rest, true};
        pool.insert(FreeKey{rest, seg_index, offset + size});
        sim->st.n_free_blocks += 1;
    }
    blk.free = false;
    sim->st.n_free_blocks -= 1;
    sim->st.allocated_bytes += blk.size;
    if (sim->st.allocated_bytes > sim->st.peak_allocated_bytes)
        sim->st.peak_allocated_bytes = sim->st.allocated_bytes;
    const uint64_t h = sim->next_handle++;
    sim->live[h] = {seg_index, offset};
    *handle_out = h;
    return RLHF_OK;
}

extern "C" int rlhf_alloc_sim_free(rlhf_alloc_sim *sim, uint64_t handle)
{
    if (!sim)
        return fail(RLHF_ERR_INVALID, "NULL simulator");
    auto lv = sim->live.find(handle);
    if (lv == sim->live.end())
        return fail(RLHF_ERR_INVALID, "handle %llu is not live", (unsigned long long)handle);
    const uint32_t seg_index = lv->second.first;
    uint64_t offset = lv->second.second;
    sim->live.erase(lv);
    Segment &seg = sim->segments[seg_index];
    auto &pool = sim->free_blocks[seg.small];
    auto it = seg.blocks.find(offset);
    sim->st.allocated_bytes -= it->second.size;
    it->second.free = true;
    sim->st.n_free_blocks += 1;
    auto next = std::next(it);
    if (next != seg.blocks.end() && next->second.free) {
        pool.erase(FreeKey{next->second.size, seg_index, next->first});
        it->second.size += next->second.size;
        seg.blocks.erase(next);
        sim->st.n_free_blocks -= 1;
    }
    if (it != seg.blocks.begin()) {
        auto prev = std::prev(it);
        if (prev->second.free) {
            pool.erase(FreeKey{prev->second.size, seg_index, prev->first});
            prev->second.size += it->second.size;
            seg.blocks.erase(it);
            it = prev;
            sim->st.n_free_blocks -= 1;
        }
    }
    pool.insert(FreeKey{it->second.size, seg_index, it->first});
    return RLHF_OK;
}

extern "C" int rlhf_alloc_sim_empty_cache(rlhf_alloc_sim *sim)
{
    if (!sim)
        return fail(RLHF_ERR_INVALID, "NULL simulator");
    for (uint32_t i = 0; i < sim->segments.size(); ++i) {
        Segment &seg = sim->segments[i];
        if (seg.released || seg.blocks.size() != 1 || !seg.blocks.begin()->second.free)
            continue;
        sim->free_blocks[seg.small].erase(FreeKey{seg.size, i, 0});
        seg.blocks.clear();
        seg.released = true;
        sim->st.reserved_bytes -= seg.size;
        sim->st.driver_frees += 1;
        sim->st.n_segments -= 1;
        sim->st.n_free_blocks -= 1;
    }
    return RLHF_OK;
}

extern "C" int rlhf_alloc_sim_stats(const rlhf_alloc_sim *sim, rlhf_alloc_sim_stats_t *out)
{
    if (!sim || !out)
        return fail(RLHF_ERR_INVALID, "NULL argument");
    *out = sim->st;
    return RLHF_OK;
}
