/*
 * rlhf_memtrace.h -- host-side simulator of a caching device allocator, for
 * replaying allocation traces of an RLHF iteration next to the KV arena.
 *
 * The paper's measurements are of the caching allocator underneath the
 * frameworks it studies (Section 2.2; Appendix A): blocks that are freed stay
 * in a pool, a request is served from the pool when a cached block fits and
 * from the driver otherwise, and `empty_cache()` returns cached memory that
 * holds no live block.  Its counters are reserved memory (taken from the
 * driver) and allocated memory (held by live tensors); fragmentation (first
 * paragraph of Section 3; Appendix B) is reserved - allocated sampled whenever
 * the allocator goes to the driver, and the overhead it reports (Section 3.1)
 * is the fragmentation present when reserved memory peaks.
 *
 * The pool policy, which the paper leaves open, is the one the allocator's
 * public documentation describes: requests rounded up to 512 bytes; rounded
 * sizes up to 1 MiB in a small pool fed by 2 MiB segments, larger ones in a
 * large pool fed by 20 MiB segments (requests of 10 MiB and more: a segment of
 * their own size rounded up to 2 MiB); best fit within the pool (ties: oldest
 * segment, lowest offset); a block is split when the remainder is at least 512
 * bytes (small pool) or more than 1 MiB (large pool); a freed block merges with
 * free neighbours of its segment.  No device is touched: everything here is
 * host memory and integers.  Not thread-safe per simulator.
 *
 * Every function returns RLHF_OK or a negative status of rlhf_rollout.h.
 */
#ifndef RLHF_MEMTRACE_H
#define RLHF_MEMTRACE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rlhf_alloc_sim rlhf_alloc_sim;

typedef struct {
    uint64_t reserved_bytes;                        /* taken from the (simulated) driver */
    uint64_t allocated_bytes;                       /* sizes of live blocks */
    uint64_t peak_reserved_bytes;
    uint64_t peak_allocated_bytes;
    uint64_t driver_allocations;
    uint64_t driver_frees;                          /* segments returned by empty_cache */
    uint64_t last_fragmentation_bytes;              /* reserved - allocated at the latest driver allocation */
    uint64_t peak_fragmentation_bytes;              /* largest such sample */
    uint64_t fragmentation_at_peak_reserved_bytes;  /* the sample taken when reserved reached its peak */
    uint64_t n_segments;
    uint64_t n_free_blocks;
} rlhf_alloc_sim_stats_t;

/* Creates an empty simulator (host memory only). */
int rlhf_alloc_sim_create(rlhf_alloc_sim **out);
int rlhf_alloc_sim_destroy(rlhf_alloc_sim *sim);

/* Serves a request of `bytes` (> 0) and returns a handle (> 0) in *handle_out. */
int rlhf_alloc_sim_malloc(rlhf_alloc_sim *sim, uint64_t bytes, uint64_t *handle_out);

/* Returns a live block to the pool.  RLHF_ERR_INVALID for an unknown handle. */
int rlhf_alloc_sim_free(rlhf_alloc_sim *sim, uint64_t handle);

/* Returns every segment without a live block to the driver (Appendix A). */
int rlhf_alloc_sim_empty_cache(rlhf_alloc_sim *sim);

int rlhf_alloc_sim_stats(const rlhf_alloc_sim *sim, rlhf_alloc_sim_stats_t *out);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_MEMTRACE_H */
