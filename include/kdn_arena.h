/*
 * kdn_arena.h -- device memory for stored KV chunks, striped over the memory's regions.
 *
 * The paper's storage module keeps KV caches on several tiers, device memory among them
 * (Sec. 3.1); the chunks a GPU holds are written by kdn_store_chunk front to back and read
 * by kdn_load_chunk / kdn_compose front to back.  On MI355X the 288 GB of HBM behave as a
 * few large regions that follow one another in allocation order: a stream of writes that
 * stays inside one region runs measurably slower than one that alternates between regions
 * (about 5.9 against 6.7 TB/s for writes in order, 5.0 against 6.6 TB/s for scattered 32 KiB
 * tiles).  A plain allocation of a few GB lies inside one region.  The arena is one range of
 * virtual addresses whose physical granules are taken from the regions in turn, so that
 * every buffer cut from it alternates between them every `granule` bytes.
 *
 * Where the regions begin and end is found by measurement when the arena is created: the
 * call takes (nearly) all free device memory as granules in allocation order, maps pairs of
 * 512 MiB runs of them side by side, times scattered tile writes over each pair with
 * kdn_probe_stream, and finds by bisection where the rate stops being the one of two runs
 * from the same region.  It then checks the result on runs it has not used, keeps the
 * granules the arena needs and gives the rest back.  This takes about a second and is meant
 * for start-up, before the engine allocates its paged pool: memory that is already taken
 * is not seen, and other allocations fail while the call runs.  When the check fails, or
 * fewer than two regions are free, the arena is still created, from consecutive granules
 * (regions = 1), and is then no faster than a plain allocation.
 *
 * One arena per device.  The calls act on the current device and are serialised by a mutex.
 * Memory from the arena is ordinary device memory for kernels and copies; it must not be
 * passed to hipFree.  Nothing here is captured by a HIP graph.
 */
#ifndef KDN_ARENA_H
#define KDN_ARENA_H

#include "kdn.h"

#ifdef __cplusplus
extern "C" {
#endif

#define KDN_ARENA_MAX_REGIONS 8

typedef struct kdn_arena_info {
    uint64_t bytes;        /* size of the arena (the request rounded up to whole granules) */
    uint64_t granule;      /* stripe unit in bytes */
    uint64_t in_use;       /* bytes handed out by kdn_arena_alloc and not yet freed */
    uint64_t largest_free; /* the largest request kdn_arena_alloc could serve now */
    int32_t regions;       /* regions the granules alternate over; 1 = not striped */
    int32_t verified;      /* 1: the regions passed the check on unused runs; 0: fell back to regions = 1,
                              or there was too little free memory to measure */
    uint64_t region_bytes[KDN_ARENA_MAX_REGIONS]; /* free memory found in each region at creation */
    float same_region_gbs; /* scattered-write rate of two runs from one region, as measured */
    float cross_region_gbs;/* lowest rate measured between runs of two different regions (0 if regions = 1) */
    float seconds;         /* wall time of kdn_arena_create */
    int32_t probes;        /* timed pair measurements taken */
} kdn_arena_info;

/* Creates the arena of the current device: `bytes` (> 0) rounded up to a multiple of the
 * granule, granule_mib MiB per stripe (0 = 16; else a power of two from 1 to 512 that the
 * device's allocation granularity divides).  info_out: [host] or NULL.  KDN_EINVAL if the
 * device already has an arena or an argument is out of range, KDN_ESIZE if less than bytes
 * plus 2 GiB of device memory is free once the measuring buffers (0.25 GiB) are taken,
 * KDN_EDEVICE if a HIP call fails (everything taken is given back). */
kdn_status kdn_arena_create(uint64_t bytes, int32_t granule_mib, kdn_arena_info *info_out);

/* Cuts `bytes` (> 0, rounded up to a multiple of 4 KiB) from the arena, first fit;
 * *ptr_out [host] receives a [device] address aligned to 4 KiB.  KDN_ENOTFOUND if the device
 * has no arena, KDN_ESIZE if no free stretch is long enough.  The contents are whatever the
 * memory held. */
kdn_status kdn_arena_alloc(uint64_t bytes, void **ptr_out);

/* Gives back what kdn_arena_alloc returned (exactly that address, else KDN_EINVAL).  The
 * caller makes sure no work that uses it is still running. */
kdn_status kdn_arena_free(void *ptr_dev);

/* Fills *info_out [host]; KDN_ENOTFOUND if the device has no arena. */
kdn_status kdn_arena_query(kdn_arena_info *info_out);

/* Synchronises the device, unmaps and releases the arena, whatever is still handed out
 * included.  KDN_ENOTFOUND if there is none. */
kdn_status kdn_arena_destroy(void);

#ifdef __cplusplus
}
#endif
#endif /* KDN_ARENA_H */
