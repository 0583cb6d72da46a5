/*
 * kdn_arena.h -- device memory for stored KV chunks, striped over the device memory.
 *
 * The paper's storage module keeps KV caches on several tiers, device memory among them
 * (Sec. 3.1); the chunks a GPU holds are written by kdn_store_chunk front to back and read
 * by kdn_load_chunk / kdn_compose front to back.  On MI355X the 288 GB of HBM behave as a
 * few large regions (thirds of the capacity, one after the other in the order a fresh
 * process is handed memory): a stream of writes that stays inside one region runs
 * measurably slower than one that alternates between regions (about 5.9 against 6.7 TB/s
 * for writes in order, 5.0 against 6.6 TB/s for scattered 32 KiB tiles).  A plain allocation
 * of a few GB lies inside one region.
 *
 * The arena is one range of virtual addresses backed by physical granules that lie far
 * apart: kdn_arena_create takes (nearly) all free device memory as granules, in the order
 * the driver hands them out, and backs granule i of the arena with free granule
 * (i * stride) mod N, where N is the number of free granules and stride is 0.382 N (the
 * golden section, made coprime to N so that no granule is used twice).  Neighbouring
 * granules of the arena then lie 38% of the free memory apart, three in a row never fall
 * into the same third, and nothing depends on knowing where a region begins.  The rest is
 * given back.  The call also times scattered tile writes (kdn_probe_stream) over the head of
 * the arena and over as much memory taken in the driver's order, and reports both rates; the
 * figures are for the record and decide nothing.
 *
 * Creating the arena takes several seconds (the driver needs about 6 s to take back 260 GB
 * of granules) and is meant for start-up, before the engine allocates its paged pool: memory
 * that is already taken is not part of the stride, and other allocations fail while the call
 * runs.
 *
 * One arena per device.  The calls act on the current device and are serialised by a mutex.
 * Memory from the arena is ordinary device memory for kernels and copies; it must not be
 * passed to hipFree.  kdn_shutdown leaves the arena alone; only kdn_arena_destroy (or the end
 * of the process) releases it.  Nothing here is captured by a HIP graph.
 */
#ifndef KDN_ARENA_H
#define KDN_ARENA_H

#include "kdn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kdn_arena_info {
    uint64_t bytes;         /* size of the arena (the request rounded up to whole granules) */
    uint64_t granule;       /* stripe unit in bytes */
    uint64_t in_use;        /* bytes handed out by kdn_arena_alloc and not yet freed */
    uint64_t largest_free;  /* the largest request kdn_arena_alloc could serve now */
    uint64_t free_granules; /* N: granules of free device memory the arena was drawn from */
    uint64_t stride;        /* granule i of the arena is free granule (i * stride) mod N */
    float striped_gbs;      /* scattered 32 KiB tile writes over the first GiB of the arena, GB/s (16 KiB read and
                               32 KiB written per tile); 0 if not measured (arena below 64 MiB, or a failed call) */
    float packed_gbs;       /* the same over as many granules that follow one another in the driver's order */
    float seconds;          /* wall time of kdn_arena_create */
    int32_t reserved;
} kdn_arena_info;

/* Creates the arena of the current device: `bytes` (> 0) rounded up to a multiple of the
 * granule, granule_mib MiB per stripe (0 = 16; else a power of two from 1 to 512 that the
 * device's allocation granularity divides).  info_out: [host] or NULL.  KDN_EINVAL if the
 * device already has an arena or an argument is out of range, KDN_ESIZE if less than bytes
 * plus 2 GiB of device memory is free once the measuring buffer (a quarter of a GiB) is taken,
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
