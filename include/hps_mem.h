/*
 * hps_mem.h -- C ABI of the host-memory parameter cache that sits behind the HBM table: the
 *              MEM-PS cache of the paper (Section 5; Appendix D "MEM-PS Implementation", cache
 *              policy).  Host memory only: every pointer here is HOST memory.
 *
 * Algorithm 1 around one batch of the outer loop, with this cache as the MEM-PS and the HBM
 * table of hps.h as the HBM-PS:
 *   pull the batch's working parameters     hps_mem_fetch (hits), the tier below for the misses
 *                                           (an SSD store; not part of this library), then
 *                                           hps_mem_store(visit = 1) of what it returned
 *   insert them into the hash table         hps_insert
 *   the mini-batches                        hps_pull / hps_push
 *   collect the updates of the HBM tier     hps_dump_dirty, then hps_mem_store(visit = 0)
 *   update the local cache, dump            hps_mem_complete_batch, hps_mem_take_evicted
 *                                           (to the tier below), hps_clear
 *
 * Cache policy (Appendix D): a visited parameter enters an LRU cache; a parameter the LRU cache
 * evicts enters an LFU cache; a parameter the LFU cache evicts is collected and must be flushed
 * to the tier below before its memory is released; the parameters of the current batch and of
 * batches fetched ahead are pinned until their batch is completed.  Capacities are numbers of
 * parameters; evictions happen in hps_mem_complete_batch; LFU ties go to the parameter that
 * entered the LFU cache first; a parameter's frequency counts its visits since it entered the
 * memory.  Calls on one cache are not thread-safe.
 */
#ifndef HPS_MEM_H_
#define HPS_MEM_H_

#include "hps.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hps_mem hps_mem; /* opaque host object, owned by the library */

typedef struct {
  uint64_t lru_size;        /* parameters in the LRU cache                         */
  uint64_t lfu_size;        /* parameters in the LFU cache                         */
  uint64_t pinned;          /* ... of the LRU cache that an open batch has visited */
  uint64_t evicted_waiting; /* collected parameters not yet taken                  */
  uint64_t hits, misses;    /* of all hps_mem_fetch calls so far                   */
} hps_mem_stats_t;

/* dim floats of weights and acc_len floats of optimizer state per parameter (1 or dim, as the
 * HBM table's optimizer has it).  Errors: HPS_EINVAL, HPS_ENOMEM. */
hps_status hps_mem_create(hps_mem** out, uint32_t dim, uint32_t acc_len, uint64_t lru_capacity,
                          uint64_t lfu_capacity);

/* Visits, on behalf of batch `batch`, every one of the n keys the cache holds: found[i] = 1 and
 * the row goes to h_w[i, :] / h_acc[i, :]; for the others found[i] = 0 and the row is left
 * alone (the caller gets them from the tier below and stores them with visit = 1). */
hps_status hps_mem_fetch(hps_mem* m, const uint64_t* h_keys, uint64_t n, uint64_t batch, float* h_w,
                         float* h_acc, uint8_t* h_found);

/* Puts n rows into the cache.  visit = 1: parameters arriving from the tier below for batch
 * `batch` (each is visited).  visit = 0: updated values of parameters the cache holds (the
 * collect step; no visit, nothing moves); a key it does not hold is taken in as a visit. */
hps_status hps_mem_store(hps_mem* m, const uint64_t* h_keys, uint64_t n, const float* h_w,
                         const float* h_acc, uint64_t batch, int visit);

/* The batch is completed: its parameters are unpinned (unless another open batch visited them),
 * then the LRU cache gives its least recently visited unpinned parameters to the LFU cache
 * until it is within its capacity, and the LFU cache's least frequently visited parameters are
 * collected until it is within its own. */
hps_status hps_mem_complete_batch(hps_mem* m, uint64_t batch);

/* Hands over collected parameters, oldest first, at most max_rows; *h_n gets their number.
 * HPS_ENOMEM if more are waiting (call again). */
hps_status hps_mem_take_evicted(hps_mem* m, uint64_t* h_keys, float* h_w, float* h_acc,
                                uint64_t max_rows, uint64_t* h_n);

/* Keys of the LRU cache, most recently visited first (which = 0), or of the LFU cache in the
 * order they entered it (which = 1): at most max of them; *h_n gets how many there are. */
hps_status hps_mem_list(hps_mem* m, int which, uint64_t* h_keys, uint64_t max, uint64_t* h_n);

hps_status hps_mem_stats(hps_mem* m, hps_mem_stats_t* h_out);

hps_status hps_mem_destroy(hps_mem* m);

#ifdef __cplusplus
}
#endif
#endif /* HPS_MEM_H_ */
