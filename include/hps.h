/*
 * hps.h -- C ABI of the HBM-resident parameter server's mini-batch pull/push path
 *          for one MI355X (gfx950).
 *
 * What is modelled (paper: "Distributed Hierarchical GPU Parameter Server for
 * Massive Scale Deep Learning Ads Systems", MLSys 2020):
 *   - Section 4.1 "Local GPU hash table": an open-addressing hash table in HBM,
 *     capacity fixed at construction (no device allocation afterwards), integrity
 *     under parallel updates kept by GPU atomics; operations insert, get, accumulate.
 *   - Algorithm 1: insert the working parameters, then for each mini-batch pull the
 *     referenced parameters, train, push the updates back; after the batch the host
 *     tier collects the table's content.
 *   - Section 3 "Workflow": the union of the parameters a batch references.
 * This library is one GPU's local share of that (no inter-GPU partition/exchange).
 *
 * A pull (i) sorts the mini-batch's uint64 feature keys into ascending unique keys
 * plus, per occurrence, the rank of its key, (ii) looks every unique key up in the
 * table, inserting a deterministic initial row for keys not yet present, and
 * (iii) sums the embedding rows of each bag (example x slot).  A push sums the
 * upstream gradients of the pooled bags per unique key and takes one Adagrad step
 * on every touched row, in place.
 *
 * Conventions
 *   - Every pointer named d_* is DEVICE memory owned by the caller (for example a
 *     torch tensor's data_ptr()); the library never allocates or frees device
 *     memory (hps_create takes 64 bytes of pinned host memory, hps_destroy frees
 *     them).  `storage` holds the table for its whole life, `workspace` holds the
 *     context of the outstanding pull.  Both must be 256-byte aligned.
 *   - Pointers named h_* are host memory.
 *   - A table belongs to the GPU that is current when hps_create is called (the one its
 *     storage lives on); make the same device current for every later call on it.  The
 *     library keeps no state outside its tables: several tables, also on several GPUs
 *     of one process, do not interfere.  Calls on ONE table are not thread-safe.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work
 *     on it and return without waiting, except where stated.
 *   - Return value: HPS_OK or a negative hps_status.  Errors that only the device
 *     can see (table full, reserved key) are recorded in a sticky device-side
 *     status word; the kernels of later calls do nothing while it is set, and it
 *     is reported by hps_stats() and cleared by hps_clear_error().
 *   - The key 0xFFFFFFFFFFFFFFFF marks an empty slot and is not a legal key.
 *   - One pull may be outstanding per table (between hps_pull and hps_push); another
 *     pull before that push is refused (HPS_ESTATE).  In addition one mini-batch may be
 *     "prepared" (its key dedup done ahead of time, see hps_prepare); the workspace
 *     holds both contexts.
 *   - Calls that touch the table (insert, pull, pull_prepared, push, get, dump) must
 *     be issued on one stream at a time (or be ordered by the caller).  hps_prepare
 *     does not touch the table and may run on another stream; the library orders it
 *     against the calls that share its buffers with HIP events.
 *   - Do not capture hps_prepare / hps_pull / hps_accumulate into a HIP graph for replay:
 *     three things about a dedup are chosen on the host when the call is made and would be
 *     frozen by a capture: which of the three lists of frequent keys its kernels read and
 *     which one the lookup after it fills (a ring, so that a dedup on another stream never
 *     reads a list that is still being written), which form the dedup takes (below), and,
 *     in the plain form, the sequence number that tells its kernels which of the
 *     workspace's hand-off words are theirs.
 *   - The key dedup has two forms with identical results; the library picks one per call
 *     from the mini-batch's size and the table's history.  A table's third and later dedups
 *     use the keys that earlier lookups found frequent and run without any waits between
 *     workgroups (counts per tile, a scan, a scatter; then every region of the array is put
 *     in order inside one workgroup).  The lookups report back, into pinned host memory that
 *     nobody waits for, when the keys did not suit that form, and the next dedups then take
 *     the plain form (radix passes with look-back between tiles), sorting by all 64 key
 *     bits if need be: hps_stats().n_plain_fallbacks, .n_full_fallbacks.
 *   - Environment variables, read by hps_create, for tests and comparison runs:
 *     HPS_DEDUP = "radix" | "bucket" pins the dedup's form; HPS_RANK = "ballot" ranks the
 *     elements of a sort tile with wave ballots even where the GPU's LDS atomics would
 *     serve (the faster way; hps_create checks on every GPU that they answer the lanes of
 *     an instruction in lane order, and uses ballots where they do not); HPS_POOL = "lds"
 *     makes the pooling kernel keep the most frequent keys' rows in LDS (measured slower);
 *     HPS_ROWS = "apart" keeps weights and accumulators in arrays of their own also where
 *     the library would put them side by side (float32 rows, elementwise Adagrad);
 *     HPS_LOOKUP_NEW_LIST = n makes the pull's lookup use only n entries of the list in
 *     which a workgroup notes the keys it creates (a key that finds it full gets its initial
 *     row on the spot: the test of that path).
 */
#ifndef HPS_H_
#define HPS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hps_table hps_table; /* opaque host object, owned by the library */

typedef enum {
  HPS_OK = 0,
  HPS_EINVAL = -1,    /* bad argument (null/misaligned pointer, size out of range) */
  HPS_EFULL = -2,     /* more keys than the table's capacity                        */
  HPS_ERESERVED = -3, /* the reserved key appeared in the input                     */
  HPS_ESTATE = -4,    /* push without an outstanding pull, or similar misuse        */
  HPS_EDEVICE = -5,   /* a HIP call failed / no usable GPU; as sticky device status: an
                         internal wait between workgroups gave up (never expected)     */
  HPS_ENOMEM = -6     /* storage or workspace buffer too small                      */
} hps_status;

typedef enum {
  /* G' = G + mean_j(g_j^2), one accumulator per row;  w_j -= lr * g_j / (sqrt(G') + eps) */
  HPS_OPT_ADAGRAD_ROWWISE = 0,
  /* G_j' = G_j + g_j^2, one accumulator per element;  w_j -= lr * g_j / (sqrt(G_j') + eps) */
  HPS_OPT_ADAGRAD_ELEMENTWISE = 1
} hps_opt_kind;

/* How the table stores weights.  Not from the paper, whose rows are float32 (Section 6:
 * 30-60 bytes per parameter); bfloat16 rows halve the bytes per row, so a GPU holds more
 * of the working set.  Every interface stays float32 (pooled rows, gradients, hps_insert /
 * hps_get / hps_dump buffers), and so do the accumulators and all arithmetic: a weight is
 * rounded to the nearest bfloat16 (ties to even) when it is stored, nothing else changes. */
typedef enum {
  HPS_ROWS_F32 = 0,
  HPS_ROWS_BF16 = 1,
  /* float32 rows with each row's accumulator(s) behind its weights, one record per row, the
   * records padded to whole 128-byte memory lines (dim 16, one accumulator per row: 128 bytes
   * per row instead of 68).  Same values as HPS_ROWS_F32; trades HBM capacity for requests:
   * the push finds a row's accumulator in the line it fetches for the weights instead of in a
   * line of its own (this GPU fetches 128 bytes for any part of a line). */
  HPS_ROWS_F32_WIDE = 2
} hps_row_format;

typedef struct {
  int32_t kind;       /* hps_opt_kind */
  float lr;
  float eps;
  float init_acc;     /* accumulator value of a newly created row                  */
  float init_range;   /* new weights are uniform on [-init_range, init_range)      */
  int32_t row_format; /* hps_row_format                                            */
  uint64_t init_seed; /* new row = function of (key, init_seed) only               */
} hps_optimizer;

typedef struct {
  uint64_t size;            /* keys currently stored                               */
  uint64_t capacity;        /* maximum number of keys                              */
  uint64_t n_slots;         /* slots of the open-addressing array (capacity / 0.7) */
  uint64_t last_n_keys;     /* key occurrences of the last pull                    */
  uint64_t last_n_unique;   /* unique keys of the last pull                        */
  uint64_t last_n_inserted; /* keys the last pull (or insert) created              */
  uint64_t last_n_absent;   /* distinct keys the last hps_accumulate did not find  */
  uint64_t n_plain_fallbacks; /* times the dedup went back to its plain form for a while
                               because the keys did not suit the bucket form          */
  uint64_t n_full_fallbacks;  /* times the dedup's plain form went over to sorting by all
                               64 key bits for a while (keys in clusters far apart)   */
  double load_factor;       /* size / n_slots                                      */
  int32_t error;            /* sticky device status (0 or a negative hps_status)   */
  int32_t pull_outstanding; /* 1 between a pull and its push                       */
} hps_stats_t;

/* Bytes of device memory the table needs (keys, rows, accumulators, status);
 * 0 if the arguments are invalid.  Section 4.1: capacity is fixed at construction. */
size_t hps_table_bytes(uint64_t capacity_keys, uint32_t dim, const hps_optimizer* opt);

/* Bytes of device workspace for pulls of at most max_keys key occurrences in at
 * most max_bags bags; 0 if the arguments are invalid. */
size_t hps_workspace_bytes(uint64_t max_keys, uint64_t max_bags, uint32_t dim);

/* Section 4.1 "Local GPU hash table": builds an empty table in caller memory.
 *   capacity_keys  maximum number of keys ever stored (1 .. 2^32 * 0.69)
 *   dim            floats per embedding row; a multiple of 4, at most 1024
 *   d_storage      >= hps_table_bytes() bytes; d_workspace >= hps_workspace_bytes()
 *   max_keys       largest n_keys a pull may pass (< 2^30); max_bags likewise
 * Enqueues the clearing of the slot array on `stream`.  *out is set on success and
 * must be released with hps_destroy (which frees host memory only).
 * Errors: HPS_EINVAL, HPS_ENOMEM, HPS_EDEVICE. */
hps_status hps_create(hps_table** out, uint64_t capacity_keys, uint32_t dim,
                      const hps_optimizer* opt, void* d_storage, size_t storage_bytes,
                      void* d_workspace, size_t workspace_bytes, uint64_t max_keys,
                      uint64_t max_bags, void* stream);

/* Algorithm 1 builds the HBM table anew for every batch of its outer loop (insert the
 * batch's working parameters, run the mini-batches, hand the updates to the host tier):
 * empties the table for the next batch -- every key, the sticky status and the counters;
 * optimizer, pooling and row format stay.  Enqueues the clearing of the slot array on
 * `stream`.  Errors: HPS_ESTATE between hps_prepare / a pull and its push. */
hps_status hps_clear(hps_table* t, void* stream);

/* Section 4.1 "insert" / Algorithm 1 insert_into_hashtable: bulk load of n keys.
 *   d_weights [n, dim] or NULL, d_acc [n, acc_len] or NULL (acc_len = 1 row-wise,
 *   dim element-wise).
 * d_weights == NULL: an absent key gets its deterministic initial row, a present
 * key is left untouched.  d_weights != NULL: the row is created or overwritten
 * (accumulators from d_acc, or init_acc when d_acc is NULL); keys must then be
 * distinct within the call.  n may exceed max_keys.  Device errors: HPS_EFULL,
 * HPS_ERESERVED (sticky). */
hps_status hps_insert(hps_table* t, const uint64_t* d_keys, uint64_t n, const float* d_weights,
                      const float* d_acc, void* stream);

/* Algorithm 1 pull_HBM-PS_kernel.
 *   d_keys    [n_keys] feature keys of the mini-batch, bag after bag
 *   d_offsets [n_examples * n_slots + 1] int32, CSR over the bags in (example, slot)
 *             row-major order: offsets[0] = 0, non-decreasing, last = n_keys
 *   d_pooled  [n_examples * n_slots, dim] float32 out: sum of the rows of each bag
 *             (an empty bag gives zeros; a key repeated in a bag counts each time)
 * Keys not in the table are inserted with their initial row before pooling.
 * n_keys <= max_keys and n_examples * n_slots <= max_bags, else HPS_EINVAL.
 * All buffers must stay valid until the work enqueued here has run; d_keys and
 * d_offsets are not needed by the later push.  HPS_ESTATE while an earlier pull still
 * waits for its push: one mini-batch at a time is between pull and push. */
hps_status hps_pull(hps_table* t, const uint64_t* d_keys, uint64_t n_keys,
                    const int32_t* d_offsets, uint32_t n_examples, uint32_t n_slots,
                    float* d_pooled, void* stream);

/* The dedup half of a pull, ahead of time (Section 3's prefetch pipeline: the next
 * mini-batch is made ready while the GPU still works on the current one).  Orders the
 * keys, finds the unique keys, ranks and grouping of the mini-batch into the context
 * that the outstanding pull does not use; reads no table row.  May be called between
 * hps_pull and hps_push of the previous mini-batch, on any stream.  A second
 * hps_prepare before hps_pull_prepared replaces the first.  d_offsets must stay valid
 * until the work of the matching hps_pull_prepared has run.  Arguments as hps_pull. */
hps_status hps_prepare(hps_table* t, const uint64_t* d_keys, uint64_t n_keys,
                       const int32_t* d_offsets, uint32_t n_examples, uint32_t n_slots,
                       void* stream);

/* The table half of a pull for the prepared mini-batch: makes `stream` wait for the
 * prepare, looks up / inserts the unique keys and pools into d_pooled.  The prepared
 * mini-batch becomes the outstanding pull.  hps_pull(...) is hps_prepare followed by
 * hps_pull_prepared on the same stream.  HPS_ESTATE if nothing is prepared, or while an
 * earlier pull still waits for its push. */
hps_status hps_pull_prepared(hps_table* t, float* d_pooled, void* stream);

/* Algorithm 1 push_parameters_updates_back_kernel / Algorithm 2's local accumulate.
 *   d_pooled_grads [n_bags, dim]: gradient of the loss w.r.t. d_pooled of the
 *   outstanding pull.
 * Each unique key's gradient is the sum over its occurrences of its bag's
 * gradient row; each touched row takes one optimizer step.  Ends the pull.
 * Errors: HPS_ESTATE when no pull is outstanding. */
hps_status hps_push(hps_table* t, const float* d_pooled_grads, void* stream);

/* Pooling of the bags: 0 = sum (the default), 1 = mean: the pooled row is the average of
 * the bag's rows (an empty bag still gives zeros), and in the push every occurrence
 * receives its bag's gradient row divided by the bag's length.  Not from the paper, which
 * leaves the reduction over a slot's features to the trainer; offered because averaged
 * slots are the other common embedding-layer form.  Takes effect from the next
 * hps_prepare / hps_pull on.  Errors: HPS_ESTATE between hps_prepare / a pull and its push. */
hps_status hps_set_pooling(hps_table* t, int mean);

/* Section 4.1 "accumulate" in the paper's literal form (Algorithm 2's per-GPU accumulate):
 * the input is a collection of (key, value row) pairs and every value row is added onto
 * the weights its key references.
 *   d_keys   [n] (device, 8-byte aligned), d_values [n, dim] float32 (device, 16-byte aligned)
 * A key that comes several times receives the sum of its rows (fixed-shape fp32 sums,
 * no floating-point atomics: two runs give the same bits).  Keys the table does not hold
 * are skipped, nothing is created; hps_stats().last_n_absent counts them.  Optimizer
 * state is not touched; touched rows count as updated for hps_dump_dirty.
 * Errors: HPS_ESTATE between hps_prepare / a pull and its push; HPS_EINVAL for
 * n > max_keys; HPS_ERESERVED (sticky, nothing is added) if a key is all ones. */
hps_status hps_accumulate(hps_table* t, const uint64_t* d_keys, uint64_t n, const float* d_values,
                          void* stream);

/* For callers that cannot allocate device memory or hand over a workspace of their own (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation): the same
 * operation as hps_accumulate, with the call's scratch data (the sorted pairs, the unique keys,
 * their rows, the work lists) in a device array that is part of the library's code object
 * instead of the table's workspace -- 10 MiB per GPU the library runs on, held until the
 * process ends.  The call allocates nothing, on the device or through the HIP runtime.
 *   n <= HPS_STATIC_MAX_KEYS, else HPS_EINVAL; other arguments and results as hps_accumulate.
 * All tables of a GPU share that GPU's array, and a call leaves its contents behind: the call
 * clears what it needs cleared, but two calls that overlap on one GPU (different streams or
 * threads, also on different tables) race.  Issue it on the stream of the table's other calls.
 * Its key dedup always takes the plain form over all 64 key bits, whatever the table's history. */
#define HPS_STATIC_MAX_KEYS 65536u
hps_status hps_accumulate_static(hps_table* t, const uint64_t* d_keys, uint64_t n,
                                 const float* d_values, void* stream);

/* Section 3 "union of the referenced parameters": copies the outstanding pull's
 * ascending unique keys (d_uniq_out, room for n_keys) and per-occurrence ranks
 * (d_inverse_out [n_keys] int32, uniq[inverse[i]] == keys[i]); either may be NULL.
 * The unique count is hps_stats().last_n_unique. */
hps_status hps_last_unique(hps_table* t, uint64_t* d_uniq_out, int32_t* d_inverse_out,
                           void* stream);

/* Section 4.1 "get": reads rows by key without inserting.
 *   d_weights_out [n, dim], d_acc_out [n, acc_len], d_found_out [n] uint8;
 *   rows of absent keys are left unwritten, found = 0. */
hps_status hps_get(hps_table* t, const uint64_t* d_keys, uint64_t n, float* d_weights_out,
                   float* d_acc_out, uint8_t* d_found_out, void* stream);

/* Algorithm 1 pull_updates_HBM-PS: writes every stored (key, row, accumulator) in
 * unspecified order, at most max_rows of them; *h_n_rows (host) gets the number of
 * stored keys.  Waits for the stream.  HPS_ENOMEM if max_rows was too small (the
 * first max_rows found are written). */
hps_status hps_dump(hps_table* t, uint64_t* d_keys_out, float* d_weights_out, float* d_acc_out,
                    uint64_t max_rows, uint64_t* h_n_rows, void* stream);

/* Section 4 / Algorithm 1's last step, incremental: the host tier collects the UPDATES of
 * the HBM tier.  Like hps_dump, but only rows that a push or an accumulate has changed
 * since the previous hps_dump_dirty (or since creation); the marks of the rows written
 * out are cleared.  Rows that were only inserted, or only created by a pull, are not
 * updates.  HPS_ENOMEM if max_rows was too small: the first max_rows found are written
 * and unmarked, the others stay marked.  HPS_ESTATE between a pull and its push. */
hps_status hps_dump_dirty(hps_table* t, uint64_t* d_keys_out, float* d_weights_out,
                          float* d_acc_out, uint64_t max_rows, uint64_t* h_n_rows, void* stream);

/* Waits for the stream and fills *h_out (host). */
hps_status hps_stats(hps_table* t, hps_stats_t* h_out, void* stream);

/* Section 4.1: the table is open-addressing with linear probing over lines of eight slots; a
 * key's sequence starts at an even line, so that its first two lines are one 128-byte memory
 * line (a bucket of sixteen slots, which a lookup reads at once).
 * Scans the whole slot array and reports how many buckets a lookup reads to find a stored key
 * (1 = the key sits in the bucket its hash names): the mean over all stored keys and the most
 * for one key (0 and 0 for an empty table).  Waits for the stream.  A diagnostic: it reads every
 * slot key, 8 bytes per slot. */
hps_status hps_probe_lengths(hps_table* t, double* h_mean, uint64_t* h_max, void* stream);

/* Clears the sticky device status and abandons the mini-batch between hps_prepare / a
 * pull and its push, if there is one: while the status was set its kernels did nothing,
 * so there is nothing valid to push (a later hps_push returns HPS_ESTATE). */
hps_status hps_clear_error(hps_table* t, void* stream);

/* Frees the host object; device memory stays with the caller. */
hps_status hps_destroy(hps_table* t);

const char* hps_strerror(hps_status s);

#ifdef __cplusplus
}
#endif
#endif /* HPS_H_ */
