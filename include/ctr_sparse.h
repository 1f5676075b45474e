/*
 * ctr_sparse.h - C ABI of the single-GPU sparse embedding cycle (MI355X / gfx950).
 *
 * One mini-batch cycle of a CTR model's embedding layer on one GPU's shard of
 * the parameter server: look up 64-bit feature keys in an HBM-resident hash
 * table (inserting unseen keys), sum-pool the rows per (sample, slot), and on
 * the way back reduce the pooled gradients per distinct key and apply one
 * sparse Adam step to the touched rows; with several model replicas on the
 * device, merge them every k steps.
 *
 * The calls mirror the per-mini-batch steps of the paper's training workflow
 * (Algorithm 1: insert into the GPU hash table, pull, train, push) and its
 * k-step Adam (Algorithm 2).
 *
 * Conventions
 *  - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  Every
 *    device buffer (table storage, workspace, keys, offsets, pooled, grads) is
 *    allocated by the caller and only borrowed; the library allocates no device
 *    memory and frees none.  ctr_table / ctr_batch are small host objects owned
 *    by the library.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *    ctr_pull_pool, ctr_push_adam and ctr_kstep_merge only enqueue work on it
 *    and return; they never synchronise.  The export/size/status calls
 *    synchronise the stream they are given.
 *  - Every call returns a ctr_status.  Errors the host can see (null pointers,
 *    bad sizes, workspace too small, a stale batch) are returned at once and
 *    change nothing.  Errors only the device can see (reserved key in the
 *    input, table full, malformed offsets) are recorded in a device status
 *    word; the pull that hit one leaves the table exactly as it was (tentative
 *    inserts are rolled back), its `pooled` output is unspecified, the push
 *    that consumes its batch is a no-op, and the code is returned (and cleared)
 *    by ctr_last_status.  While the status word is set, later pulls, pushes
 *    and merges are no-ops too.
 *  - Determinism: the same call sequence on the same inputs gives bit-identical
 *    key->row assignment (new keys take consecutive rows in order of their
 *    first occurrence in the batch), unique sets and pooled/updated values.
 *  - Limits: dim a multiple of 4 and <= 256; capacity_rows <= 2^30 and at most
 *    2^30 index slots (the power of two >= capacity_rows / load_factor: 2^29
 *    rows at a load factor of 0.5); n_keys < 2^31 per call; n_replicas <= 31.
 *  - Calls on one table must be issued from one host thread at a time and on
 *    one stream (or on streams the caller has ordered).
 */
#ifndef CTR_SPARSE_H
#define CTR_SPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ctr_table ctr_table; /* opaque host-side handle */
typedef struct ctr_batch ctr_batch; /* opaque token for the dedup result of one pull: never dereferenced by the
                                       caller, never reused by the table, so a stale one is always recognised */

typedef enum {
  CTR_OK = 0,
  CTR_E_INVAL = 1,  /* bad argument / malformed offsets */
  CTR_E_NOMEM = 2,  /* caller-provided table memory or workspace too small */
  CTR_E_FULL = 3,   /* the pull would need more than capacity_rows rows */
  CTR_E_BADKEY = 4, /* input holds the reserved key 0xFFFFFFFFFFFFFFFF */
  CTR_E_STATE = 5,  /* push without a matching live pull */
  CTR_E_DEVICE = 6  /* a HIP runtime call failed */
} ctr_status;

/* flags (ctr_config.flags) */
#define CTR_F_KSTEP 1u /* k-step Adam of Algorithm 2: shared frozen denominator + merge */
/* Rows hold [x | G] and are updated by AdaGrad, the optimizer the paper uses for its sparse
 * parameters (Section 5, to save the first moment): G += g^2; x -= lr g / sqrt(G), with G = eps
 * in a new row (eps placed as in Algorithm 2's "Initialize").  Single table only (no other flag,
 * n_replicas = 1). */
#define CTR_F_ADAGRAD 2u
/* With CTR_F_KSTEP: the reading of Section 4's prose instead of the printed Algorithm 2 - every
 * step, the k-th included, is a local step x -= lr m / sqrt(own v) (CTR_STEP_MERGE_PENDING is
 * rejected), and the merge sets every replica's x to the mean of the x_j and every v_j to the
 * mean of the v_j.  There is no shared-denominator array. */
#define CTR_F_KSTEP_PROSE 4u
/* The Adam the paper cites (Kingma & Ba) instead of Algorithm 2's form: m = v = 0 in a new row,
 * x -= lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps), t = number of ctr_push_adam calls
 * accepted by this table so far (rows not in a batch are untouched).  Single table only. */
#define CTR_F_BIAS_CORRECTION 8u

/* step modes for ctr_push_adam */
#define CTR_STEP_LOCAL 0u         /* t mod k != 0 (or single-table mode): moments and model */
#define CTR_STEP_MERGE_PENDING 1u /* t mod k == 0: moments only; the model update of this step \
                                     is applied inside the next ctr_kstep_merge */

typedef struct {
  uint64_t capacity_rows; /* R: value rows; the key index has pow2ceil(R / load_factor) slots */
  uint32_t dim;           /* D: floats per embedding row */
  float load_factor;      /* in (0, 0.9]; 0 selects 0.5 */
  uint32_t n_replicas;    /* W >= 1 model replicas sharing one key->row index (W > 1 needs CTR_F_KSTEP) */
  float lr, beta1, beta2, eps; /* alpha, beta_1, beta_2, epsilon of Algorithm 2 */
  uint64_t init_seed;     /* seed of the deterministic row initialiser */
  float init_std;         /* spread of a new row's parameters */
  uint32_t flags;         /* CTR_F_* */
} ctr_config;

/* Bytes of device memory a table with this configuration needs (0 if the
 * configuration is invalid).  The caller allocates them (256-byte aligned)
 * and passes them to ctr_table_create. */
size_t ctr_table_bytes(const ctr_config* cfg);

/* Bytes of device workspace needed by a pull/push pair of at most `max_keys`
 * key occurrences in `max_segments` segments (0 if invalid). */
size_t ctr_workspace_bytes(const ctr_config* cfg, uint64_t max_keys, uint32_t max_segments);

/* Creates an empty table in caller-provided device memory (Algorithm 1: the
 * per-GPU HBM hash table that receives the working parameters; Algorithm 2,
 * "Initialize", fixes the state of a row when it is created: m = 0, v = eps).
 * Enqueues the clearing of the key index on `hip_stream`.
 * d_mem: device, >= ctr_table_bytes(cfg) bytes, 256-byte aligned, must outlive
 * the table.  *out receives the handle.  Errors: CTR_E_INVAL, CTR_E_NOMEM,
 * CTR_E_DEVICE. */
int ctr_table_create(const ctr_config* cfg, void* d_mem, size_t bytes, void* hip_stream,
                     ctr_table** out);

/* Releases the host handle (and any live batch).  Never touches d_mem. */
int ctr_table_destroy(ctr_table* t);

/* Pull (Algorithm 1: insert_into_hash_table + pull for one mini-batch; the
 * training workflow's "union of the referenced parameters"; the embedding
 * layer of Section 2.1 with per-slot sum pooling).
 *   d_keys[n_keys]        device, uint64 feature keys in CSR order
 *   d_offsets[n_seg + 1]  device, uint32 CSR boundaries, offsets[0] = 0,
 *                         non-decreasing, offsets[n_seg] = n_keys
 *   d_pooled[n_seg * D]   device, out: pooled[g, :] = sum of replica `replica`'s
 *                         rows of the keys in segment g (zeros if empty)
 *   d_workspace           device, >= ctr_workspace_bytes(cfg, n_keys, n_seg),
 *                         256-byte aligned; owned by the returned batch until
 *                         the batch is pushed or the next pull on this table
 *   *batch_out            handle to the dedup result, consumed by ctr_push_adam
 * Unseen keys are inserted (rows created in all replicas).  A previous batch
 * of this table that was not pushed becomes stale.
 * Errors: CTR_E_INVAL, CTR_E_NOMEM (workspace); deferred: CTR_E_INVAL
 * (offsets), CTR_E_BADKEY, CTR_E_FULL. */
int ctr_pull_pool(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                  const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled,
                  void* d_workspace, size_t workspace_bytes, ctr_batch** batch_out,
                  void* hip_stream);

/* The same pull with the pooled embeddings also (or only) written as bfloat16, the operand type
 * of the dense tower's matrix products (ctr_mlp_step_bf16), so that no separate conversion pass
 * over the pooled tensor is needed between pull and train_mini-batch (Algorithm 1).
 *   d_pooled_bf16[n_seg * D]  device, out, 8-byte aligned: the fp32 pooled value rounded to bf16
 *                             (nearest-even), bit-identical to converting d_pooled afterwards
 *   d_pooled                  device, out, may be NULL when only the bf16 copy is wanted
 * Everything else as ctr_pull_pool. */
int ctr_pull_pool_bf16(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                       const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled,
                       uint16_t* d_pooled_bf16, void* d_workspace, size_t workspace_bytes,
                       ctr_batch** batch_out, void* hip_stream);

/* Lookup-only pooling, for prediction with a trained table (the embedding layer of Section 2.1
 * without the insert-on-miss of the training workflow): pooled[g, :] = sum of the rows of the keys
 * of segment g that ARE in the table; absent keys contribute nothing and are not inserted.  Table,
 * counters and optimizer state are untouched and no batch handle is produced.  Either output may
 * be NULL (not both).  The workspace (sized as for ctr_pull_pool) is overwritten: if it is the one
 * a live batch owns, that batch goes stale.  Errors as ctr_pull_pool, except that the table cannot
 * become full. */
int ctr_lookup_pool(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                    const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled,
                    uint16_t* d_pooled_bf16, void* d_workspace, size_t workspace_bytes,
                    void* hip_stream);

/* ctr_lookup_pool for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The two per-occurrence lists
 * that ctr_lookup_pool keeps in the caller's workspace live in a fixed device array inside the library
 * instead (CTR_NOALLOC_SCRATCH_BYTES = 32 MiB, held on every GPU that loads the library until the
 * process ends; its address is looked up per device by ctr_table_create or by the first call).  The
 * call makes no hipMalloc / hipFree and no allocating library call, records no stage timers, and only
 * enqueues kernels on `hip_stream`.
 *   n_keys <= CTR_NOALLOC_MAX_KEYS, else CTR_E_NOMEM (nothing is enqueued)
 * Arguments, results and the other errors as ctr_lookup_pool; outputs are bit-identical to it.
 * All calls on one GPU share that GPU's array (also calls on different tables), which keeps the
 * previous call's lists: each call overwrites the entries of its own n_keys occurrences before
 * reading them, so nothing has to be cleared, but two calls that overlap in time on one GPU
 * (different streams without ordering, different threads) race.  A live batch of a pull is not
 * affected. */
#define CTR_NOALLOC_MAX_KEYS (1u << 22)
#define CTR_NOALLOC_SCRATCH_BYTES ((size_t)CTR_NOALLOC_MAX_KEYS * 2u * sizeof(uint32_t))
int ctr_lookup_pool_noalloc(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                            const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled,
                            uint16_t* d_pooled_bf16, void* hip_stream);

/* Push (Algorithm 1: push_parameters_updates_back; Algorithm 2: the m, v and
 * model lines).  The gradient of sum pooling hands grad_pooled[g, :] to every
 * key occurrence of segment g; per distinct key the occurrences' gradients are
 * summed and ONE Adam step is applied to that key's row of replica `replica`:
 *   m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;  x -= lr m / sqrt(den)
 * with den = v (single-table mode) or the shared denominator frozen at the
 * last merge (CTR_F_KSTEP, CTR_STEP_LOCAL); with CTR_STEP_MERGE_PENDING only
 * m and v change.  CTR_F_ADAGRAD, CTR_F_KSTEP_PROSE and CTR_F_BIAS_CORRECTION
 * select the row updates described at their definitions.  Rows not in the
 * batch are untouched.
 *   d_grad_pooled[n_seg * D]  device, in
 * `batch` must be the live batch of the last pull on `t` with the same
 * replica; it is consumed (freed) whatever the outcome, unless CTR_E_INVAL.
 * Errors: CTR_E_INVAL, CTR_E_STATE. */
int ctr_push_adam(ctr_table* t, uint32_t replica, ctr_batch* batch, const float* d_grad_pooled,
                  uint32_t mode, void* hip_stream);

/* ctr_push_adam with the pooled gradients held as bfloat16 (the 16 high bits of the fp32 value
 * they stand for; 8-byte aligned): what a bf16 tower hands back when it writes the input gradient
 * in its own precision.  Every value is widened exactly and summed in binary64 like an fp32 one,
 * so the result is that of ctr_push_adam on the widened gradients; each occurrence reads half the
 * bytes.
 *   d_grad_pooled_bf16[n_seg * D]  device, in */
int ctr_push_adam_bf16(ctr_table* t, uint32_t replica, ctr_batch* batch, const uint16_t* d_grad_pooled_bf16,
                       uint32_t mode, void* hip_stream);

/* k-step merge (Algorithm 2, "global averaging" branch), over every row touched
 * by any replica since the previous merge:
 *   vhat = (1/W) sum_j v_j;
 *   x_i  = (1/W) sum_j (x_j - [row pending in j] lr m_j / sqrt(vhat))   for all i.
 * m_j and v_j stay local.  With CTR_F_KSTEP_PROSE instead: x_i = (1/W) sum_j x_j
 * and v_i = (1/W) sum_j v_j for all i.  Needs CTR_F_KSTEP.  Errors: CTR_E_INVAL. */
int ctr_kstep_merge(ctr_table* t, void* hip_stream);

/* Working-set load (Algorithm 1: partition_parameters_to_GPUs + insert_into_hash_table): places
 * the parameters of a batch's working set, as handed over by the host-side tiers, in the table.
 *   d_keys[n_keys]                  device, distinct keys (a repeated key makes its row's
 *                                   contents unspecified)
 *   d_x, d_m, d_v[n_keys * D]       device, the rows' state (d_m ignored and may be NULL under
 *                                   CTR_F_ADAGRAD, where d_v is the accumulator)
 *   d_workspace                     device, >= ctr_workspace_bytes(cfg, n_keys, 0), 256-byte aligned
 * Keys not yet in the table get new rows (numbered in the order given); keys already there have
 * their rows overwritten.  Every replica receives the same state; Algorithm 2's shared denominator
 * of the row is set to v.  A live batch of this table goes stale.  Enqueues only.
 * Errors: CTR_E_INVAL, CTR_E_NOMEM; deferred: CTR_E_BADKEY, CTR_E_FULL (nothing is loaded). */
int ctr_table_load(ctr_table* t, const uint64_t* d_keys, uint64_t n_keys, const float* d_x, const float* d_m,
                   const float* d_v, void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Empties the table without giving up its memory (Algorithm 1's outer loop: the hash table holds
 * the working parameters of one batch; the next batch loads its own with ctr_table_load): no keys,
 * no rows, no pending merge steps, device status cleared.  Row storage is not wiped: rows are
 * (re)initialised when keys are inserted again.  A live batch goes stale.  The step count of the
 * bias-corrected form keeps running.  Enqueues only.  Errors: CTR_E_INVAL, CTR_E_DEVICE. */
int ctr_table_clear(ctr_table* t, void* hip_stream);

/* Collection of updated rows (Algorithm 1: pull_updates_peer_GPU, the step that hands the batch's
 * parameters back to the host-side tiers): looks up n_keys keys WITHOUT inserting and copies the
 * rows of replica `replica` to dense device arrays (any of d_x, d_m, d_v, d_found may be NULL;
 * d_m must be NULL under CTR_F_ADAGRAD).  d_found[p] = 1 if keys[p] is in the table, else 0 and
 * its output rows are zeros.  Enqueues only.  Errors: CTR_E_INVAL. */
int ctr_table_collect(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys, float* d_x,
                      float* d_m, float* d_v, uint32_t* d_found, void* hip_stream);

/* ---- parity / debug surface (synchronising, not part of the timed path) ---- */

/* Number of rows in use. */
int ctr_table_size(ctr_table* t, uint64_t* n_rows, void* hip_stream);

/* Table contents in row order into HOST buffers (any may be NULL):
 * h_keys[n_rows], h_x/h_m/h_v[n_rows * D] of one replica (h_v is the AdaGrad
 * accumulator under CTR_F_ADAGRAD, where asking for h_m is CTR_E_INVAL),
 * h_vhat[n_rows * D] (Algorithm 2's shared denominator: CTR_F_KSTEP without
 * CTR_F_KSTEP_PROSE only, else CTR_E_INVAL if requested). */
int ctr_table_export(ctr_table* t, uint32_t replica, uint64_t* h_keys, float* h_x, float* h_m,
                     float* h_v, float* h_vhat, void* hip_stream);

/* Dedup result of a live batch in canonical form into HOST buffers (any may be
 * NULL): *n_unique; h_uniq[n_unique] distinct keys ascending; h_rows[n_unique]
 * their row ids; h_inverse[n_keys] index of each occurrence's key in h_uniq.
 * Call with NULL arrays first to learn n_unique. */
int ctr_batch_export(ctr_table* t, ctr_batch* batch, uint64_t* n_unique, uint64_t* h_uniq,
                     uint32_t* h_rows, uint32_t* h_inverse, void* hip_stream);

/* Counters of the last pull/push pair: distinct keys in the batch (valid after
 * the push) and rows created by the pull. */
int ctr_batch_stats(ctr_table* t, uint64_t* n_unique, uint64_t* n_new, void* hip_stream);

/* Rows averaged by all ctr_kstep_merge calls on this table so far (a merge covers the rows touched
 * by any replica since the merge before; Algorithm 2, global-averaging branch) and, in
 * *pending_applied (may be NULL), the number of (row, replica) pairs whose deferred k-th step those
 * merges applied: the unit counts of the merge's byte accounting.  Reset by ctr_table_clear. */
int ctr_merge_stats(ctr_table* t, uint64_t* rows_merged, uint64_t* pending_applied, void* hip_stream);

/* Measurement aid, no part of the method: enqueues a plain streaming copy of `bytes` bytes (a multiple
 * of 16; both pointers device, 16-byte aligned, not overlapping) with the library's own copy kernel,
 * so that a benchmark can report the kernels' rates against this GPU's practical copy rate measured
 * in the same run, beside the published peak.  non_temporal != 0 uses streaming loads and stores.
 * Errors: CTR_E_INVAL. */
int ctr_stream_copy(void* d_dst, const void* d_src, size_t bytes, int non_temporal, void* hip_stream);

/* Returns the deferred device status (a ctr_status) and clears it. */
int ctr_last_status(ctr_table* t, void* hip_stream);

/* ---- stage timers (measurement aid) ---- */

#define CTR_STAGE_PROBE 0   /* key probe / tentative insert */
#define CTR_STAGE_INSERT 1  /* ranking of new keys, row creation */
#define CTR_STAGE_POOL 2    /* row gather + per-segment sum */
#define CTR_STAGE_SORT 3    /* grouping of occurrences by row */
#define CTR_STAGE_PUSH 4    /* gradient segment-reduce fused with Adam */
#define CTR_STAGE_FIXUP 5   /* rows whose occurrences span several work spans */
#define CTR_STAGE_MERGE 6   /* k-step merge */
#define CTR_STAGE_ORDER 7   /* execution order of the push's work spans (large gradient arrays only) */
#define CTR_N_STAGES 8

/* Test hook: fixes the work geometry of later pulls and pushes instead of letting the batch size
 * choose it (span: occurrences per work span of the push, 16/32/64/128; probe_items: occurrences
 * per thread of the probe, 1 or 8; 0 = by batch size), so that every code path can be exercised
 * on small inputs.  Results do not depend on the geometry.  A geometry that needs more workspace
 * than the call was given makes the call return CTR_E_NOMEM.  Errors: CTR_E_INVAL. */
int ctr_debug_set_geometry(ctr_table* t, uint32_t span, uint32_t probe_items);

/* Measurement and test hook: the order in which later pushes run their work spans (Algorithm 1's push
 * step; results do not depend on it).  windows = 0: list order.  windows = 2..128 (a power of two): the
 * spans that lie inside one row - gradient gathers in ascending segment order - run first, grouped by which
 * of `windows` equal parts of the gradient array they begin in, so that the spans in flight together gather
 * from one part and the second use of a gradient row finds it in the last-level cache; the others follow in
 * list order.  split_launch = 1: those spans get a launch of their own; 2: one launch, the other spans dealt
 * evenly between the parts.  Pushes whose gradient array is smaller than min_grad_bytes keep the list order.
 * A new table starts with 32 windows, one launch, 256 MiB.  Errors: CTR_E_INVAL. */
int ctr_debug_set_push_order(ctr_table* t, uint32_t windows, uint32_t split_launch, uint64_t min_grad_bytes);

/* When enabled, a pair of HIP events is recorded around each stage of the
 * following calls, on the stream they run on (one pair per execution). */
int ctr_profile_enable(ctr_table* t, int on);
/* Synchronises the device, writes per stage the summed milliseconds
 * (h_ms[CTR_N_STAGES]) and the number of executions (h_count[CTR_N_STAGES],
 * may be NULL) recorded since the previous read, and starts a new record. */
int ctr_profile_read(ctr_table* t, float* h_ms, uint32_t* h_count);

#ifdef __cplusplus
}
#endif
#endif /* CTR_SPARSE_H */
