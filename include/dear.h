/*
 * dear.h -- C ABI of the MI355X (gfx950) gradient-aggregation path of DeAR
 * (decoupled all-reduce: reduce-scatter during back-propagation, all-gather during the
 * next feed-forward, with threshold tensor fusion).
 *
 * One GPU emulates P data-parallel workers: worker p's per-layer gradient tensors and
 * per-layer parameter tensors are P separate sets of device buffers.  Per fusion group
 * ("bucket") the library
 *   1. reduce-scatters the P gradient replicas into P shards (ring summation order,
 *      1/P average),
 *   2. applies SGD with momentum to each owned shard,
 *   3. all-gathers the updated shards back into all P replicas' per-layer tensors.
 *
 * Conventions
 *   - Every function returns a status (DEAR_OK = 0, errors < 0); nothing is printed,
 *     nothing aborts.  On error nothing is launched and outputs are untouched.
 *   - "host" / "device" is stated for every pointer.  All large device memory is owned
 *     by the caller; the library owns only its plan/context objects and their small
 *     tables (host and device), released by dear_plan_free / dear_ctx_destroy.
 *   - Kernel calls enqueue on the given HIP stream (a hipStream_t passed as void*,
 *     NULL = default stream) and return without synchronising.
 *   - Layers are indexed in forward order (0 = first layer).  Buckets are indexed in
 *     the order their gradients become ready (bucket 0 holds the LAST layers).
 *   - A plan or context may be used by one thread at a time.
 */
#ifndef DEAR_H
#define DEAR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    DEAR_OK = 0,
    DEAR_EINVAL = -1, /* null pointer, non-positive size, unknown dtype, ...        */
    DEAR_ENOMEM = -2, /* host or device allocation of a library table failed       */
    DEAR_EHIP = -3,   /* a HIP call or a kernel launch reported an error           */
    DEAR_ERANGE = -4, /* bucket / worker index outside the plan                    */
    DEAR_EALIGN = -5, /* a device pointer is not aligned as documented             */
    DEAR_ETOOBIG = -6 /* input exceeds the static device scratch (see below)       */
};

enum { DEAR_F32 = 0, DEAR_BF16 = 1 }; /* gradient element type */

/* fusion_threshold_bytes = DEAR_NO_LIMIT puts every layer into one bucket;
 * fusion_threshold_bytes = 0 gives every layer a bucket of its own (no tensor fusion). */
#define DEAR_NO_LIMIT INT64_MAX

/* Shard lengths are rounded up to this many elements (128 bytes of fp32). */
#define DEAR_SHARD_ALIGN 32

typedef struct dear_plan_s dear_plan_t; /* immutable bucket / shard plan, host memory  */
typedef struct dear_ctx_s dear_ctx_t;  /* plan + device tables for one set of tensors */

/* ---------------------------------------------------------------------------------
 * dear_plan -- threshold tensor fusion and chunking.
 *
 * Paper: Section IV-B (consecutive layers form one group while their total number of
 * gradients does not exceed the buffer size x; one reduce-scatter and one all-gather
 * per group), Section III-B (groups are issued last layer -> first layer in the
 * backward pass and in the reverse order in the forward pass; tensors are never
 * partitioned), Section III-A (the d elements of a group are cut into P chunks).
 *
 *   layer_sizes  host, n_layers element counts (each >= 1), forward order
 *   P            number of workers (>= 1)
 *   fusion_threshold_bytes  buffer size x in bytes of the gradient type (>= 0); a group
 *                holds X = floor(x / grad_elem_bytes) elements at most, unless it is a
 *                single layer larger than that
 *   grad_elem_bytes  4 (fp32 gradients) or 2 (bf16 gradients)
 *   out          receives a new plan; release with dear_plan_free
 *
 * Layers are packed densely in arrival order (highest layer index first).  Bucket b
 * with d_b elements gets shard length S_b = ceil(d_b / P) rounded up to
 * DEAR_SHARD_ALIGN; bucket position e belongs to shard e / S_b at slot e % S_b;
 * positions d_b .. P*S_b-1 are padding.
 * Errors: DEAR_EINVAL (bad argument), DEAR_ENOMEM.
 */
int dear_plan(const int64_t *layer_sizes, int32_t n_layers, int32_t P,
              int64_t fusion_threshold_bytes, int32_t grad_elem_bytes, dear_plan_t **out);

/* dear_plan_fixed_layers -- alternative grouping: every bucket holds
 * `layers_per_bucket` (>= 1) consecutive layers in arrival order, the last bucket the
 * remainder (the fixed-number-of-layers fusion the paper compares against in its
 * tensor-fusion study, Section VI-G).  Chunking and all other arguments as dear_plan. */
int dear_plan_fixed_layers(const int64_t *layer_sizes, int32_t n_layers, int32_t P,
                           int32_t layers_per_bucket, int32_t grad_elem_bytes, dear_plan_t **out);

void dear_plan_free(dear_plan_t *plan); /* NULL is ignored */

/* Read-only view of a plan.  All pointers are host memory owned by the plan and stay
 * valid until dear_plan_free. */
typedef struct {
    int32_t n_layers;        /* L */
    int32_t n_buckets;       /* B */
    int32_t P;
    int32_t grad_elem_bytes; /* 2 or 4 */
    int32_t shard_align;     /* DEAR_SHARD_ALIGN */
    int32_t reserved;
    int64_t threshold_bytes;
    int64_t total_elems;     /* N = sum of layer sizes */
    int64_t total_shard_len; /* sum of S_b: length of one worker's row of a shard buffer */
    const int64_t *layer_sizes;        /* [L] */
    const int32_t *layer_bucket;       /* [L] bucket holding layer l                      */
    const int64_t *layer_offset;       /* [L] position of layer l's element 0 in its bucket */
    const int32_t *bucket_first_layer; /* [B] lowest layer index in bucket b              */
    const int32_t *bucket_n_layers;    /* [B] layers bucket_first_layer .. +n_layers-1    */
    const int64_t *bucket_len;         /* [B] d_b                                         */
    const int64_t *bucket_shard_len;   /* [B] S_b                                         */
    const int64_t *bucket_shard_base;  /* [B] start of bucket b inside a worker's row     */
} dear_plan_view_t;

int dear_plan_view(const dear_plan_t *plan, dear_plan_view_t *out);

/* One workgroup's share of a bucket, as the kernels consume it: `count` consecutive
 * elements of ONE layer that all belong to ONE shard (layer >= 0), or a run of padding
 * slots of one shard (layer = -1, src_begin = 0).  Tiles of a bucket are stored in
 * bucket-position order; a layer run is cut at multiples of DEAR_TILE_ELEMS of the
 * layer's own element index, so only the first and last 16-byte vector of a run can be
 * partial. */
#ifndef DEAR_TILE_ELEMS
#define DEAR_TILE_ELEMS 4096
#endif
typedef struct {
    int64_t src_begin; /* first element inside the layer tensor                         */
    int64_t dst_begin; /* element offset inside a shard buffer: row*total_shard_len+...  */
    int32_t count;     /* 1 .. DEAR_TILE_ELEMS                                           */
    int32_t layer;     /* forward layer index, or -1 for padding                         */
    int32_t shard;     /* owning worker s                                                */
    int32_t bucket;
} dear_tile_t;

/* dear_plan_tiles -- the tile table dear_ctx_create uploads, for inspection and tests.
 *   out       host, capacity entries (may be NULL when capacity = 0)
 *   n_tiles   host, receives the number of tiles of the plan (always)
 *   bucket_tile_begin  host, n_buckets+1 entries or NULL: tiles of bucket b are
 *             [bucket_tile_begin[b], bucket_tile_begin[b+1])
 * Writes min(capacity, n_tiles) entries.  Errors: DEAR_EINVAL, DEAR_ENOMEM. */
int dear_plan_tiles(const dear_plan_t *plan, dear_tile_t *out, int64_t capacity, int64_t *n_tiles,
                    int64_t *bucket_tile_begin);

/* ---------------------------------------------------------------------------------
 * dear_ctx_create -- bind a plan to the P x L gradient and parameter tensors.
 *
 *   grad_dtype   DEAR_F32 or DEAR_BF16; must agree with the plan's grad_elem_bytes
 *   grad_ptrs    host array of P*n_layers DEVICE pointers; entry [p*n_layers + l] is
 *                worker p's gradient tensor of layer l (layer_sizes[l] contiguous
 *                elements of grad_dtype)
 *   param_ptrs   host array, same indexing, DEVICE pointers to fp32 parameter tensors
 *   out          receives the context; release with dear_ctx_destroy
 *
 * Every tensor base pointer must be 16-byte aligned (DEAR_EALIGN otherwise).  The two
 * pointer arrays are copied; the tensors themselves stay owned by the caller and must
 * outlive the context.  The context copies what it needs from the plan, so the plan
 * may be freed first.  Allocates device memory for its tables (pointer tables and a
 * tile table of 32 bytes per DEAR_TILE_ELEMS elements).  Uses the current HIP device;
 * every later call on the context must be made with that device current (DEAR_EINVAL
 * otherwise).
 * Errors: DEAR_EINVAL, DEAR_EALIGN, DEAR_ENOMEM, DEAR_EHIP.
 */
int dear_ctx_create(const dear_plan_t *plan, int32_t grad_dtype,
                    const void *const *grad_ptrs, float *const *param_ptrs, dear_ctx_t **out);

void dear_ctx_destroy(dear_ctx_t *ctx); /* NULL is ignored; synchronises the device */

/* dear_ctx_set_max_workgroups -- bound the grid of the kernels launched through this
 * context.  0 (the default) gives every work item its own workgroup, which is fastest
 * when the aggregation has the GPU to itself.  A positive bound (a few hundred; 256 =
 * one per compute unit) makes each workgroup stride over the items; this is meant for
 * the DeAR schedule on one GPU (paper Section III-B), where the reduce-scatter runs
 * beside back-propagation kernels and the all-gather beside feed-forward kernels: a
 * bounded grid disturbs the compute kernels far less.  Results are identical for every
 * setting.  Takes effect for calls made afterwards.
 * Errors: DEAR_EINVAL (null context, negative bound). */
int dear_ctx_set_max_workgroups(dear_ctx_t *ctx, int32_t max_workgroups);

/* dear_ctx_set_wave_priority -- wave priority (0..3, default 0) of the kernels launched with
 * a bounded grid through this context (it has no effect on unbounded launches).  A raised
 * priority lets the aggregation's wavefronts win instruction issue against the wavefronts
 * of a compute kernel on the same compute unit: the aggregation finishes sooner, the
 * compute kernel is slowed more.  Which setting hides more depends on how much slack the
 * schedule leaves the aggregation.  Results are identical for every setting.
 * Errors: DEAR_EINVAL (null context, priority outside 0..3). */
int dear_ctx_set_wave_priority(dear_ctx_t *ctx, int32_t priority);

/* Shard buffers (arguments shard_grad, shard_param, shard_mom below): DEVICE, fp32,
 * P rows of total_shard_len elements, row stride total_shard_len, base 256-byte
 * aligned (DEAR_EALIGN otherwise).  Row p holds worker p's owned shards of all buckets;
 * bucket b occupies [bucket_shard_base[b], +S_b) of every row.
 *
 * bucket argument: 0 .. n_buckets-1, or -1 for every bucket in one launch
 * (DEAR_ERANGE otherwise). */

/* ---------------------------------------------------------------------------------
 * dear_reduce_scatter -- first half of the decoupled all-reduce, with the copy into
 * the fusion buffer folded into the loads.
 *
 * Paper: Section III-A (ring reduce-scatter: chunk s is reduced onto worker s through
 * P-1 rounds, Eq. 3), Section IV-A (gradients of a group are communicated together),
 * Eq. 2 (the 1/P of S-SGD).
 *
 * For every position e of the bucket, owned by shard s = e / S_b:
 *     acc = g[(s+1)%P][e]; acc += g[(s+2)%P][e]; ... ; acc += g[s][e]   (fp32, RN-even)
 *     shard_grad[s][shard_base_b + e % S_b] = acc * (1.0f / P)
 * where g[p][e] is worker p's gradient at that position, widened to fp32 if bf16.
 * Padding slots are written as +0.0f.
 *   shard_grad  device, written (layout above)
 * Errors: DEAR_EINVAL, DEAR_ERANGE, DEAR_EALIGN, DEAR_EHIP.
 */
int dear_reduce_scatter(dear_ctx_t *ctx, int32_t bucket, float *shard_grad, void *hip_stream);

/* ---------------------------------------------------------------------------------
 * dear_reduce_scatter_static -- dear_reduce_scatter for callers that cannot allocate
 * device memory: tight serving or training loops and harnesses that forbid hipMalloc
 * once running, where creating a context (which allocates its tile and pointer tables)
 * is not possible.  It needs no context and calls neither hipMalloc nor hipFree nor any
 * other allocating routine, on the device or the host: the two tables its kernel reads
 * are built in a fixed host staging area and uploaded into a fixed device array that
 * the library holds on every GPU it runs on until the process ends
 * (DEAR_STATIC_MAX_POINTERS * 8 + DEAR_STATIC_MAX_TILES * 32 bytes = 4 MiB).
 *
 *   plan        host, as for dear_ctx_create
 *   grad_dtype  DEAR_F32 or DEAR_BF16, must agree with the plan
 *   grad_ptrs   host array of P*n_layers DEVICE pointers, index [p*n_layers + l], each
 *               16-byte aligned (read during the call; may be reused afterwards)
 *   bucket      0 .. n_buckets-1, or -1 for every bucket in one launch
 *   shard_grad  device, written; layout and values exactly as dear_reduce_scatter
 *
 * Limits: P*n_layers <= DEAR_STATIC_MAX_POINTERS and the processed buckets must cut into
 * at most DEAR_STATIC_MAX_TILES tiles (one tile per DEAR_TILE_ELEMS elements of a layer
 * within a shard, plus ragged ends: about 400 M elements); beyond that DEAR_ETOOBIG is
 * returned and nothing is launched.
 * The call uploads the tables on hip_stream, waits for that stream (so work queued on it
 * earlier has finished when the call returns), then enqueues the kernel and returns
 * without waiting for it.  Uses the current HIP device.  All calls on one GPU share that
 * GPU's array, which keeps the last call's tables: nothing in it needs clearing (every
 * entry the kernel reads is rewritten by the call), but calls that overlap on one GPU --
 * different host threads, or a second call on another stream while the first call's
 * kernel still runs -- race and must be serialised by the caller.
 * Errors: DEAR_EINVAL, DEAR_ERANGE, DEAR_EALIGN, DEAR_ETOOBIG, DEAR_EHIP.
 */
#define DEAR_STATIC_MAX_POINTERS 131072
#define DEAR_STATIC_MAX_TILES 98304
int dear_reduce_scatter_static(const dear_plan_t *plan, int32_t grad_dtype,
                               const void *const *grad_ptrs, int32_t bucket, float *shard_grad,
                               void *hip_stream);

/* ---------------------------------------------------------------------------------
 * dear_shard_update -- SGD with momentum on the owned shards of a bucket.
 *
 * Paper: Eq. 1-2 (w <- w - lr * averaged gradient); momentum as in the optimizer the
 * paper wraps (Section V-B).  Per slot, each operation rounded separately (no FMA):
 *     v = momentum * v + gbar;   w = w - lr * v
 *   shard_grad   device, read;  shard_param, shard_mom  device, updated in place
 * The three buffers share the shard-buffer layout and must not overlap.
 * Errors: DEAR_EINVAL, DEAR_ERANGE, DEAR_EALIGN, DEAR_EHIP.
 */
int dear_shard_update(dear_ctx_t *ctx, int32_t bucket, const float *shard_grad,
                      float *shard_param, float *shard_mom, float lr, float momentum,
                      void *hip_stream);

/* ---------------------------------------------------------------------------------
 * dear_reduce_scatter_update -- dear_reduce_scatter and dear_shard_update of a bucket in
 * one kernel: the averaged gradient of a slot is consumed by the slot's update while it
 * is still in registers and is never written to memory (no shard_grad buffer).  Same
 * operations in the same order as the two separate calls, so shard_param and shard_mom
 * come out bit-identical.  It still runs in the backward pass, before any all-gather
 * (paper Section III-B), so the decoupling of the two halves is untouched.
 *   shard_param, shard_mom  device, updated in place (padding slots are updated with
 *                           an averaged gradient of +0.0f)
 * Errors: DEAR_EINVAL, DEAR_ERANGE, DEAR_EALIGN, DEAR_EHIP.
 */
int dear_reduce_scatter_update(dear_ctx_t *ctx, int32_t bucket, float *shard_param, float *shard_mom,
                               float lr, float momentum, void *hip_stream);

/* ---------------------------------------------------------------------------------
 * dear_all_gather -- second half of the decoupled all-reduce, with the copy from the
 * fusion buffer back to the original tensors folded into the stores.
 *
 * Paper: Section III-A (all-gather: every reduced chunk reaches all workers, Eq. 4),
 * Section IV-A (buffer contents are copied back to the tensors), Section II-B (all
 * workers hold identical parameters).
 *
 * For every worker p, every layer l of the bucket and element i:
 *     param[p][l][i] = shard_param[s][shard_base_b + e % S_b],  e = layer_offset[l] + i
 *   shard_param  device, read
 * Errors: DEAR_EINVAL, DEAR_ERANGE, DEAR_EALIGN, DEAR_EHIP.
 */
int dear_all_gather(dear_ctx_t *ctx, int32_t bucket, const float *shard_param, void *hip_stream);

/* ---------------------------------------------------------------------------------
 * dear_update_all_gather -- dear_shard_update and dear_all_gather of a bucket in one kernel:
 * the updated parameter of a slot is stored to the shard buffer and to all P replicas' layer
 * tensors while it is still in registers, so shard_param is not read again.  Same operations
 * in the same order as the two separate calls: shard_param, shard_mom and every replica's
 * parameters come out bit-identical.  It moves 4 bytes per element less than the two calls,
 * but the update then runs where the all-gather runs (in the forward pass of the next
 * iteration, paper Section III-B) and the replicas are written as P interleaved streams,
 * which the memory system sustains less well than the replica-by-replica order of
 * dear_all_gather; it is provided for comparison.
 *   shard_grad   device, read;  shard_param, shard_mom  device, updated in place
 * Errors: DEAR_EINVAL, DEAR_ERANGE, DEAR_EALIGN, DEAR_EHIP.
 */
int dear_update_all_gather(dear_ctx_t *ctx, int32_t bucket, const float *shard_grad, float *shard_param,
                           float *shard_mom, float lr, float momentum, void *hip_stream);

/* dear_all_gather_workers -- dear_all_gather restricted to the workers
 * first_worker .. first_worker+n_workers-1 (only their parameter tensors are written).
 * With one worker it turns any shard buffer (e.g. the momentum shards) back into that
 * worker's per-layer layout, which is what a caller needs to re-shard optimizer state
 * when the bucket plan changes (run-time tuning of the buffer size, paper Section IV-B).
 * Errors as dear_all_gather; DEAR_ERANGE also for a worker range outside 0 .. P-1. */
int dear_all_gather_workers(dear_ctx_t *ctx, int32_t bucket, const float *shard_param,
                            int32_t first_worker, int32_t n_workers, void *hip_stream);

/* ---------------------------------------------------------------------------------
 * dear_scatter_params -- seed the owned parameter shards from worker `worker`'s full
 * parameter tensors (inverse of dear_all_gather for one worker; run once before the
 * first iteration; padding slots become +0.0f).  Every bucket is processed.
 *   shard_param  device, written
 * Errors: DEAR_EINVAL, DEAR_ERANGE (worker), DEAR_EALIGN, DEAR_EHIP.
 */
int dear_scatter_params(dear_ctx_t *ctx, int32_t worker, float *shard_param, void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *dear_strerror(int status);

/* Library version as major*10000 + minor*100 + patch. */
int dear_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DEAR_H */
