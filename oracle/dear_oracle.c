/*
 * CPU oracle for DeAR's decoupled gradient aggregation -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded restatement of what the path computes, used by the
 * tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no code,
 * header, table or helper with the HIP library and the product path never calls it.
 *
 * What is computed (paper sections in brackets):
 *   plan            -- threshold tensor fusion: consecutive layers, taken in the order
 *                      their gradients become ready (last layer first), form one group
 *                      while their total gradient count does not exceed the buffer
 *                      size x [Sec. IV-B; issue order Sec. III-B]; each group of d
 *                      elements is cut into P chunks, one per worker [Sec. III-A].
 *   plan_fixed_layers -- the other grouping of the tensor-fusion study: a fixed number
 *                      of consecutive layers per group [Sec. VI-G]; chunking as above.
 *   reduce_scatter  -- chunk s of every group is reduced onto worker s through P-1 ring
 *                      rounds [Sec. III-A, Eq. 3]; the 1/P of S-SGD is applied to the
 *                      finished sum [Eq. 2].
 *   shard_update    -- SGD with momentum on the owned chunk [Eq. 1-2].
 *   all_gather      -- every worker's chunk is copied to all workers [Sec. III-A, Eq. 4]
 *                      and from the fusion buffer back to the original tensors [Sec. IV-A].
 *
 * Arithmetic is IEEE binary32, round-to-nearest-even, one rounding per operation
 * (build with -ffp-contract=off, no fast-math).  A "group" in the paper is a "bucket"
 * here; a "chunk" is a "shard".
 *
 * Readings where the paper is silent:
 *   - a group is closed BEFORE the layer that would push it past x; a total equal to x
 *     stays in the group; a single tensor larger than x is a group of its own
 *     (tensors are never partitioned, Sec. III-B);
 *   - x is given in bytes of the gradient type: X = floor(x / g) elements;
 *   - layers sit in a group in arrival order, densely packed;
 *   - shard length S = ceil(d / P) rounded up to 32 elements; positions >= d are padding
 *     and reduce to +0;
 *   - chunk s is owned by worker s, the ring sends r -> r+1, so the sum of chunk s
 *     starts at worker s+1 and ends with worker s's own contribution;
 *   - the average is one multiplication by the binary32 value 1/P;
 *   - momentum form v <- mu*v + g ; w <- w - lr*v.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_SHARD_ALIGN 32

/* ------------------------------------------------------------- chunking [Sec. III-A] */
/* Every group of d elements is cut into P chunks of d/P elements, one per worker; the
 * chunk length is rounded up so that P chunks cover d and stay 32-element aligned. */
static void cut_into_chunks(int32_t B, int32_t P, const int64_t *bucket_len,
                            int64_t *bucket_shard_len, int64_t *bucket_shard_base)
{
    int64_t base = 0;
    for (int32_t b = 0; b < B; ++b) {
        int64_t per = (bucket_len[b] + P - 1) / P;
        int64_t S = (per + ORACLE_SHARD_ALIGN - 1) / ORACLE_SHARD_ALIGN * ORACLE_SHARD_ALIGN;
        bucket_shard_len[b] = S;
        bucket_shard_base[b] = base;
        base += S;
    }
}

/* ------------------------------------------------------------------ plan [Sec. IV-B] */
/* Outputs: layer_bucket[L], layer_offset[L]; per bucket (arrays of capacity L):
 * first layer (lowest forward index), layer count, d, S, and the start of the bucket's
 * slots inside a worker's row of the shard buffers.  Returns the number of buckets, or
 * a negative value for invalid arguments. */
int32_t oracle_plan(const int64_t *n, int32_t L, int32_t P, int64_t x_bytes, int32_t g,
                    int32_t *layer_bucket, int64_t *layer_offset,
                    int32_t *bucket_first_layer, int32_t *bucket_n_layers,
                    int64_t *bucket_len, int64_t *bucket_shard_len, int64_t *bucket_shard_base)
{
    if (L < 1 || P < 1 || x_bytes < 0 || (g != 2 && g != 4)) return -1;
    for (int32_t l = 0; l < L; ++l)
        if (n[l] < 1) return -1;

    const int64_t X = x_bytes / g;          /* buffer size in gradient elements */
    int32_t B = 0;
    int64_t tot = 0;                        /* elements in the open group */
    int32_t cnt = 0;                        /* layers in the open group   */
    for (int32_t l = L - 1; l >= 0; --l) {  /* gradient-ready order */
        /* n[l] > X - tot  <=>  tot + n[l] > X, written so that it cannot overflow */
        if (cnt > 0 && n[l] > X - tot) {
            bucket_first_layer[B] = l + 1;
            bucket_n_layers[B] = cnt;
            bucket_len[B] = tot;
            ++B;
            tot = 0;
            cnt = 0;
        }
        layer_bucket[l] = B;
        layer_offset[l] = tot;
        tot += n[l];
        ++cnt;
    }
    bucket_first_layer[B] = 0;
    bucket_n_layers[B] = cnt;
    bucket_len[B] = tot;
    ++B;

    cut_into_chunks(B, P, bucket_len, bucket_shard_len, bucket_shard_base);
    return B;
}

/* ------------------------------------------- plan, fixed number of layers [Sec. VI-G] */
/* The naive grouping the tensor-fusion study compares against: every group is k
 * consecutive layers, taken in gradient-ready order (last layer first), whatever their
 * sizes; the layers left over at the front of the model form the last, shorter group.
 * Outputs and return value as oracle_plan. */
int32_t oracle_plan_fixed_layers(const int64_t *n, int32_t L, int32_t P, int32_t k, int32_t g,
                                 int32_t *layer_bucket, int64_t *layer_offset,
                                 int32_t *bucket_first_layer, int32_t *bucket_n_layers,
                                 int64_t *bucket_len, int64_t *bucket_shard_len, int64_t *bucket_shard_base)
{
    if (L < 1 || P < 1 || k < 1 || (g != 2 && g != 4)) return -1;
    for (int32_t l = 0; l < L; ++l)
        if (n[l] < 1) return -1;

    int32_t B = 0;
    int64_t pos = 0;                        /* elements packed into the open group */
    int32_t held = 0;                       /* layers in the open group            */
    for (int32_t l = L - 1; l >= 0; --l) {  /* same arrival order as the threshold rule */
        if (held == k) {                     /* the open group is full */
            bucket_first_layer[B] = l + 1;
            bucket_n_layers[B] = held;
            bucket_len[B] = pos;
            ++B;
            pos = 0;
            held = 0;
        }
        layer_bucket[l] = B;
        layer_offset[l] = pos;
        pos += n[l];
        ++held;
    }
    bucket_first_layer[B] = 0;
    bucket_n_layers[B] = held;
    bucket_len[B] = pos;
    ++B;

    cut_into_chunks(B, P, bucket_len, bucket_shard_len, bucket_shard_base);
    return B;
}

/* --------------------------------------------------------------------------- helpers */
static float widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* gradient element i of layer l on worker p; grad[p*L + l] points at that tensor */
static float grad_at(const void *const *grad, int32_t L, int32_t g, int32_t p, int32_t l, int64_t i)
{
    const void *t = grad[(size_t)p * L + l];
    if (g == 4) return ((const float *)t)[i];
    return widen_bf16(((const uint16_t *)t)[i]);
}

/* layer holding bucket position e: the layers of a bucket are first..first+count-1 and
 * are packed from the highest index down */
static int32_t layer_of(const int64_t *n, const int64_t *layer_offset,
                        int32_t first, int32_t count, int64_t e)
{
    for (int32_t l = first + count - 1; l >= first; --l)
        if (e >= layer_offset[l] && e < layer_offset[l] + n[l]) return l;
    return -1;
}

/* ------------------------------------------------- reduce-scatter [Sec. III-A; Eq. 2] */
/* One bucket; shards s_begin <= s < s_end (so callers may split the work by shard).
 * shard_grad has P rows of row_stride floats; row s receives chunk s. */
void oracle_reduce_scatter(const int64_t *n, int32_t L, int32_t P, int32_t g,
                           const int64_t *layer_offset,
                           int32_t first, int32_t count, int64_t d, int64_t S, int64_t shard_base,
                           const void *const *grad, float *shard_grad, int64_t row_stride,
                           int32_t s_begin, int32_t s_end)
{
    const float inv_P = 1.0f / (float)P;
    for (int32_t s = s_begin; s < s_end; ++s) {
        float *out = shard_grad + (size_t)s * row_stride + shard_base;
        int32_t l = -1;                     /* layer holding the current position */
        for (int64_t j = 0; j < S; ++j) {
            const int64_t e = (int64_t)s * S + j;
            if (e >= d) {
                out[j] = 0.0f;
                continue;
            }
            /* positions ascend, so the layer only ever steps to the next-packed one */
            if (l < 0) l = layer_of(n, layer_offset, first, count, e);
            while (e >= layer_offset[l] + n[l]) --l;
            const int64_t i = e - layer_offset[l];
            /* ring: worker s+1 starts, each next worker adds its own copy, worker s last */
            float acc = grad_at(grad, L, g, (s + 1) % P, l, i);
            for (int32_t k = 2; k <= P; ++k)
                acc = acc + grad_at(grad, L, g, (s + k) % P, l, i);
            out[j] = acc * inv_P;
        }
    }
}

/* ------------------------------------------------------ shard update [Eq. 1, Eq. 2] */
/* One bucket, shards s_begin..s_end-1; all three buffers share the row layout. */
void oracle_shard_update(int32_t P, int64_t S, int64_t shard_base, int64_t row_stride,
                         const float *shard_grad, float *shard_param, float *shard_mom,
                         float lr, float mu, int32_t s_begin, int32_t s_end)
{
    (void)P;
    for (int32_t s = s_begin; s < s_end; ++s) {
        const size_t r = (size_t)s * row_stride + shard_base;
        for (int64_t j = 0; j < S; ++j) {
            float t1 = mu * shard_mom[r + j];
            float v = t1 + shard_grad[r + j];
            float t2 = lr * v;
            shard_mom[r + j] = v;
            shard_param[r + j] = shard_param[r + j] - t2;
        }
    }
}

/* --------------------------------------------- all-gather + copy-back [Sec. III-A, IV-A] */
/* One bucket; param[p*L + l] points at worker p's parameter tensor l.  Workers
 * p_begin..p_end-1 receive (so callers may split the work by receiving worker). */
void oracle_all_gather(const int64_t *n, int32_t L, int32_t P,
                       const int64_t *layer_offset,
                       int32_t first, int32_t count, int64_t S, int64_t shard_base,
                       const float *shard_param, int64_t row_stride,
                       float *const *param, int32_t p_begin, int32_t p_end)
{
    (void)P;
    for (int32_t p = p_begin; p < p_end; ++p)
        for (int32_t l = first; l < first + count; ++l)
            for (int64_t i = 0; i < n[l]; ++i) {
                const int64_t e = layer_offset[l] + i;
                const int64_t s = e / S;
                const int64_t slot = shard_base + e % S;
                param[(size_t)p * L + l][i] = shard_param[(size_t)s * row_stride + slot];
            }
}

/* inverse of the copy-back for one worker: seeds the owned parameter shards from
 * worker p's full parameter tensors before the first iteration; padding becomes +0 */
void oracle_scatter_params(const int64_t *n, int32_t L, int32_t P,
                           const int64_t *layer_offset,
                           int32_t first, int32_t count, int64_t d, int64_t S, int64_t shard_base,
                           float *const *param, int32_t p, float *shard_param, int64_t row_stride)
{
    for (int32_t s = 0; s < P; ++s)
        for (int64_t j = 0; j < S; ++j) {
            const int64_t e = (int64_t)s * S + j;
            float val = 0.0f;
            if (e < d) {
                const int32_t l = layer_of(n, layer_offset, first, count, e);
                val = param[(size_t)p * L + l][e - layer_offset[l]];
            }
            shard_param[(size_t)s * row_stride + shard_base + j] = val;
        }
}
