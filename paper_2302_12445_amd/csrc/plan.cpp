// Host-side bucket / shard planner of libdear (integer work only).
//
// Threshold tensor fusion (paper Sec. IV-B): gradients arrive last layer first
// (Sec. III-B); arriving layers are appended to the open bucket until the next one would
// make the bucket hold more than X = floor(x / g) elements; then the bucket is closed.
// A layer is never split (Sec. III-B), so one that alone exceeds X is a bucket by itself.
// Each closed bucket of d elements is cut into P shards (Sec. III-A).
#include <memory>
#include <new>

#include "dear_internal.h"

namespace {

int validate(const int64_t *sizes, int32_t L, int32_t P, int32_t g, dear_plan_t **out)
{
    if (!sizes || !out || L < 1 || P < 1 || (g != 2 && g != 4)) return DEAR_EINVAL;
    for (int32_t l = 0; l < L; ++l)
        if (sizes[l] < 1) return DEAR_EINVAL;
    return DEAR_OK;
}

// Given where each bucket ends (cut[b] = lowest layer index of bucket b), fill in all tables.
void finish(dear_plan_s &pl, const std::vector<int32_t> &cuts)
{
    const int32_t B = static_cast<int32_t>(cuts.size());
    pl.B = B;
    pl.bucket_first_layer = cuts;
    pl.bucket_n_layers.resize(B);
    pl.bucket_len.resize(B);
    pl.bucket_shard_len.resize(B);
    pl.bucket_shard_base.resize(B);
    pl.layer_bucket.resize(pl.L);
    pl.layer_offset.resize(pl.L);

    int32_t top = pl.L;  // one past the highest layer of the bucket being filled
    int64_t row = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t lo = cuts[b];
        int64_t pos = 0;
        for (int32_t l = top - 1; l >= lo; --l) {  // dense packing in arrival order
            pl.layer_bucket[l] = b;
            pl.layer_offset[l] = pos;
            pos += pl.layer_sizes[l];
        }
        pl.bucket_n_layers[b] = top - lo;
        pl.bucket_len[b] = pos;
        const int64_t per_worker = pos / pl.P + (pos % pl.P != 0);
        const int64_t S = (per_worker + DEAR_SHARD_ALIGN - 1) & ~int64_t(DEAR_SHARD_ALIGN - 1);
        pl.bucket_shard_len[b] = S;
        pl.bucket_shard_base[b] = row;
        row += S;
        top = lo;
    }
    pl.row_len = row;
}

std::unique_ptr<dear_plan_s> start(const int64_t *sizes, int32_t L, int32_t P, int32_t g)
{
    std::unique_ptr<dear_plan_s> pl(new dear_plan_s);
    pl->L = L;
    pl->P = P;
    pl->g = g;
    pl->layer_sizes.assign(sizes, sizes + L);
    for (int32_t l = 0; l < L; ++l) pl->N += sizes[l];
    return pl;
}

}  // namespace

extern "C" int dear_plan(const int64_t *layer_sizes, int32_t n_layers, int32_t P,
                         int64_t fusion_threshold_bytes, int32_t grad_elem_bytes, dear_plan_t **out)
{
    int rc = validate(layer_sizes, n_layers, P, grad_elem_bytes, out);
    if (rc != DEAR_OK) return rc;
    if (fusion_threshold_bytes < 0) return DEAR_EINVAL;
    try {
        std::unique_ptr<dear_plan_s> pl = start(layer_sizes, n_layers, P, grad_elem_bytes);
        pl->threshold_bytes = fusion_threshold_bytes;
        const int64_t X = fusion_threshold_bytes / grad_elem_bytes;
        std::vector<int32_t> cuts;
        int64_t room = X;        // elements the open bucket can still take
        bool open = false;
        for (int32_t l = n_layers - 1; l >= 0; --l) {
            const int64_t n = layer_sizes[l];
            if (open && n > room) {  // would exceed x: close before this layer
                cuts.push_back(l + 1);
                room = X;
            }
            open = true;
            room = (n > room) ? 0 : room - n;  // an oversized single layer fills the bucket
        }
        cuts.push_back(0);
        finish(*pl, cuts);
        *out = pl.release();
    } catch (const std::bad_alloc &) {
        return DEAR_ENOMEM;
    }
    return DEAR_OK;
}

extern "C" int dear_plan_fixed_layers(const int64_t *layer_sizes, int32_t n_layers, int32_t P,
                                      int32_t layers_per_bucket, int32_t grad_elem_bytes,
                                      dear_plan_t **out)
{
    int rc = validate(layer_sizes, n_layers, P, grad_elem_bytes, out);
    if (rc != DEAR_OK) return rc;
    if (layers_per_bucket < 1) return DEAR_EINVAL;
    try {
        std::unique_ptr<dear_plan_s> pl = start(layer_sizes, n_layers, P, grad_elem_bytes);
        pl->threshold_bytes = -1;
        std::vector<int32_t> cuts;
        for (int32_t top = n_layers; top > 0; top -= layers_per_bucket)
            cuts.push_back(top > layers_per_bucket ? top - layers_per_bucket : 0);
        finish(*pl, cuts);
        *out = pl.release();
    } catch (const std::bad_alloc &) {
        return DEAR_ENOMEM;
    }
    return DEAR_OK;
}

// Cut the buckets b_first .. b_last-1 into tiles: runs of one layer within one shard, split
// at multiples of DEAR_TILE_ELEMS of the layer's own element index so that tile-interior
// vectors stay aligned; then the padding slots behind the last real element.  Tiles are
// written to out[0 .. capacity) as far as they fit; the return value is the number of tiles
// the buckets have (so a first call with capacity 0 sizes the table).  tile_begin, if given,
// receives b_last - b_first + 1 range starts relative to the first tile written.
int64_t dear_emit_tiles(const dear_plan_s &pl, int32_t b_first, int32_t b_last, dear_tile *out,
                        int64_t capacity, int64_t *tile_begin)
{
    int64_t n_out = 0;
    auto emit = [&](const dear_tile &t) {
        if (n_out < capacity) out[n_out] = t;
        ++n_out;
    };
    for (int32_t b = b_first; b < b_last; ++b) {
        if (tile_begin) tile_begin[b - b_first] = n_out;
        const int64_t S = pl.bucket_shard_len[b], base = pl.bucket_shard_base[b];
        const int32_t lo = pl.bucket_first_layer[b], hi = lo + pl.bucket_n_layers[b];
        for (int32_t l = hi - 1; l >= lo; --l) {
            const int64_t off = pl.layer_offset[l], n = pl.layer_sizes[l];
            int64_t i = 0;
            while (i < n) {
                const int64_t s = (off + i) / S;
                const int64_t run_end = (s + 1) * S - off < n ? (s + 1) * S - off : n;
                while (i < run_end) {
                    const int64_t next_cut = (i / DEAR_TILE_ELEMS + 1) * DEAR_TILE_ELEMS;
                    const int64_t end = next_cut < run_end ? next_cut : run_end;
                    dear_tile t;
                    t.src_begin = i;
                    t.dst_begin = s * pl.row_len + base + (off + i - s * S);
                    t.count = static_cast<int32_t>(end - i);
                    t.layer = l;
                    t.shard = static_cast<int32_t>(s);
                    t.bucket = b;
                    emit(t);
                    i = end;
                }
            }
        }
        int64_t e = pl.bucket_len[b];
        const int64_t total = S * pl.P;
        while (e < total) {
            const int64_t s = e / S;
            int64_t end = (s + 1) * S;
            if (end - e > DEAR_TILE_ELEMS) end = e + DEAR_TILE_ELEMS;
            dear_tile t;
            t.src_begin = 0;
            t.dst_begin = s * pl.row_len + base + (e - s * S);
            t.count = static_cast<int32_t>(end - e);
            t.layer = -1;
            t.shard = static_cast<int32_t>(s);
            t.bucket = b;
            emit(t);
            e = end;
        }
    }
    if (tile_begin) tile_begin[b_last - b_first] = n_out;
    return n_out;
}

void dear_build_tiles(const dear_plan_s &pl, std::vector<dear_tile> &tiles, std::vector<int64_t> &tile_begin)
{
    tile_begin.assign(pl.B + 1, 0);
    const int64_t n = dear_emit_tiles(pl, 0, pl.B, nullptr, 0, nullptr);
    tiles.resize(static_cast<size_t>(n));
    dear_emit_tiles(pl, 0, pl.B, tiles.data(), n, tile_begin.data());
}

extern "C" int dear_plan_tiles(const dear_plan_t *plan, dear_tile_t *out, int64_t capacity,
                               int64_t *n_tiles, int64_t *bucket_tile_begin)
{
    if (!plan || !n_tiles || capacity < 0 || (capacity > 0 && !out)) return DEAR_EINVAL;
    try {
        std::vector<dear_tile> tiles;
        std::vector<int64_t> begin;
        dear_build_tiles(*plan, tiles, begin);
        *n_tiles = static_cast<int64_t>(tiles.size());
        const int64_t n = capacity < *n_tiles ? capacity : *n_tiles;
        for (int64_t i = 0; i < n; ++i) out[i] = tiles[i];
        if (bucket_tile_begin)
            for (int32_t b = 0; b <= plan->B; ++b) bucket_tile_begin[b] = begin[b];
    } catch (const std::bad_alloc &) {
        return DEAR_ENOMEM;
    }
    return DEAR_OK;
}

extern "C" void dear_plan_free(dear_plan_t *plan) { delete plan; }

extern "C" int dear_plan_view(const dear_plan_t *pl, dear_plan_view_t *v)
{
    if (!pl || !v) return DEAR_EINVAL;
    v->n_layers = pl->L;
    v->n_buckets = pl->B;
    v->P = pl->P;
    v->grad_elem_bytes = pl->g;
    v->shard_align = DEAR_SHARD_ALIGN;
    v->reserved = 0;
    v->threshold_bytes = pl->threshold_bytes;
    v->total_elems = pl->N;
    v->total_shard_len = pl->row_len;
    v->layer_sizes = pl->layer_sizes.data();
    v->layer_bucket = pl->layer_bucket.data();
    v->layer_offset = pl->layer_offset.data();
    v->bucket_first_layer = pl->bucket_first_layer.data();
    v->bucket_n_layers = pl->bucket_n_layers.data();
    v->bucket_len = pl->bucket_len.data();
    v->bucket_shard_len = pl->bucket_shard_len.data();
    v->bucket_shard_base = pl->bucket_shard_base.data();
    return DEAR_OK;
}

extern "C" const char *dear_strerror(int status)
{
    switch (status) {
    case DEAR_OK: return "ok";
    case DEAR_EINVAL: return "invalid argument";
    case DEAR_ENOMEM: return "out of memory (library table)";
    case DEAR_EHIP: return "HIP runtime error";
    case DEAR_ERANGE: return "bucket or worker index out of range";
    case DEAR_EALIGN: return "device pointer not aligned as required";
    case DEAR_ETOOBIG: return "input exceeds the capacity of the static device scratch";
    default: return "unknown status";
    }
}

extern "C" int dear_version(void) { return 200; }
