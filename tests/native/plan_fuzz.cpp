// Host-only fuzz driver for libdear's planner and tile table, meant to be built with
// -fsanitize=address,undefined.  Exits non-zero on the first broken invariant.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "dear.h"
#include "dear_internal.h"  // dear_emit_tiles, the emitter behind the tile table and the allocation-free entry point

#define CHECK(c)                                                         \
    do {                                                                 \
        if (!(c)) {                                                      \
            std::fprintf(stderr, "FAILED %s (line %d)\n", #c, __LINE__); \
            std::exit(1);                                                \
        }                                                                \
    } while (0)

static void one_case(std::mt19937_64 &rng)
{
    const int L = 1 + static_cast<int>(rng() % 40);
    const int P = 1 + static_cast<int>(rng() % 70);
    const int g = (rng() & 1) ? 2 : 4;
    static const int64_t picks[] = {1, 2, 3, 5, 31, 32, 33, 100, 4095, 4096, 4097, 10000, 30001};
    std::vector<int64_t> n(L);
    int64_t N = 0;
    for (auto &v : n) {
        v = picks[rng() % (sizeof(picks) / sizeof(picks[0]))];
        N += v;
    }
    static const int64_t thr[] = {0, 1, 4000, 40000, 1000000, DEAR_NO_LIMIT};
    const int64_t x = thr[rng() % 6];
    dear_plan_t *pl = nullptr;
    const bool fixed = (rng() % 5) == 0;
    if (fixed)
        CHECK(dear_plan_fixed_layers(n.data(), L, P, 1 + static_cast<int>(rng() % 6), g, &pl) == DEAR_OK);
    else
        CHECK(dear_plan(n.data(), L, P, x, g, &pl) == DEAR_OK);
    dear_plan_view_t v;
    CHECK(dear_plan_view(pl, &v) == DEAR_OK);
    CHECK(v.n_layers == L && v.P == P && v.total_elems == N);

    int64_t n_tiles = 0;
    CHECK(dear_plan_tiles(pl, nullptr, 0, &n_tiles, nullptr) == DEAR_OK);
    std::vector<dear_tile_t> tiles(static_cast<size_t>(n_tiles));   // exact size: overruns are caught
    std::vector<int64_t> begin(static_cast<size_t>(v.n_buckets) + 1);
    CHECK(dear_plan_tiles(pl, tiles.data(), n_tiles, &n_tiles, begin.data()) == DEAR_OK);
    CHECK(begin[0] == 0 && begin[v.n_buckets] == n_tiles);

    std::vector<uint8_t> slot(static_cast<size_t>(P * v.total_shard_len), 0);
    int64_t covered_elems = 0;
    for (int b = 0; b < v.n_buckets; ++b) {
        const int64_t S = v.bucket_shard_len[b], base = v.bucket_shard_base[b];
        CHECK(S % DEAR_SHARD_ALIGN == 0 && S * P >= v.bucket_len[b]);
        for (int64_t i = begin[b]; i < begin[b + 1]; ++i) {
            const dear_tile_t &t = tiles[static_cast<size_t>(i)];
            CHECK(t.bucket == b && t.count >= 1 && t.count <= DEAR_TILE_ELEMS && t.shard >= 0 && t.shard < P);
            const int64_t lo = t.shard * v.total_shard_len + base;
            CHECK(t.dst_begin >= lo && t.dst_begin + t.count <= lo + S);
            for (int64_t k = 0; k < t.count; ++k) CHECK(slot[static_cast<size_t>(t.dst_begin + k)]++ == 0);
            if (t.layer >= 0) {
                CHECK(t.layer < L && v.layer_bucket[t.layer] == b);
                CHECK(t.src_begin >= 0 && t.src_begin + t.count <= n[static_cast<size_t>(t.layer)]);
                const int64_t e = v.layer_offset[t.layer] + t.src_begin;
                CHECK(e / S == t.shard && (e + t.count - 1) / S == t.shard);
                CHECK(t.dst_begin == lo + e % S);
                covered_elems += t.count;
            }
        }
    }
    CHECK(covered_elems == N);
    for (uint8_t s : slot) CHECK(s == 1);

    // a capacity below the tile count: exactly that many entries are written, the count is still the full one
    {
        const int64_t cap = n_tiles / 2;
        std::vector<dear_tile_t> part(static_cast<size_t>(cap));
        int64_t n2 = -1;
        CHECK(dear_plan_tiles(pl, part.data(), cap, &n2, nullptr) == DEAR_OK && n2 == n_tiles);
        for (int64_t i = 0; i < cap; ++i) CHECK(part[i].dst_begin == tiles[i].dst_begin && part[i].count == tiles[i].count);
    }
    // the emitter on a range of buckets, into an exactly sized array, equals that range of the full table
    {
        const int b0 = static_cast<int>(rng() % v.n_buckets), b1 = b0 + 1 + static_cast<int>(rng() % (v.n_buckets - b0));
        const int64_t want = begin[b1] - begin[b0];
        std::vector<dear_tile_t> range(static_cast<size_t>(want));
        std::vector<int64_t> rb(static_cast<size_t>(b1 - b0) + 1);
        CHECK(dear_emit_tiles(*pl, b0, b1, range.data(), want, rb.data()) == want);
        for (int64_t i = 0; i < want; ++i) {
            const dear_tile_t &x = range[i], &y = tiles[begin[b0] + i];
            CHECK(x.src_begin == y.src_begin && x.dst_begin == y.dst_begin && x.count == y.count &&
                  x.layer == y.layer && x.shard == y.shard && x.bucket == y.bucket);
        }
        for (int b = b0; b <= b1; ++b) CHECK(rb[b - b0] == begin[b] - begin[b0]);
        CHECK(dear_emit_tiles(*pl, b0, b1, nullptr, 0, nullptr) == want);
    }
    dear_plan_free(pl);
}

int main(int argc, char **argv)
{
    const int cases = argc > 1 ? std::atoi(argv[1]) : 300;
    std::mt19937_64 rng(20230212);
    for (int i = 0; i < cases; ++i) one_case(rng);
    // argument errors must not touch their outputs
    dear_plan_t *pl = nullptr;
    int64_t one = 1, zero = 0;
    CHECK(dear_plan(&zero, 1, 1, 0, 4, &pl) == DEAR_EINVAL && pl == nullptr);
    CHECK(dear_plan(&one, 1, 0, 0, 4, &pl) == DEAR_EINVAL && pl == nullptr);
    CHECK(dear_plan(&one, 1, 1, -1, 4, &pl) == DEAR_EINVAL && pl == nullptr);
    CHECK(dear_plan(&one, 1, 1, 0, 3, &pl) == DEAR_EINVAL && pl == nullptr);
    dear_plan_free(nullptr);
    std::printf("plan_fuzz: %d cases ok\n", cases);
    return 0;
}
