// Drives the host-side planner (adasum_plan.cpp: tile tables, pass schedules, workspace
// layout) over seeded random inputs and checks its invariants.  Built by
// tests/test_host_sanitizers_cpu.py with AddressSanitizer and UndefinedBehaviorSanitizer on
// the CPU; exits non-zero on the first violated invariant (the sanitizers abort on their own).
#include <algorithm>
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "adasum_host.h"

using namespace adasum;

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                            \
        }                                                                            \
    } while (0)

static std::vector<int64_t> random_table(std::mt19937_64& rng, int n_layers, int kind) {
    std::vector<int64_t> offs(1, 0);
    for (int l = 0; l < n_layers; ++l) {
        int64_t len;
        const uint64_t r = rng();
        switch (kind) {
            case 0: len = static_cast<int64_t>(r % 40); break;                    // tiny, many empty or small
            case 1: len = static_cast<int64_t>(r % 70000); break;                 // around the tile sizes
            case 2: len = (r % 7 == 0) ? 0 : static_cast<int64_t>(1) << (r % 27); break;   // powers of two
            default: len = static_cast<int64_t>(r % (static_cast<uint64_t>(1) << 33)); break;   // beyond 2^32 in all
        }
        offs.push_back(offs.back() + len);
    }
    return offs;
}

static void check_tiles(const std::vector<int64_t>& offs, int64_t cap) {
    const int L = static_cast<int>(offs.size()) - 1;
    std::vector<adasum_tile> tiles;
    std::vector<int32_t> begin;
    build_tiles(offs.data(), L, cap, tiles, begin);
    CHECK(static_cast<int64_t>(tiles.size()) == count_tiles(offs.data(), L, cap));
    CHECK(static_cast<int>(begin.size()) == L + 1 && begin[0] == 0 && begin[L] == static_cast<int32_t>(tiles.size()));
    for (int l = 0; l < L; ++l) {
        int64_t pos = offs[l];
        CHECK(begin[l] <= begin[l + 1]);
        for (int32_t t = begin[l]; t < begin[l + 1]; ++t) {
            CHECK(tiles[t].layer == l && tiles[t].start == pos && tiles[t].len >= 1 && tiles[t].len <= cap);
            // a tile never crosses a global multiple of the capacity
            CHECK(tiles[t].start / cap == (tiles[t].start + tiles[t].len - 1) / cap);
            pos += tiles[t].len;
        }
        CHECK(pos == offs[l + 1]);
    }
}

static void check_schedule(int K, int radix, int order, const std::vector<int64_t>& offs, int dtype) {
    const int L = static_cast<int>(offs.size()) - 1;
    std::vector<int> radices;
    const int rc = order == ADASUM_ORDER_LINEAR ? build_linear_passes(K, radix, radices) : build_levels(K, radix, radices);
    CHECK(rc == ADASUM_OK);
    int Kv = K;
    if (order == ADASUM_ORDER_LINEAR) {
        int covered = 0;
        for (size_t b = 0; b < radices.size(); ++b) {
            CHECK(radices[b] >= 2 && radices[b] <= (radix == 0 ? kDefaultRadix : radix));
            covered += b == 0 ? radices[b] : radices[b] - 1;
        }
        CHECK(covered == (K == 1 ? 0 : K));
    } else {
        Kv = virtual_leaves(radices);
        CHECK(Kv >= K && (K == 1 || Kv < 2 * K));
        CHECK(is_pow2(Kv));
        const int depth = first_depth(radices);
        const int groups = 1 << depth;
        int next = 0;
        for (int g = 0; g < groups && K > 1; ++g) {
            int lo, hi;
            leaf_range(K, depth, g, lo, hi);
            CHECK(lo == next && hi >= lo && hi - lo <= radices[0]);
            next = hi;
        }
        CHECK(K == 1 || next == K);
    }
    std::vector<SmallLayer> small;
    const int64_t small_elems = find_small_layers(offs.data(), L, small);
    int64_t sum = 0;
    for (const SmallLayer& s : small) {
        CHECK(s.len >= 1 && s.len <= kSmallLayer && s.coff == sum && s.start == offs[s.layer]);
        sum += s.len;
    }
    CHECK(sum == small_elems);
    const int node_type = node_dtype(dtype);
    const int gcap = gram_tile_capacity(offs.data(), L);
    CHECK(gcap == kTile || gcap == kTileSmall);
    const int64_t n_tiles = count_tiles(offs.data(), L, gcap);
    const int64_t ne = norm_entries_bound(Kv, offs.data(), L, radices, node_type);
    // (room for what the combines leave for the pass above: the larger of the two schemes)
    int64_t de = 0;
    if (order == ADASUM_ORDER_TREE) {
        de = std::max(dot_entries_bound(Kv, offs.data(), L, radices, node_type),
                      next_entries_bound(Kv, offs.data(), L, radices, node_type));
        int g = Kv;
        for (size_t lv = 0; lv + 1 < radices.size(); ++lv) {
            g /= radices[lv];
            if (!pass_feeds_next(radices, lv)) continue;
            CHECK(radices[lv] * radices[lv + 1] <= kMaxPack && g % radices[lv + 1] == 0);
            const int in = lv == 0 ? dtype : node_type;
            const int64_t ct = count_tiles(offs.data(), L, feed_tile_capacity(in, radices[lv]));
            CHECK(static_cast<int64_t>(g / radices[lv + 1]) * ct * gram_entries(radices[lv + 1], true) <= de);
        }
    }
    // a wide first pass (tree order, 16-bit leaves): its span table and what it leaves per span
    int64_t n_spans = 0;
    if (!radices.empty() && wide_radix(radices[0])) {
        CHECK(order == ADASUM_ORDER_TREE && elem_bytes(dtype) == 2 && radices[0] <= kMaxWideRadix);
        for (size_t lv = 1; lv < radices.size(); ++lv) CHECK(radices[lv] <= kMaxRadix);
        const int n_parts = wide_part_count(offs[L]);
        CHECK(n_parts >= 1 && (n_parts <= kWideParts || wide_part_elems(offs[L], n_parts / 2) > kWideMaxPart));
        const int64_t E = wide_part_elems(offs[L], n_parts);
        CHECK(E % kWidePartAlign == 0 && E * n_parts >= offs[L] && E <= kWideMaxPart);
        std::vector<adasum_tile> spans;
        std::vector<int32_t> part_begin, layer_begin;
        build_spans(offs.data(), L, n_parts, spans, part_begin, layer_begin);
        n_spans = static_cast<int64_t>(spans.size());
        CHECK(n_spans == count_spans(offs.data(), L, n_parts) && n_spans <= static_cast<int64_t>(n_parts) + L);
        CHECK(static_cast<int>(part_begin.size()) == n_parts + 1 && part_begin[0] == 0 && part_begin[n_parts] == n_spans);
        CHECK(static_cast<int>(layer_begin.size()) == L + 1 && layer_begin[L] == n_spans);
        int64_t pos = 0;
        for (int p = 0; p < n_parts; ++p) {
            CHECK(part_begin[p] <= part_begin[p + 1]);
            for (int32_t i = part_begin[p]; i < part_begin[p + 1]; ++i) {
                const adasum_tile& t = spans[static_cast<size_t>(i)];
                // inside its part and its layer, and the spans tile the elements in order
                CHECK(t.len >= 1 && t.start == pos && t.start >= p * E && t.start + t.len <= (p + 1) * E);
                CHECK(t.layer >= 0 && t.layer < L && t.start >= offs[t.layer] && t.start + t.len <= offs[t.layer + 1]);
                CHECK(i >= layer_begin[t.layer] && i < layer_begin[t.layer + 1]);
                pos = t.start + t.len;
            }
        }
        CHECK(pos == offs[L]);
    }
    const Layout lay = make_layout(Kv, offs[L], L, n_tiles, ne, radices, order, K + 1, small_elems, node_type, de, n_spans);
    {
        // room for the widest pass's partials
        int g = Kv;
        for (size_t lv = 0; lv < radices.size(); ++lv) {
            g = order == ADASUM_ORDER_LINEAR ? 1 : g / radices[lv];
            const int64_t rows = wide_radix(radices[lv]) ? n_spans : n_tiles;
            CHECK(lay.off_normparts - lay.off_partials >=
                  static_cast<size_t>(g) * gram_partial_entries(radices[lv]) * static_cast<size_t>(rows) * sizeof(double));
        }
    }
    const size_t sections[] = {lay.off_slots, lay.off_partials, lay.off_normparts, lay.off_normcoarse, lay.off_gram,
                               lay.off_weights, lay.off_leafnorm, lay.off_small, lay.off_dotparts, lay.total};
    CHECK(lay.total - lay.off_dotparts >= static_cast<size_t>(de) * sizeof(double));
    for (size_t i = 0; i + 1 < sizeof(sections) / sizeof(sections[0]); ++i) {
        CHECK(sections[i] % 256 == 0 && sections[i] <= sections[i + 1]);
    }
    CHECK(lay.off_partials - lay.off_slots >= static_cast<size_t>(lay.n_slots) * lay.slot_elems * lay.node_bytes);
    CHECK(lay.off_normcoarse - lay.off_normparts >= static_cast<size_t>(ne) * sizeof(double));
    CHECK(lay.off_dotparts - lay.off_small >= static_cast<size_t>(K + 1) * static_cast<size_t>(small_elems) * sizeof(double));
    // every pass's squared norms fit the reserved entries, for every storage type the pass may read
    int groups = Kv;
    for (size_t lv = 0; lv < radices.size(); ++lv) {
        groups = order == ADASUM_ORDER_LINEAR ? 1 : groups / radices[lv];
        const int in = (lv == 0 || order == ADASUM_ORDER_LINEAR) ? dtype : node_type;
        const int64_t ct = count_tiles(offs.data(), L, combine_tile_capacity(in, radices[lv]));
        CHECK(static_cast<int64_t>(groups) * ct <= ne);
    }
}

int main(int argc, char** argv) {
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 300;
    std::mt19937_64 rng(20060292);
    const int radix_choices[] = {0, 2, 4, 8, 16, 32, 64};
    const int dtypes[] = {ADASUM_F32, ADASUM_BF16, ADASUM_F16, ADASUM_F64};
    const int64_t caps[] = {1, 7, 64, 256, 512, 2048, kTileSmall, kTile};
    // tile capacities the combine kernels are written for: lanes (or half-waves) x one 16-byte granule
    CHECK(combine_tile_capacity(ADASUM_BF16, 16) == 256 && combine_tile_capacity(ADASUM_F16, 16) == 256);
    CHECK(combine_tile_capacity(ADASUM_F32, 16) == 256 && combine_tile_capacity(ADASUM_BF16, 8) == 1024);
    CHECK(combine_tile_capacity(ADASUM_BF16, 64) == 512 && combine_tile_capacity(ADASUM_BF16, 32) == 512);
    CHECK(combine_tile_capacity(ADASUM_F64, 8) == 256 && combine_tile_capacity(ADASUM_F32, 2) == 1024);
    CHECK(feed_tile_capacity(ADASUM_BF16, 16) == 256 && feed_tile_capacity(ADASUM_BF16, 8) == 512);
    CHECK(feed_tile_capacity(ADASUM_F32, 16) == 256 && feed_tile_capacity(ADASUM_F64, 8) == 128);
    for (int dt : dtypes)
        for (int R : {2, 4, 8, 16}) {
            // the planner sizes its sections for the node type's tables: never coarser than the input type's
            CHECK(combine_tile_capacity(node_dtype(dt), R) <= combine_tile_capacity(dt, R));
            CHECK(feed_tile_capacity(node_dtype(dt), R) <= feed_tile_capacity(dt, R));
        }
    for (int it = 0; it < rounds; ++it) {
        const int kind = static_cast<int>(rng() % 4);
        const int n_layers = kind == 3 ? static_cast<int>(rng() % 6) : static_cast<int>(rng() % 2000);
        const std::vector<int64_t> offs = random_table(rng, n_layers, kind);
        CHECK(check_layer_table(offs.data(), n_layers) == ADASUM_OK);
        if (kind != 3) {
            for (int64_t cap : caps) {
                // (a table of 2^33 elements in tiles of 1 would only exhaust memory)
                if (offs.back() / cap < (1 << 22)) check_tiles(offs, cap);
            }
        } else {
            check_tiles(offs, kTile);
        }
        for (int rep = 0; rep < 8; ++rep) {
            int K;
            switch (rng() % 4) {
                case 0: K = 1 + static_cast<int>(rng() % 40); break;
                case 1: K = 1 << (rng() % 21); break;
                case 2: K = (1 << (rng() % 20)) + 1; break;
                default: K = 1 + static_cast<int>(rng() % (1 << 20)); break;
            }
            const int dtype = dtypes[rng() % 4];
            int radix = radix_choices[rng() % 7];
            if (radix > max_radix(dtype) || (radix == 0 && dtype == ADASUM_F64)) radix = 8;
            // (the wide radices exist in the tree order only)
            const int order = (K <= 4096 && !wide_radix(radix) && rng() % 2) ? ADASUM_ORDER_LINEAR : ADASUM_ORDER_TREE;
            check_schedule(K, radix, order, offs, dtype);
        }
    }
    // the error paths
    std::vector<int> r;
    CHECK(build_levels(0, 2, r) == ADASUM_ERR_INVALID_ARG && build_levels(4, 3, r) == ADASUM_ERR_UNSUPPORTED);
    CHECK(build_linear_passes(0, 2, r) == ADASUM_ERR_INVALID_ARG && build_linear_passes(4, 5, r) == ADASUM_ERR_UNSUPPORTED);
    const int64_t bad1[] = {1, 2}, bad2[] = {0, 5, 3};
    CHECK(check_layer_table(bad1, 1) == ADASUM_ERR_INVALID_ARG && check_layer_table(bad2, 2) == ADASUM_ERR_INVALID_ARG);
    CHECK(check_layer_table(nullptr, 1) == ADASUM_ERR_INVALID_ARG && check_layer_table(bad1, -1) == ADASUM_ERR_INVALID_ARG);
    std::printf("planner ok: %d random tables\n", rounds);
    return 0;
}
