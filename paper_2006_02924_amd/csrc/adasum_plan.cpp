// Host-side planning for the Adasum tree combiner: layer-table validation, the
// tile table (the bookkeeping of tensor boundaries inside the fused buffer,
// Section 4.4.3 of arXiv 2006.02924), the pass schedule over the binary tree of
// Section 3.4, and the device workspace layout.  Pure C++, no GPU calls.
#include "adasum_host.h"

#include <algorithm>



namespace adasum {

int check_layer_table(const int64_t* layer_offsets, int n_layers) {
    if (n_layers < 0) return ADASUM_ERR_INVALID_ARG;
    if (layer_offsets == nullptr) return ADASUM_ERR_INVALID_ARG;
    if (layer_offsets[0] != 0) return ADASUM_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        if (layer_offsets[l + 1] < layer_offsets[l]) return ADASUM_ERR_INVALID_ARG;
    }
    return ADASUM_OK;
}

void build_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity,
                 std::vector<adasum_tile>& tiles, std::vector<int32_t>& layer_tile_begin) {
    tiles.clear();
    layer_tile_begin.assign(static_cast<size_t>(n_layers) + 1, 0);
    for (int l = 0; l < n_layers; ++l) {
        layer_tile_begin[l] = static_cast<int32_t>(tiles.size());
        int64_t pos = layer_offsets[l];
        const int64_t end = layer_offsets[l + 1];
        while (pos < end) {
            // next global multiple of the capacity strictly above pos, clipped to the layer
            int64_t stop = (pos / capacity + 1) * capacity;
            if (stop > end) stop = end;
            adasum_tile t;
            t.start = pos;
            t.len = static_cast<int32_t>(stop - pos);
            t.layer = l;
            tiles.push_back(t);
            pos = stop;
        }
    }
    layer_tile_begin[n_layers] = static_cast<int32_t>(tiles.size());
}

int build_levels(int K, int radix, std::vector<int>& radices) {
    radices.clear();
    if (K < 1) return ADASUM_ERR_INVALID_ARG;
    if (radix == 0) radix = kDefaultRadix;
    if (radix != 2 && radix != 4 && radix != 8 && radix != 16 && radix != 32 && radix != 64) return ADASUM_ERR_UNSUPPORTED;
    if (K == 1) return ADASUM_OK;
    // the shallowest depth whose sub-trees have at most `radix` leaves
    int depth = 0;
    while ((K + (1 << depth) - 1) / (1 << depth) > radix) ++depth;
    const int widest = (K + (1 << depth) - 1) / (1 << depth);
    int first = 2;
    while (first < widest) first *= 2;
    radices.push_back(first);
    int rest = 1 << depth;
    while (rest > 1) {
        // (only the first pass, over the 16-bit leaves, can be wider than kMaxRadix)
        int r = std::min(rest, std::min(radix, kMaxRadix));
        radices.push_back(r);
        rest /= r;
    }
    return ADASUM_OK;
}

int build_linear_passes(int K, int radix, std::vector<int>& passes) {
    passes.clear();
    if (K < 1) return ADASUM_ERR_INVALID_ARG;
    if (radix == 0) radix = kDefaultRadix;
    if (radix != 2 && radix != 4 && radix != 8 && radix != 16) return ADASUM_ERR_UNSUPPORTED;
    if (K == 1) return ADASUM_OK;
    int first = radix;
    while (first > K) first /= 2;
    passes.push_back(first);
    int rest = K - first;
    while (rest > 0) {
        int r = radix;
        while (r - 1 > rest) r /= 2;
        passes.push_back(r);
        rest -= r - 1;
    }
    return ADASUM_OK;
}

int wide_part_count(int64_t N) {
    int64_t parts = (N + kWidePartAlign - 1) / kWidePartAlign;
    if (parts > kWideParts) parts = kWideParts;
    if (parts < 1) parts = 1;
    // a part is what one wave quarter sums in fp32 before it widens: kept to kWideMaxPart elements, so
    // very long buffers get more parts than the chip holds workgroups (they run in several rounds)
    while (wide_part_elems(N, static_cast<int>(parts)) > kWideMaxPart) parts *= 2;
    return static_cast<int>(parts);
}

int64_t wide_part_elems(int64_t N, int n_parts) {
    const int64_t e = (N + n_parts - 1) / n_parts;
    return (e + kWidePartAlign - 1) / kWidePartAlign * kWidePartAlign;
}

void build_spans(const int64_t* layer_offsets, int n_layers, int n_parts, std::vector<adasum_tile>& spans,
                 std::vector<int32_t>& part_begin, std::vector<int32_t>& layer_begin) {
    // tiles whose capacity is a part: cut at the part boundaries and at the layer boundaries, sorted by
    // start, so the spans of a part are one contiguous run as those of a layer are
    const int64_t E = wide_part_elems(layer_offsets[n_layers], n_parts);
    build_tiles(layer_offsets, n_layers, E, spans, layer_begin);
    part_begin.assign(static_cast<size_t>(n_parts) + 1, 0);
    for (const adasum_tile& t : spans) ++part_begin[static_cast<size_t>(t.start / E) + 1];
    for (int p = 0; p < n_parts; ++p) part_begin[p + 1] += part_begin[p];
}

int64_t count_spans(const int64_t* layer_offsets, int n_layers, int n_parts) {
    const int64_t E = wide_part_elems(layer_offsets[n_layers], n_parts);
    return count_tiles(layer_offsets, n_layers, E);
}

int64_t find_small_layers(const int64_t* layer_offsets, int n_layers, std::vector<SmallLayer>& small) {
    small.clear();
    int64_t total = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int64_t len = layer_offsets[l + 1] - layer_offsets[l];
        if (len < 1 || len > kSmallLayer) continue;
        SmallLayer s;
        s.start = layer_offsets[l];
        s.len = static_cast<int32_t>(len);
        s.layer = l;
        s.coff = static_cast<int32_t>(total);
        s.pad = 0;
        small.push_back(s);
        total += len;
    }
    return total;
}

int64_t count_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity) {
    int64_t n = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int64_t lo = layer_offsets[l], hi = layer_offsets[l + 1];
        if (hi > lo) n += (hi - 1) / capacity - lo / capacity + 1;
    }
    return n;
}

int gram_tile_capacity(const int64_t* layer_offsets, int n_layers) {
    return count_tiles(layer_offsets, n_layers, kTile) < kFewTiles ? kTileSmall : kTile;
}

int64_t norm_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices,
                           int node_type) {
    int64_t need = 1;
    int groups = K;
    for (size_t lv = 0; lv < radices.size(); ++lv) {
        groups /= radices[lv];
        // the widest storage type a pass may read gives its finest table
        const int64_t t = count_tiles(layer_offsets, n_layers, combine_tile_capacity(node_type, radices[lv]));
        // (the left-to-right order has one group per pass)
        need = std::max<int64_t>(need, static_cast<int64_t>(std::max(groups, 1)) * t);
    }
    if (radices.empty())
        need = std::max<int64_t>(need, count_tiles(layer_offsets, n_layers, combine_tile_capacity(node_type, 1)));
    return need;
}

int64_t next_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices,
                           int node_type) {
    int64_t need = 0;
    int groups = K;
    for (size_t lv = 0; lv + 1 < radices.size(); ++lv) {
        groups /= radices[lv];
        if (!pass_feeds_next(radices, lv)) continue;
        const int R2 = radices[lv + 1];
        // the widest storage type a pass may read gives its finest table
        const int64_t t = count_tiles(layer_offsets, n_layers, feed_tile_capacity(node_type, radices[lv]));
        need = std::max<int64_t>(need, static_cast<int64_t>(groups / R2) * t * gram_entries(R2, true));
    }
    return need;
}

int64_t dot_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices,
                          int node_type) {
    int64_t need = 0;
    int groups = K;
    for (size_t lv = 0; lv + 1 < radices.size(); ++lv) {
        groups /= radices[lv];
        if (radices[lv] != 2) continue;
        const int64_t t = count_tiles(layer_offsets, n_layers, combine_tile_capacity(node_type, 2));
        need = std::max<int64_t>(need, static_cast<int64_t>(groups / 2) * t);
    }
    return need;
}

Layout make_layout(int K, int64_t N, int n_layers, int64_t n_tiles, int64_t norm_entries,
                   const std::vector<int>& radices, int order, int64_t small_rows, int64_t small_elems,
                   int node_type, int64_t dot_entries, int64_t wide_spans) {
    Layout lay;
    lay.N = N;
    lay.n_tiles = n_tiles;
    lay.norm_entries = norm_entries;
    lay.n_layers = n_layers;
    lay.slot_elems = static_cast<int64_t>(align_up(static_cast<size_t>(N), 64));
    lay.node_bytes = elem_bytes(node_type);
    // nodes written by the first pass, unless that pass is already the root
    lay.n_slots = radices.size() > 1 ? K / radices[0] : 0;

    size_t max_partials = 0, max_gram = 0, max_weights = 0, max_nodes = 1;
    int groups = K;
    if (order == ADASUM_ORDER_LINEAR) {
        // one group per pass; slot 0 holds the running result
        lay.n_slots = radices.size() > 1 ? 1 : 0;
    }
    for (size_t lv = 0; lv < radices.size(); ++lv) {
        const int R = radices[lv];
        groups = order == ADASUM_ORDER_LINEAR ? 1 : groups / R;
        // (with the diagonal: a pass fed by the combine below it finds its whole matrix in the partials)
        const size_t np = static_cast<size_t>(gram_partial_entries(R));
        // (a wide pass -- always the first -- leaves its blocks per span, every other pass per Gram tile)
        const size_t rows = wide_radix(R) ? static_cast<size_t>(wide_spans) : static_cast<size_t>(n_tiles);
        max_partials = std::max(max_partials, static_cast<size_t>(groups) * np * rows);
        max_gram = std::max(max_gram, static_cast<size_t>(groups) * n_layers * R * R);
        max_weights = std::max(max_weights, static_cast<size_t>(groups) * n_layers * R);
        max_nodes = std::max(max_nodes, static_cast<size_t>(groups));
    }
    size_t off = 0;
    lay.off_slots = off;
    off = align_up(off + static_cast<size_t>(lay.n_slots) * lay.slot_elems * lay.node_bytes, 256);
    lay.off_partials = off;
    off = align_up(off + max_partials * sizeof(double), 256);
    lay.off_normparts = off;
    off = align_up(off + static_cast<size_t>(norm_entries) * sizeof(double), 256);
    lay.off_normcoarse = off;
    off = align_up(off + max_nodes * static_cast<size_t>(n_tiles) * sizeof(double), 256);
    lay.off_gram = off;
    off = align_up(off + max_gram * sizeof(double), 256);
    lay.off_weights = off;
    off = align_up(off + max_weights * sizeof(double), 256);
    lay.off_leafnorm = off;
    off = align_up(off + static_cast<size_t>(n_layers) * sizeof(double), 256);
    lay.off_small = off;
    lay.small_elems = small_elems;
    off = align_up(off + static_cast<size_t>(small_rows) * static_cast<size_t>(small_elems) * sizeof(double), 256);
    lay.off_dotparts = off;
    lay.dot_entries = dot_entries;
    off = align_up(off + static_cast<size_t>(dot_entries) * sizeof(double), 256);
    lay.total = off;
    return lay;
}

}  // namespace adasum
