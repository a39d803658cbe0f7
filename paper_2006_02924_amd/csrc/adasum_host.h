// Internal host-side declarations shared by the planner, the kernel launchers
// and the C-ABI layer of libadasum.  Nothing here is exported.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "adasum.h"

namespace adasum {

// Elements one Gram workgroup covers at most (a long tile amortises the
// workgroup's start-up and its reduction of up to 136 values).  A multiple of every
// granule (4 fp32 or 8 bf16 elements per 16-byte access) times the workgroup size.
#ifndef ADASUM_TILE
#define ADASUM_TILE 65536
#endif
#ifndef ADASUM_THREADS
#define ADASUM_THREADS 256
#endif
constexpr int kTile = ADASUM_TILE;
// Small problems (fewer than kFewTiles long tiles: not even a few workgroups per compute
// unit) are cut into shorter Gram tiles so that the pass still fills the chip evenly.
constexpr int kTileSmall = 16384;
constexpr int kFewTiles = 2048;
constexpr int kThreads = ADASUM_THREADS;
// A combine workgroup covers one 16-byte load per lane and operand and then
// ends: short-lived workgroups that walk memory in launch order keep the mixed
// read/write stream close to sequential.  Measured on MI355X, such a workgroup
// streams best when it moves 16-20 KB in all, so wider groups get fewer lanes.
constexpr int combine_threads(int R) { return R >= 16 ? 64 : (R >= 8 ? 128 : 256); }
// Sixteen operands of a 16-bit type: a load instruction takes 512 bytes of two operands (lanes 0-31 the
// even-numbered ones, lanes 32-63 the odd-numbered ones) instead of 1 KB of one, the halves add up what
// they hold with one exchange, and each stores half of the tile's result.  The wave then moves 9-10 KB
// and ends; measured on MI355X this streams 8-15 % faster than 1 KB per operand and wave.
constexpr bool combine_pairs_operands(int elem_size, int R) { return elem_size == 2 && R == 16; }
// Granules (16 input bytes) of a combine tile, hence its capacity: depends on the input type and the radix.
inline int elem_bytes(int dtype) { return dtype == ADASUM_F64 ? 8 : dtype == ADASUM_F32 ? 4 : 2; }
inline int combine_tile_capacity(int dtype, int R) {
    const int granules = combine_pairs_operands(elem_bytes(dtype), R) ? 32 : combine_threads(R);
    return granules * (16 / elem_bytes(dtype));
}

// Largest number of explicit operand pointers one launch carries by value.
constexpr int kMaxPack = 128;
// Widest pass of the vector-unit kernels (136 Gram entries per lane), and of the wide first pass
// (16-bit leaves only), whose Gram entries are 32 x 32 blocks from the matrix cores.
constexpr int kMaxRadix = 16;
constexpr int kMaxWideRadix = 64;
inline bool wide_radix(int R) { return R > kMaxRadix; }
// 32 x 32 blocks a wide Gram pass keeps per tile: the three distinct ones of a 64 x 64 matrix, or one.
constexpr int wide_blocks(int R) { return R == 64 ? 3 : 1; }
// Radix used when the caller asks for 0: the widest pass moves the fewest bytes.
constexpr int kDefaultRadix = 16;

inline bool known_dtype(int dtype) { return dtype == ADASUM_F32 || dtype == ADASUM_BF16 || dtype == ADASUM_F16 || dtype == ADASUM_F64; }
// Storage type of the intermediate tree nodes for an input type.
inline int node_dtype(int dtype) { return dtype == ADASUM_F64 ? ADASUM_F64 : ADASUM_F32; }
// Widest radix a storage type is instantiated for.
inline int max_radix(int dtype) {
    return dtype == ADASUM_F64 ? 8 : (dtype == ADASUM_BF16 || dtype == ADASUM_F16) ? kMaxWideRadix : kMaxRadix;
}
// Output storage types a combine supports for an input type: the same type or fp32; any type from fp32.
inline bool dtype_pair_ok(int in, int out) {
    if (!known_dtype(in) || !known_dtype(out)) return false;
    if (in == ADASUM_F64 || out == ADASUM_F64) return in == out;
    return in == out || in == ADASUM_F32 || out == ADASUM_F32;
}
inline bool is_pow2(long long v) { return v > 0 && (v & (v - 1)) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- planning (pure host code) ----------------------------------------------

// Validates a layer table; returns ADASUM_OK or an error code.
int check_layer_table(const int64_t* layer_offsets, int n_layers);

// Tile table: boundaries at layer boundaries and at global multiples of `capacity`.
// layer_tile_begin[l] .. layer_tile_begin[l+1] are the tiles of layer l.
void build_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity,
                 std::vector<adasum_tile>& tiles, std::vector<int32_t>& layer_tile_begin);

// The halving tree of Section 3.4 over K leaves, for any K: the node over leaves [lo, hi)
// splits at lo + (hi - lo) / 2, i.e. the left part takes floor(count / 2) leaves (for a
// power of two, the balanced tree).  Returns the leaves of node g of depth `depth`
// (g's bits from the most significant: 1 = right child).  Sizes at one depth differ by at
// most one.  Host and device.
constexpr void leaf_range(int K, int depth, int g, int& lo, int& hi) {
    lo = 0;
    hi = K;
    for (int b = depth - 1; b >= 0; --b) {
        const int mid = lo + (hi - lo) / 2;
        if ((g >> b) & 1) lo = mid;
        else hi = mid;
    }
}

// Radix of every pass.  The first pass takes the sub-trees of depth `first_depth(radices)`
// as its groups: at most radices[0] leaves each (fewer when K is not a power of two; a
// short group is padded up to the radix with repeats of its first leaf, which get weight
// 0).  Above them the tree is a balanced one over 2^depth nodes.  The product of the
// radices is K for a power of two, else the next power of two.  Largest radices first
// (the first pass reads the narrow input dtype and touches the most data).
int build_levels(int K, int radix, std::vector<int>& radices);
inline int virtual_leaves(const std::vector<int>& radices) {
    int v = 1;
    for (int r : radices) v *= r;
    return v;
}
inline int first_depth(const std::vector<int>& radices) {
    int groups = radices.empty() ? 1 : virtual_leaves(radices) / radices[0];
    int d = 0;
    while ((1 << d) < groups) ++d;
    return d;
}

// Left-to-right order (Section 3.4, first recursion): operand counts of the
// passes.  The first pass folds the largest power of two of leaves that is at most
// min(K, radix); every later pass folds
// the running result with up to radix - 1 further leaves (operand 0 is the
// running result), using the widest instantiated radix that the remaining
// leaves fill.  E.g. K = 64, radix 16 -> {16, 16, 16, 16, 4}.
int build_linear_passes(int K, int radix, std::vector<int>& passes);

// A pass of the tree order can leave the next pass's Gram entries itself: its combine then takes
// the radices[lv + 1] sibling groups of a tile in one workgroup (one wave per group), the waves
// exchange what they wrote through LDS, and the squared norms and dot products of those nodes --
// the whole Gram matrix of the next pass's group -- go out per tile, so the next pass makes no
// reduce pass of its own.  Possible when the operand pointers of the sibling groups fit one launch.
inline bool pass_feeds_next(const std::vector<int>& radices, size_t lv) {
    return lv + 1 < radices.size() && radices[lv] <= kMaxRadix && radices[lv] * radices[lv + 1] <= kMaxPack;
}
// Lanes per group in such a combine (one wave), hence its tile capacity (pairs of operands per load
// as above).
constexpr int kFeedLanes = 64;
inline int feed_tile_capacity(int dtype, int R) {
    const int granules = combine_pairs_operands(elem_bytes(dtype), R) ? 32 : kFeedLanes;
    return granules * (16 / elem_bytes(dtype));
}

// Number of Gram entries a pass of radix R accumulates per tile: all pairs
// i < j, plus the R diagonal entries when `diag` (the first pass; later passes
// get their squared norms from the previous combine).
inline int gram_entries(int R, bool diag) { return R * (R - 1) / 2 + (diag ? R : 0); }
// Doubles a pass of radix R may leave per (group, Gram tile): its entries with the diagonal, or the
// whole blocks of a wide pass.
inline int gram_partial_entries(int R) { return wide_radix(R) ? wide_blocks(R) * 1024 : gram_entries(R, true); }

// The wide first pass (radix 32 and 64) walks spans instead of fixed-size tiles: the elements are cut
// into `n_parts` equal parts (one workgroup each; boundaries at multiples of kWidePartAlign), and a part
// into spans at the layer boundaries.  One set of Gram blocks is written per span, so the pass stores
// as rarely as it can.  spans[part_begin[p]] .. [part_begin[p + 1]] are the spans of part p, and
// layer_begin[l] .. [l + 1] those of layer l (both runs are contiguous: the spans are sorted by start).
constexpr int kWideParts = 512;          // two workgroups of the wide Gram kernel fit a compute unit: 2 x 256
constexpr int kWidePartAlign = 2048;     // elements; a part holds at least this many
constexpr int64_t kWideMaxPart = 1 << 20;   // and at most this many (bounds the fp32 sums of the wide Gram pass)
int wide_part_count(int64_t N);
int64_t wide_part_elems(int64_t N, int n_parts);
void build_spans(const int64_t* layer_offsets, int n_layers, int n_parts, std::vector<adasum_tile>& spans,
                 std::vector<int32_t>& part_begin, std::vector<int32_t>& layer_begin);
int64_t count_spans(const int64_t* layer_offsets, int n_layers, int n_parts);

// Layers of at most kSmallLayer elements are reduced a second time by the definition
// itself, pair by pair in fp64 over all K workers with no stored intermediate, and that
// result replaces what the passes wrote.  Vectors of a few elements can nearly cancel at
// a tree node (two scalars of opposite sign do so with probability ~eps); the relative
// error of an fp32 node is amplified by 1/eps there, and the Gram route's scalars by its
// square, so the passes alone cannot hold a relative bound on such layers.  From some ten
// elements on the chance of a cancellation is negligible.
constexpr int kSmallLayer = 16;
struct SmallLayer {
    int64_t start;   // first element in the fused buffer
    int32_t len;     // 1 .. kSmallLayer
    int32_t layer;
    int32_t coff;    // first element in a row of the compact copy
    int32_t pad;
};
// Small layers of a layer table; returns the elements they hold in total.
int64_t find_small_layers(const int64_t* layer_offsets, int n_layers, std::vector<SmallLayer>& small);

// Device workspace layout (byte offsets from a 256-byte aligned base).
struct Layout {
    int64_t N = 0;            // elements per gradient
    int64_t slot_elems = 0;   // N rounded up so that slots stay 256-byte aligned
    int64_t n_slots = 0;      // intermediate tree nodes after the first pass
    int     node_bytes = 4;   // element size of a node: 4 (fp32), 8 for fp64 inputs
    int64_t n_tiles = 0;      // Gram tiles
    int64_t norm_entries = 0; // doubles reserved for the combines' squared norms
    int     n_layers = 0;
    size_t  off_slots = 0;    // n_slots x slot_elems x node_bytes
    size_t  off_partials = 0; // doubles [group][tile][entry], sized for the widest pass
    size_t  off_normparts = 0;// doubles [node][combine tile]: squared norm of every node a combine wrote
    size_t  off_normcoarse = 0;// doubles [node][Gram tile]: the same, summed per Gram tile
    size_t  off_gram = 0;     // doubles [group][layer][R*R] (finished Gram matrices)
    size_t  off_weights = 0;  // doubles [group][layer][R]
    size_t  off_leafnorm = 0; // doubles [layer]: sum over workers of the input squared norms
    size_t  off_small = 0;    // doubles [K + 1][small_elems]: the small layers of every worker, widened
                              // (row K: those of delta_start)
    int64_t small_elems = 0;
    size_t  off_dotparts = 0; // doubles [sibling pair][combine tile]: dot product of the two nodes a
                              // sibling-fused combine wrote (only with fuse_siblings)
    int64_t dot_entries = 0;
    size_t  total = 0;
};
// `norm_entries`: doubles needed for the squared norms the combines leave
// (max over passes of nodes written x combine tiles of that pass).
// `K` is the padded leaf count in the tree order; `small_rows` x `small_elems` doubles are
// reserved for the compact copy of the small layers.
// `wide_spans`: spans of a wide first pass (count_spans), which sizes that pass's partials.
Layout make_layout(int K, int64_t N, int n_layers, int64_t n_tiles, int64_t norm_entries,
                   const std::vector<int>& radices, int order = ADASUM_ORDER_TREE, int64_t small_rows = 0,
                   int64_t small_elems = 0, int node_type = ADASUM_F32, int64_t dot_entries = 0,
                   int64_t wide_spans = 0);
// Doubles the passes that feed the next one (pass_feeds_next) need for the Gram entries they leave:
// the most any of them writes, next pass's groups x combine tiles x entries of a full Gram matrix.
int64_t next_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices,
                           int node_type = ADASUM_F32);
// Doubles a sibling-fused radix-2 schedule needs for the dot products its combines leave: the most
// any level but the last writes, pairs of groups x combine tiles of that level.
int64_t dot_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices,
                          int node_type = ADASUM_F32);
// Number of tiles build_tiles would produce.
int64_t count_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity);
// Gram tile capacity for a layer table: kTile, or kTileSmall for a small problem.
int gram_tile_capacity(const int64_t* layer_offsets, int n_layers);
// Upper bound (over input dtypes) of make_layout's norm_entries for a schedule.
int64_t norm_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices,
                           int node_type = ADASUM_F32);

// ---- kernel launchers (adasum_kernels.hip) -----------------------------------

// Operand r of group g is pack[g * R + r]: explicit device pointers carried by
// value in the kernel arguments (one contiguous run of R pointers per group, so a
// workgroup fetches its operands with one wide scalar load).
struct Operands {
    const void* pack[kMaxPack];
};

// Same idea for where a combine writes group g's result.
struct Outputs {
    char*     base;        // explicit single output when n_groups == 1 and stride == 0
    long long slot_bytes;
    int       stride;      // group g writes slot g*stride
};

// Device-side view of one tile table.
struct TileSet {
    const adasum_tile* tiles = nullptr;      // device
    const int32_t* layer_begin = nullptr;    // device, n_layers + 1
    // combine tables only: device, n_gram_tiles + 1; the tiles of this table
    // that lie inside Gram tile t are first_in_gram[t] .. first_in_gram[t + 1]
    const int32_t* first_in_gram = nullptr;
    int64_t n_tiles = 0;
    int capacity = 0;                        // elements a tile holds at most
    // span tables (wide first pass) only: device, n_parts + 1
    const int32_t* part_begin = nullptr;
    int n_parts = 0;
};

// All launchers return a hipError_t as int (0 = success) and enqueue on `stream`.
// partials[(group * gt.n_tiles + tile) * entries + entry]
// delta_start (or null): operands are x_r - delta_start, same storage type as the operands; diag only.
// A wide pass (R = 32, 64; 16-bit `dtype`, diag, no delta) takes the span table for `gt` and writes
// partials[(group * gt.n_tiles + span) * gram_partial_entries(R) + ...].
int launch_gram(int dtype, bool diag, const Operands& ops, const TileSet& gt, int n_groups, int R,
                double* partials, const void* delta_start, void* stream);
// coarse[node * gt.n_tiles + t] = sum of fine[node * ct.n_tiles + c] over the combine tiles c inside
// Gram tile t.
int launch_norm_coarsen(const double* fine, int n_nodes, const TileSet& ct, const TileSet& gt, double* coarse,
                        void* stream);
// Sums the per-tile partials (and, when !diag, the coarsened squared norms
// normparts[(group * R + i) * gt.n_tiles + tile] of the operand nodes) into full
// R x R Gram matrices gram[group][layer][R*R].
int launch_gram_finish(bool diag, const TileSet& gt, int n_layers, int n_groups, int R,
                       const double* partials, const double* normparts, double* gram,
                       double* weights /* or null: step 2b is not done here */, int order, int K_leaves, int depth,
                       void* stream);
// Gram matrices -> per-layer weights of the binary (or linear) tree over R leaves.
// Item i is (group i / n_layers, layer i % n_layers).  K_leaves > 0: group g holds only the
// leaves of node g of depth `depth` in the halving tree over K_leaves (leaf_range), in its
// first operands; the rest are padding and get weight 0.  K_leaves = 0: every group is full.
int launch_weights(const double* gram, int R, int64_t n_items, int order, int n_layers, int K_leaves, int depth,
                   double* weights, void* stream);
// `ct` must be the table of capacity combine_tile_capacity(dtype, R);
// normparts[group * ct.n_tiles + tile] (or null).
int launch_combine(int dtype, int out_dtype, const Operands& ops, const Outputs& out,
                   const TileSet& ct, int n_layers, int n_groups, int R,
                   const double* weights /* or null: unit weights */, double* normparts,
                   const void* sub_in /* type of the operands, or null */,
                   const void* add_out /* type of the output, or null */, void* stream);
// Step 3 for the sibling pairs of one radix-2 level at once (the tree recursion of Section 3.4 taken two
// pairs at a time): group 2j combines operands (4j, 4j+1) into node P, group 2j+1 combines (4j+2, 4j+3) into
// node Q, one workgroup does both for a tile and also leaves P.Q, so that the level above needs no pass of
// its own over P and Q: dotparts[j * ct.n_tiles + tile], normparts[(2j | 2j+1) * ct.n_tiles + tile].
// n_groups must be even; `ct` the table of capacity combine_tile_capacity(dtype, 2).
int launch_combine_siblings(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                            int n_layers, int n_groups, const double* weights, double* normparts, double* dotparts,
                            void* stream);
// Step 3 of a pass that feeds the next one (pass_feeds_next): workgroup (tile, s) combines the R2
// sibling groups s * R2 .. s * R2 + R2 - 1 of the tile, one wave each, and leaves the full Gram
// matrix of the nodes it wrote: nextparts[(s * ct.n_tiles + tile) * NP2 + entry], entries in the
// Gram pass's order with the diagonal, NP2 = R2 (R2 + 1) / 2.  n_groups must be a multiple of R2
// and n_groups * R at most kMaxPack; `ct` the table of capacity feed_tile_capacity(dtype, R).
int launch_combine_feed(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                        int n_layers, int n_groups, int R, int R2, const double* weights, double* nextparts,
                        void* stream);
// coarse[(s * gt.n_tiles + t) * NP + e] = sum of fine[(s * ct.n_tiles + c) * NP + e] over the combine
// tiles c inside Gram tile t (the rows are whole sets of NP Gram entries).
int launch_parts_coarsen(const double* fine, int n_rows, int NP, const TileSet& ct, const TileSet& gt,
                         double* coarse, void* stream);
// Steps 1 and 3 for one group whose operand 0 is stored as fp32 while operands 1..R-1 are
// 16-bit (`dtype`): the running result of the left-to-right order folded with the next leaves.
// Always the full Gram matrix (diagonal included); tiles as for `dtype`.
int launch_gram_head32(int dtype, const Operands& ops, const TileSet& gt, int R, double* partials, void* stream);
int launch_combine_head32(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                          int n_layers, int R, const double* weights, double* normparts, void* stream);
// layer_sum[l * out_stride] = sum over `n_rows` rows and the tiles of layer l of parts[row][tile].
int launch_layer_sums(const double* parts, int n_rows, const TileSet& t, int n_layers,
                      double* layer_sum, int out_stride, void* stream);
// out[l * out_stride] = sum over groups of the diagonal entries first_entry.. of gram[group][l]
// (over each group's real leaves: K_leaves and depth as in launch_weights); `accumulate` adds to
// what out holds instead of replacing it.
int launch_trace_sums(const double* gram, int R, int n_groups, int n_layers, int K_leaves, int depth,
                      int first_entry, bool accumulate, double* out, int out_stride, void* stream);

// Copies the small layers of `n_leaves` operands (ops.pack[0..n_leaves)), widened to fp64 and
// minus `delta_start` when given, into rows leaf0.. of the compact copy; with `stash_start`
// also delta_start's own small layers into row `start_row`.
int launch_small_gather(int dtype, const Operands& ops, int n_leaves, int leaf0, const SmallLayer* small,
                        int n_small, int64_t small_elems, const void* delta_start, bool stash_start,
                        int start_row, double* compact, void* stream);
// Reduces every small layer over the K rows of the compact copy by the definition (tree or
// left-to-right), adds row `start_row` when add_start, stores to `out` (out_dtype) and, when
// stats is given, writes stats[layer][0..1].
int launch_small_reduce(int out_dtype, const double* compact, int K, const SmallLayer* small, int n_small,
                        int64_t small_elems, int order, bool add_start, int start_row, void* out, double* stats,
                        void* stream);

const char* kernel_name(const char* kind, int dtype, int out_dtype, int R, bool diag, char* buf, size_t n);

// ---- set-up without allocation (adasum_reduce_noalloc) ---------------------------

// Device address and size of the library's static scratch array on the current device
// (looked up once per device).  Returns a hipError_t as int.
int static_scratch(char** base, size_t* bytes);
// Copies a host layer table (n_layers + 1 entries) to `d_offsets` through kernel arguments,
// a few hundred entries per launch: no copy engine, no staging buffer.
int launch_put_offsets(const int64_t* layer_offsets, int n_layers, int64_t* d_offsets, void* stream);
// The same for any small host table of 8-byte words.
int launch_put_words(const int64_t* words, size_t n_words, int64_t* d_words, void* stream);
// The device-side twin of build_tiles: writes the tile table of `capacity` elements for the
// layer table at d_offsets.  `n_tiles` must be count_tiles(...) for the same table.
int launch_build_tiles(const int64_t* d_offsets, int n_layers, int64_t capacity, int64_t n_tiles,
                       adasum_tile* d_tiles, int32_t* d_layer_begin, void* stream);
// first_in_gram[t] = first tile of the combine table (capacity `ccap`, a divisor of the Gram
// tiles' capacity) inside Gram tile t; first_in_gram[n_gram] = n_comb.
int launch_index_tiles(const int64_t* d_offsets, const adasum_tile* d_gram_tiles, int64_t n_gram, int64_t ccap,
                       const int32_t* d_comb_layer_begin, int64_t n_comb, int32_t* d_first_in_gram, void* stream);
// The device-side twin of find_small_layers; `n_small` must be what that returns in `small`.
int launch_build_small(const int64_t* d_offsets, int n_layers, int n_small, SmallLayer* d_small, void* stream);

}  // namespace adasum
