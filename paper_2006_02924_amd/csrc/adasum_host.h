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
// workgroup's start-up and its 36-value reduction).  A multiple of every
// granule (4 fp32 or 8 bf16 elements per 16-byte access) times the workgroup size.
#ifndef ADASUM_TILE
#define ADASUM_TILE 65536
#endif
#ifndef ADASUM_THREADS
#define ADASUM_THREADS 256
#endif
constexpr int kTile = ADASUM_TILE;
constexpr int kThreads = ADASUM_THREADS;
// A combine workgroup covers one 16-byte load per lane and operand and then
// ends: short-lived workgroups that walk memory in launch order keep the mixed
// read/write stream close to sequential.  Measured on MI355X, such a workgroup
// streams best when it moves 16-20 KB in all, so wider groups get fewer lanes.
constexpr int combine_threads(int R) { return R >= 16 ? 64 : (R >= 8 ? 128 : 256); }
// Tile capacity of the combine pass: depends on the input type and the radix.
inline int combine_tile_capacity(int dtype, int R) { return combine_threads(R) * (dtype == ADASUM_F32 ? 4 : 8); }

// Largest number of explicit operand pointers one launch carries by value.
constexpr int kMaxPack = 128;
constexpr int kMaxRadix = 16;
// Radix used when the caller asks for 0: the widest pass moves the fewest bytes.
constexpr int kDefaultRadix = 16;

inline int elem_bytes(int dtype) { return dtype == ADASUM_F32 ? 4 : 2; }
inline bool known_dtype(int dtype) { return dtype == ADASUM_F32 || dtype == ADASUM_BF16 || dtype == ADASUM_F16; }
// Output storage types a combine supports for an input type: the same type or fp32; any type from fp32.
inline bool dtype_pair_ok(int in, int out) { return known_dtype(in) && known_dtype(out) && (in == out || in == ADASUM_F32 || out == ADASUM_F32); }
inline bool is_pow2(long long v) { return v > 0 && (v & (v - 1)) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- planning (pure host code) ----------------------------------------------

// Validates a layer table; returns ADASUM_OK or an error code.
int check_layer_table(const int64_t* layer_offsets, int n_layers);

// Tile table: boundaries at layer boundaries and at global multiples of `capacity`.
// layer_tile_begin[l] .. layer_tile_begin[l+1] are the tiles of layer l.
void build_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity,
                 std::vector<adasum_tile>& tiles, std::vector<int32_t>& layer_tile_begin);

// Radix of every pass; product equals K.  Largest radices first (the first pass
// reads the narrow input dtype and touches the most data).
int build_levels(int K, int radix, std::vector<int>& radices);

// Left-to-right order (Section 3.4, first recursion): operand counts of the
// passes.  The first pass folds `min(K, radix)` leaves; every later pass folds
// the running result with up to radix - 1 further leaves (operand 0 is the
// running result), using the widest instantiated radix that the remaining
// leaves fill.  E.g. K = 64, radix 16 -> {16, 16, 16, 16, 4}.
int build_linear_passes(int K, int radix, std::vector<int>& passes);

// Number of Gram entries a pass of radix R accumulates per tile: all pairs
// i < j, plus the R diagonal entries when `diag` (the first pass; later passes
// get their squared norms from the previous combine).
inline int gram_entries(int R, bool diag) { return R * (R - 1) / 2 + (diag ? R : 0); }

// Device workspace layout (byte offsets from a 256-byte aligned base).
struct Layout {
    int64_t N = 0;            // elements per gradient
    int64_t slot_elems = 0;   // N rounded up so that fp32 slots stay 256-byte aligned
    int64_t n_slots = 0;      // fp32 intermediate tree nodes after the first pass
    int64_t n_tiles = 0;      // Gram tiles
    int64_t norm_entries = 0; // doubles reserved for the combines' squared norms
    int     n_layers = 0;
    size_t  off_slots = 0;    // n_slots x slot_elems floats
    size_t  off_partials = 0; // doubles [group][entry][tile], sized for the widest pass
    size_t  off_normparts = 0;// doubles [node][combine tile]: squared norm of every node a combine wrote
    size_t  off_normcoarse = 0;// doubles [node][Gram tile]: the same, summed per Gram tile
    size_t  off_gram = 0;     // doubles [group][layer][R*R] (finished Gram matrices)
    size_t  off_weights = 0;  // doubles [group][layer][R]
    size_t  off_leafnorm = 0; // doubles [layer]: sum over workers of the input squared norms
    size_t  total = 0;
};
// `norm_entries`: doubles needed for the squared norms the combines leave
// (max over passes of nodes written x combine tiles of that pass).
Layout make_layout(int K, int64_t N, int n_layers, int64_t n_tiles, int64_t norm_entries,
                   const std::vector<int>& radices, int order = ADASUM_ORDER_TREE);
// Number of tiles build_tiles would produce.
int64_t count_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity);
// Upper bound (over input dtypes) of make_layout's norm_entries for a schedule.
int64_t norm_entries_bound(int K, const int64_t* layer_offsets, int n_layers, const std::vector<int>& radices);

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
};

// All launchers return a hipError_t as int (0 = success) and enqueue on `stream`.
// partials[(group * entries + entry) * gt.n_tiles + tile]
// delta_start (or null): operands are x_r - delta_start, same storage type as the operands; diag only.
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
                       const double* partials, const double* normparts, double* gram, void* stream);
// Gram matrices -> per-layer weights of the binary (or linear) tree over R leaves.
int launch_weights(const double* gram, int R, int64_t n_items, int order,
                   double* weights, void* stream);
// `ct` must be the table of capacity combine_tile_capacity(dtype, R);
// normparts[group * ct.n_tiles + tile] (or null).
int launch_combine(int dtype, int out_dtype, const Operands& ops, const Outputs& out,
                   const TileSet& ct, int n_layers, int n_groups, int R,
                   const double* weights /* or null: unit weights */, double* normparts,
                   const void* sub_in /* type of the operands, or null */,
                   const void* add_out /* type of the output, or null */, void* stream);
// layer_sum[l * out_stride] = sum over `n_rows` rows and the tiles of layer l of parts[row][tile].
int launch_layer_sums(const double* parts, int n_rows, const TileSet& t, int n_layers,
                      double* layer_sum, int out_stride, void* stream);
// out[l * out_stride] = sum over groups of trace(gram[group][l]).
int launch_trace_sums(const double* gram, int R, int n_groups, int n_layers,
                      double* out, int out_stride, void* stream);

const char* kernel_name(const char* kind, int dtype, int out_dtype, int R, bool diag, char* buf, size_t n);

}  // namespace adasum
