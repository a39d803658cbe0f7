// Internal host-side declarations shared by the planner, the kernel launchers
// and the C-ABI layer of libadasum.  Nothing here is exported.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "adasum.h"

namespace adasum {

// Elements one workgroup covers at most.  A multiple of every granule
// (4 fp32 or 8 bf16 elements per 16-byte access) times the workgroup size.
#ifndef ADASUM_TILE
#define ADASUM_TILE 16384
#endif
#ifndef ADASUM_THREADS
#define ADASUM_THREADS 256
#endif
constexpr int kTile = ADASUM_TILE;
constexpr int kThreads = ADASUM_THREADS;
// Largest number of explicit operand pointers one launch carries by value.
constexpr int kMaxPack = 128;
constexpr int kMaxRadix = 8;
// Radix used when the caller asks for 0: the widest pass moves the fewest bytes.
constexpr int kDefaultRadix = 8;

inline int elem_bytes(int dtype) { return dtype == ADASUM_BF16 ? 2 : 4; }
inline bool is_pow2(long long v) { return v > 0 && (v & (v - 1)) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- planning (pure host code) ----------------------------------------------

// Validates a layer table; returns ADASUM_OK or an error code.
int check_layer_table(const int64_t* layer_offsets, int n_layers);

// Tile table: boundaries at layer boundaries and at global multiples of kTile.
// layer_tile_begin[l] .. layer_tile_begin[l+1] are the tiles of layer l.
void build_tiles(const int64_t* layer_offsets, int n_layers,
                 std::vector<adasum_tile>& tiles, std::vector<int32_t>& layer_tile_begin);

// Radix of every pass; product equals K.  Largest radices first (the first pass
// reads the narrow input dtype and touches the most data).
int build_levels(int K, int radix, std::vector<int>& radices);

// Number of Gram entries a pass of radix R accumulates per tile: all pairs
// i < j, plus the R diagonal entries when `diag` (the first pass; later passes
// get their squared norms from the previous combine).
inline int gram_entries(int R, bool diag) { return R * (R - 1) / 2 + (diag ? R : 0); }

// Device workspace layout (byte offsets from a 256-byte aligned base).
struct Layout {
    int64_t N = 0;            // elements per gradient
    int64_t slot_elems = 0;   // N rounded up so that fp32 slots stay 256-byte aligned
    int64_t n_slots = 0;      // fp32 intermediate tree nodes after the first pass
    int64_t n_tiles = 0;
    int     n_layers = 0;
    size_t  off_slots = 0;    // n_slots x slot_elems floats
    size_t  off_partials = 0; // doubles [group][entry][tile], sized for the widest pass
    size_t  off_normparts = 0;// doubles [node][tile][part]: squared norm of every node a combine wrote
    size_t  off_gram = 0;     // doubles [group][layer][R*R] (finished Gram matrices)
    size_t  off_weights = 0;  // doubles [group][layer][R]
    size_t  off_leafnorm = 0; // doubles [layer]: sum over workers of the input squared norms
    size_t  total = 0;
};
Layout make_layout(int K, int64_t N, int n_layers, int64_t n_tiles, const std::vector<int>& radices);

// ---- kernel launchers (adasum_kernels.hip) -----------------------------------

// How a kernel finds operand r of group g: either an explicit pointer
// (index g*R + r into `pack`), or slot (g*R + r)*stride of a strided fp32 arena.
struct Operands {
    const void* pack[kMaxPack];
    const char* base;
    long long   slot_bytes;
    int         stride;
    int         use_pack;
};

// Same idea for where a combine writes group g's result.
struct Outputs {
    char*     base;        // explicit single output when n_groups == 1 and stride == 0
    long long slot_bytes;
    int       stride;      // group g writes slot g*stride
};

struct LevelArgs {
    const adasum_tile* tiles;          // device
    const int32_t* layer_tile_begin;   // device, n_layers + 1
    int64_t n_tiles;
    int     n_layers;
    int     n_groups;
    int     R;
};

// All launchers return a hipError_t as int (0 = success) and enqueue on `stream`.
int launch_gram(int dtype, bool diag, const Operands& ops, const LevelArgs& a,
                double* partials, void* stream);
// Sums the per-tile partials (and, when !diag, the carried squared norms of the
// operand nodes) into full R x R Gram matrices gram[group][layer][R*R].
int launch_gram_finish(bool diag, const LevelArgs& a, const double* partials,
                       const double* normparts, int norm_sub, double* gram, void* stream);
// Workgroups ("parts") a combine of these dtypes spends on one tile; the squared
// norms it leaves are indexed [node][tile * parts + part].
int combine_parts_per_tile(int dtype, int out_dtype);
constexpr int kMaxCombineParts = 16;
// Gram matrices -> per-layer weights of the binary (or linear) tree over R leaves.
int launch_weights(const double* gram, int R, int64_t n_items, int order,
                   double* weights, void* stream);
int launch_combine(int dtype, int out_dtype, const Operands& ops, const Outputs& out,
                   const LevelArgs& a, const double* weights /* or null: unit weights */,
                   double* normparts /* [group][tile] or null */, void* stream);
// layer_sum[l] = sum over `n_rows` rows and the tiles of layer l of parts[row][tile * sub + part].
int launch_layer_sums(const double* parts, int n_rows, int sub, const LevelArgs& a,
                      double* layer_sum, int out_stride, void* stream);
// leafnorm[l] = sum over groups of trace(gram[group][l]).
int launch_trace_sums(const double* gram, int R, int n_groups, int n_layers,
                      double* out, int out_stride, void* stream);

const char* kernel_name(const char* kind, int dtype, int out_dtype, int R, bool diag, char* buf, size_t n);

}  // namespace adasum
