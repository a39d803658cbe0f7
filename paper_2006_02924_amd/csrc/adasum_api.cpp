// C-ABI layer of libadasum: argument validation, plan cache, the level
// scheduler that walks the binary tree of Section 3.4 (arXiv 2006.02924) one
// pass per group of `radix` siblings, and per-kernel event timing.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "adasum_host.h"

namespace adasum {
namespace {

thread_local int g_last_hip_error = 0;

#define ADASUM_HIP(call)                                        \
    do {                                                        \
        hipError_t e_ = (call);                                 \
        if (e_ != hipSuccess) {                                 \
            g_last_hip_error = static_cast<int>(e_);            \
            return e_ == hipErrorOutOfMemory ? ADASUM_ERR_OUT_OF_MEMORY : ADASUM_ERR_HIP; \
        }                                                       \
    } while (0)

#define ADASUM_LAUNCH(expr)                                     \
    do {                                                        \
        int e_ = (expr);                                        \
        if (e_ != 0) {                                          \
            g_last_hip_error = e_;                              \
            return ADASUM_ERR_HIP;                              \
        }                                                       \
    } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

struct Opts {
    int dtype;       // storage type of the inputs
    int out_dtype;
    int radix;
    int order;
    int use_graph;
    int fuse;        // radix 2: sibling pairs combined together, one level ahead
    int separate;    // every pass makes its own reduce pass (no pass feeds the next)
    void* workspace;
    size_t workspace_bytes;
    double* layer_stats;
    const void* delta_start;
};

// adasum_options as it was before delta_start, and before separate_passes, were appended: still accepted.
constexpr uint32_t kOptionsBytesV1 = offsetof(adasum_options, delta_start);
constexpr uint32_t kOptionsBytesV2 = offsetof(adasum_options, separate_passes);

int read_opts(const adasum_options* o, int dtype, Opts& r) {
    r.dtype = dtype;
    r.out_dtype = dtype;
    r.radix = 0;
    r.order = ADASUM_ORDER_TREE;
    r.use_graph = 0;
    r.fuse = 0;
    r.separate = 0;
    r.workspace = nullptr;
    r.workspace_bytes = 0;
    r.layer_stats = nullptr;
    r.delta_start = nullptr;
    if (o != nullptr) {
        if (o->struct_bytes < kOptionsBytesV1) return ADASUM_ERR_INVALID_ARG;
        if (o->struct_bytes >= kOptionsBytesV2) r.delta_start = o->delta_start;
        if (o->struct_bytes >= sizeof(adasum_options)) {
            if (o->reserved1 != 0) return ADASUM_ERR_INVALID_ARG;
            r.separate = o->separate_passes != 0;
        }
        if (o->out_dtype >= 0) r.out_dtype = o->out_dtype;
        r.radix = o->radix;
        r.order = o->order;
        r.use_graph = o->use_graph;
        r.fuse = o->fuse_siblings != 0;
        r.workspace = o->workspace;
        r.workspace_bytes = o->workspace_bytes;
        r.layer_stats = o->layer_stats;
    }
    if (!dtype_pair_ok(dtype, r.out_dtype)) return ADASUM_ERR_UNSUPPORTED;
    if (r.radix != 0 && r.radix != 2 && r.radix != 4 && r.radix != 8 && r.radix != 16 && r.radix != 32 && r.radix != 64)
        return ADASUM_ERR_UNSUPPORTED;
    if (r.radix > max_radix(dtype)) return ADASUM_ERR_UNSUPPORTED;
    if (r.order != ADASUM_ORDER_TREE && r.order != ADASUM_ORDER_LINEAR) return ADASUM_ERR_UNSUPPORTED;
    // the wide first pass: tree order over 16-bit leaves as they are
    if (wide_radix(r.radix) && (r.order != ADASUM_ORDER_TREE || r.delta_start != nullptr)) return ADASUM_ERR_UNSUPPORTED;
    if (r.fuse && (r.radix != 2 || r.order != ADASUM_ORDER_TREE || r.delta_start != nullptr))
        return ADASUM_ERR_UNSUPPORTED;
    if (r.delta_start != nullptr) {
        if (r.order != ADASUM_ORDER_TREE || r.out_dtype != dtype) return ADASUM_ERR_UNSUPPORTED;
        if (!aligned16(r.delta_start)) return ADASUM_ERR_MISALIGNED;
    }
    if (r.workspace != nullptr && (reinterpret_cast<uintptr_t>(r.workspace) & 255u) != 0)
        return ADASUM_ERR_WORKSPACE;
    if (r.layer_stats != nullptr && (reinterpret_cast<uintptr_t>(r.layer_stats) & 7u) != 0)
        return ADASUM_ERR_MISALIGNED;
    return ADASUM_OK;
}

// The delta form's Gram pass subtracts before it multiplies and so cannot use the packed
// dot instructions; with 16 operands it runs out of registers, 8 is its fastest radix.
// fp64 accumulators are twice as wide: 8 as well.
int default_radix(const Opts& o) {
    return (o.delta_start != nullptr || o.dtype == ADASUM_F64) ? 8 : kDefaultRadix;
}

// ---- plans -------------------------------------------------------------------

// One tile table on the host and on the device.
struct TileTable {
    int capacity = 0;
    std::vector<adasum_tile> tiles;
    std::vector<int32_t> layer_begin;
    std::vector<int32_t> first_in_gram;   // combine tables only
    std::vector<int32_t> part_begin;      // span tables (wide first pass) only
    adasum_tile* d_tiles = nullptr;
    int32_t* d_layer_begin = nullptr;
    int32_t* d_first_in_gram = nullptr;
    int32_t* d_part_begin = nullptr;
    int n_parts = 0;
    // >= 0: the device tables are borrowed (built on the device inside someone else's memory,
    // no host copy, never freed here) and hold this many tiles
    int64_t n_borrowed = -1;

    TileSet view() const {
        TileSet t;
        t.tiles = d_tiles;
        t.layer_begin = d_layer_begin;
        t.first_in_gram = d_first_in_gram;
        t.n_tiles = n_borrowed >= 0 ? n_borrowed : static_cast<int64_t>(tiles.size());
        t.capacity = capacity;
        t.part_begin = d_part_begin;
        t.n_parts = n_parts;
        return t;
    }
    // Both tables are sorted by start and a combine tile never straddles a Gram tile.
    void index_against(const std::vector<adasum_tile>& gram_tiles) {
        first_in_gram.assign(gram_tiles.size() + 1, 0);
        size_t c = 0;
        for (size_t t = 0; t < gram_tiles.size(); ++t) {
            while (c < tiles.size() && tiles[c].start < gram_tiles[t].start) ++c;
            first_in_gram[t] = static_cast<int32_t>(c);
        }
        first_in_gram[gram_tiles.size()] = static_cast<int32_t>(tiles.size());
    }
    int upload() {
        if (!tiles.empty()) {
            ADASUM_HIP(hipMalloc(reinterpret_cast<void**>(&d_tiles), tiles.size() * sizeof(adasum_tile)));
            ADASUM_HIP(hipMemcpy(d_tiles, tiles.data(), tiles.size() * sizeof(adasum_tile), hipMemcpyHostToDevice));
        }
        ADASUM_HIP(hipMalloc(reinterpret_cast<void**>(&d_layer_begin), layer_begin.size() * sizeof(int32_t)));
        ADASUM_HIP(hipMemcpy(d_layer_begin, layer_begin.data(), layer_begin.size() * sizeof(int32_t),
                             hipMemcpyHostToDevice));
        if (!first_in_gram.empty()) {
            ADASUM_HIP(hipMalloc(reinterpret_cast<void**>(&d_first_in_gram), first_in_gram.size() * sizeof(int32_t)));
            ADASUM_HIP(hipMemcpy(d_first_in_gram, first_in_gram.data(), first_in_gram.size() * sizeof(int32_t),
                                 hipMemcpyHostToDevice));
        }
        if (!part_begin.empty()) {
            ADASUM_HIP(hipMalloc(reinterpret_cast<void**>(&d_part_begin), part_begin.size() * sizeof(int32_t)));
            ADASUM_HIP(hipMemcpy(d_part_begin, part_begin.data(), part_begin.size() * sizeof(int32_t),
                                 hipMemcpyHostToDevice));
        }
        return ADASUM_OK;
    }
    void release() {
        if (n_borrowed >= 0) return;
        if (d_tiles) (void)hipFree(d_tiles);
        if (d_layer_begin) (void)hipFree(d_layer_begin);
        if (d_first_in_gram) (void)hipFree(d_first_in_gram);
        if (d_part_begin) (void)hipFree(d_part_begin);
        d_part_begin = nullptr;
        d_tiles = nullptr;
        d_layer_begin = nullptr;
        d_first_in_gram = nullptr;
    }
};

struct Plan {
    int device = 0;
    int K = 0;
    int radix = 0;
    int order = ADASUM_ORDER_TREE;
    int node_type = ADASUM_F32;           // storage type of the intermediate nodes
    // cache key of library-owned plans beyond the shape: calls that differ in any of these get
    // plans (and workspaces) of their own
    int in_dtype = -1, out_dtype = -1, delta = 0;
    int fuse = 0;                         // laid out for the sibling-fused radix-2 schedule
    int separate = 0;                     // cache key: made with separate_passes
    int feed = 0;                         // passes leave the next pass's Gram entries where they can
                                          // (pass_feeds_next): tree order, no delta form, no fuse
    std::vector<int64_t> offsets;
    TileTable gram_tiles;                 // capacity kTile
    TileTable wide_spans;                 // the span table of a wide first pass (else empty)
    std::map<int, TileTable> comb_tables; // by capacity, built on first use
    std::vector<int> radices;
    std::vector<SmallLayer> small;        // layers reduced by the definition in fp64 (see kSmallLayer)
    int n_small = 0;                      // entries of d_small
    SmallLayer* d_small = nullptr;
    Layout lay;
    char* d_ws = nullptr;   // library-owned workspace (lazily allocated)
    bool borrowed = false;  // every device pointer lives in memory this plan does not own

    // Calls on one plan share its workspace.  Each eager call leaves `done` on its stream; a call
    // that arrives on another stream first waits for it, so calls from several streams are
    // serialised on the device instead of racing.  `mu` serialises the host side.
    std::mutex mu;
    hipEvent_t done = nullptr;
    hipStream_t last_stream = nullptr;
    bool has_last = false;

    // Captured level ladders, one per distinct set of buffers (see launch_as_graph).
    struct GraphEntry {
        std::vector<uintptr_t> key;
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
    };
    std::vector<GraphEntry> graphs;
    hipStream_t capture_stream = nullptr;

    // The combine tile table for this input dtype and radix (device copy made on first use).
    int comb_tiles(int dtype, int R, TileSet* out) { return comb_tiles_of(combine_tile_capacity(dtype, R), out); }
    // ... and the one of a given capacity
    int comb_tiles_of(int cap, TileSet* out) {
        auto it = comb_tables.find(cap);
        if (it == comb_tables.end()) {
            if (borrowed) return ADASUM_ERR_INVALID_ARG;   // such a plan comes with all its tables
            try {
                TileTable t;
                t.capacity = cap;
                build_tiles(offsets.data(), static_cast<int>(offsets.size()) - 1, cap, t.tiles, t.layer_begin);
                t.index_against(gram_tiles.tiles);
                it = comb_tables.emplace(cap, std::move(t)).first;
            } catch (const std::bad_alloc&) {
                return ADASUM_ERR_OUT_OF_MEMORY;
            }
            int rc = it->second.upload();
            if (rc != ADASUM_OK) {
                it->second.release();
                comb_tables.erase(it);
                return rc;
            }
        }
        *out = it->second.view();
        return ADASUM_OK;
    }

    ~Plan() {
        for (auto& g : graphs) {
            if (g.exec) (void)hipGraphExecDestroy(g.exec);
            if (g.graph) (void)hipGraphDestroy(g.graph);
        }
        if (capture_stream) (void)hipStreamDestroy(capture_stream);
        if (done) (void)hipEventDestroy(done);
        gram_tiles.release();
        wide_spans.release();
        for (auto& kv : comb_tables) kv.second.release();
        if (borrowed) return;
        if (d_small) (void)hipFree(d_small);
        if (d_ws) (void)hipFree(d_ws);
    }
};

std::mutex g_mutex;
std::vector<std::unique_ptr<Plan>> g_plans;   // least recently used first
constexpr size_t kMaxPlans = 64;

// Builds a plan (host tables, their device copies; no workspace yet) on the current device.
// Capacity of the combine tile table pass lv uses, reading operands of type `dtype`: a pass that feeds
// the next one works with one wave per group whatever its radix.
int table_capacity(bool feed, const std::vector<int>& radices, size_t lv, int dtype) {
    return feed && pass_feeds_next(radices, lv) ? feed_tile_capacity(dtype, radices[lv])
                                                : combine_tile_capacity(dtype, radices[lv]);
}

// `no_feed`: the delta form, the step plans and separate_passes: no pass feeds the next.
int make_plan(int K, int radix, int order, int node_type, bool fuse, bool no_feed, const int64_t* offsets, int n_layers,
              std::unique_ptr<Plan>& out) {
    int device = 0;
    ADASUM_HIP(hipGetDevice(&device));
    std::unique_ptr<Plan> p(new (std::nothrow) Plan());
    if (!p) return ADASUM_ERR_OUT_OF_MEMORY;
    try {
        p->device = device;
        p->K = K;
        p->radix = radix;
        p->order = order;
        p->node_type = node_type;
        p->fuse = fuse ? 1 : 0;
        p->feed = (order == ADASUM_ORDER_TREE && !fuse && !no_feed) ? 1 : 0;
        p->offsets.assign(offsets, offsets + n_layers + 1);
        p->gram_tiles.capacity = gram_tile_capacity(offsets, n_layers);
        build_tiles(offsets, n_layers, p->gram_tiles.capacity, p->gram_tiles.tiles, p->gram_tiles.layer_begin);
        int rc = order == ADASUM_ORDER_LINEAR ? build_linear_passes(K, radix, p->radices)
                                              : build_levels(K, radix, p->radices);
        if (rc != ADASUM_OK) return rc;
        // the tree order lays its nodes out for the padded (power of two) leaf count
        const int Kv = order == ADASUM_ORDER_LINEAR ? K : virtual_leaves(p->radices);
        const int64_t small_elems = K > 1 ? find_small_layers(offsets, n_layers, p->small) : 0;
        if (!p->radices.empty() && wide_radix(p->radices[0])) {
            p->wide_spans.n_parts = wide_part_count(offsets[n_layers]);
            build_spans(offsets, n_layers, p->wide_spans.n_parts, p->wide_spans.tiles, p->wide_spans.part_begin,
                        p->wide_spans.layer_begin);
        }
        p->lay = make_layout(Kv, offsets[n_layers], n_layers, static_cast<int64_t>(p->gram_tiles.tiles.size()),
                             norm_entries_bound(Kv, offsets, n_layers, p->radices, node_type), p->radices, order,
                             K + 1, small_elems, node_type,
                             fuse      ? dot_entries_bound(Kv, offsets, n_layers, p->radices, node_type)
                             : p->feed ? next_entries_bound(Kv, offsets, n_layers, p->radices, node_type)
                                       : 0,
                             static_cast<int64_t>(p->wide_spans.tiles.size()));
    } catch (const std::bad_alloc&) {
        return ADASUM_ERR_OUT_OF_MEMORY;
    }
    int rc = p->gram_tiles.upload();
    if (rc != ADASUM_OK) return rc;
    if (p->wide_spans.n_parts > 0) {
        rc = p->wide_spans.upload();
        if (rc != ADASUM_OK) return rc;
    }
    if (!p->small.empty()) {
        const size_t bytes = p->small.size() * sizeof(SmallLayer);
        ADASUM_HIP(hipMalloc(reinterpret_cast<void**>(&p->d_small), bytes));
        ADASUM_HIP(hipMemcpy(p->d_small, p->small.data(), bytes, hipMemcpyHostToDevice));
    }
    p->n_small = static_cast<int>(p->small.size());
    ADASUM_HIP(hipEventCreateWithFlags(&p->done, hipEventDisableTiming));
    out = std::move(p);
    return ADASUM_OK;
}

// The library's own cache of plans, keyed by shape.
// `order` is a tree order or kStepPlans (the step entry points keep plans of their own).
constexpr int kStepPlans = 100;
int find_or_make_plan(int K, int radix, int order, int in_dtype, int out_dtype, bool delta, bool fuse, bool separate,
                      const int64_t* offsets, int n_layers, Plan** out) {
    const int node_type = node_dtype(in_dtype);
    int device = 0;
    ADASUM_HIP(hipGetDevice(&device));
    for (size_t i = 0; i < g_plans.size(); ++i) {
        Plan* p = g_plans[i].get();
        if (p->device == device && p->K == K && p->radix == radix && p->order == order && p->node_type == node_type &&
            p->in_dtype == in_dtype && p->out_dtype == out_dtype && p->delta == (delta ? 1 : 0) &&
            p->fuse == (fuse ? 1 : 0) && p->separate == (separate ? 1 : 0) &&
            static_cast<int>(p->offsets.size()) == n_layers + 1 &&
            std::memcmp(p->offsets.data(), offsets, sizeof(int64_t) * (n_layers + 1)) == 0) {
            // most recently used last
            std::rotate(g_plans.begin() + i, g_plans.begin() + i + 1, g_plans.end());
            *out = p;
            return ADASUM_OK;
        }
    }
    // a bounded cache: the least recently used plan goes (hipFree waits for work in flight)
    while (g_plans.size() >= kMaxPlans) g_plans.erase(g_plans.begin());
    std::unique_ptr<Plan> p;
    const int rc = make_plan(K, radix, order == kStepPlans ? ADASUM_ORDER_TREE : order, node_type, fuse,
                             delta || separate || order == kStepPlans, offsets, n_layers, p);
    if (rc != ADASUM_OK) return rc;
    p->order = order;
    p->in_dtype = in_dtype;
    p->out_dtype = out_dtype;
    p->delta = delta ? 1 : 0;
    p->separate = separate ? 1 : 0;
    *out = p.get();
    g_plans.push_back(std::move(p));
    return ADASUM_OK;
}

int plan_workspace(Plan* p, const Opts& o, char** ws) {
    if (o.workspace != nullptr) {
        if (o.workspace_bytes < p->lay.total) return ADASUM_ERR_WORKSPACE;
        *ws = static_cast<char*>(o.workspace);
        return ADASUM_OK;
    }
    if (p->d_ws == nullptr && p->lay.total > 0) {
        ADASUM_HIP(hipMalloc(reinterpret_cast<void**>(&p->d_ws), p->lay.total));
    }
    *ws = p->d_ws;
    return ADASUM_OK;
}

// ---- per-kernel timing ---------------------------------------------------------

struct ProfRecord {
    std::string name;
    hipEvent_t start, stop;
    double bytes;
};
std::atomic<bool> g_profile{false};
std::mutex g_prof_mutex;   // guards g_records and g_event_pool
thread_local bool t_no_profile = false;   // set while adasum_reduce_noalloc enqueues: events are allocations
std::vector<ProfRecord> g_records;
std::vector<hipEvent_t> g_event_pool;

int take_event(hipEvent_t* e) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_event_pool.empty()) {
        *e = g_event_pool.back();
        g_event_pool.pop_back();
        return ADASUM_OK;
    }
    ADASUM_HIP(hipEventCreate(e));
    return ADASUM_OK;
}

// Brackets one launch with events when profiling is on.
struct Timed {
    bool active = false;
    ProfRecord rec;
    hipStream_t st;
    int begin(const char* name, double bytes, void* stream) {
        st = static_cast<hipStream_t>(stream);
        if (!g_profile || t_no_profile) return ADASUM_OK;
        int rc = take_event(&rec.start);
        if (rc != ADASUM_OK) return rc;
        rc = take_event(&rec.stop);
        if (rc != ADASUM_OK) {
            std::lock_guard<std::mutex> lock(g_prof_mutex);
            g_event_pool.push_back(rec.start);
            return rc;
        }
        rec.name = name;
        rec.bytes = bytes;
        const hipError_t e = hipEventRecord(rec.start, st);
        if (e != hipSuccess) {
            give_back();
            g_last_hip_error = static_cast<int>(e);
            return ADASUM_ERR_HIP;
        }
        active = true;
        return ADASUM_OK;
    }
    int end() {
        if (!active) return ADASUM_OK;
        active = false;
        const hipError_t e = hipEventRecord(rec.stop, st);
        if (e != hipSuccess) {
            give_back();
            g_last_hip_error = static_cast<int>(e);
            return ADASUM_ERR_HIP;
        }
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        g_records.push_back(rec);
        return ADASUM_OK;
    }
    // a launch that failed leaves no record: its events go back to the pool
    void give_back() {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        g_event_pool.push_back(rec.start);
        g_event_pool.push_back(rec.stop);
    }
    ~Timed() {
        if (active) give_back();
    }
};

#define ADASUM_TIMED(name, bytes, stream, launch_expr)          \
    do {                                                        \
        Timed t_;                                               \
        int rc_ = t_.begin(name, bytes, stream);                \
        if (rc_ != ADASUM_OK) return rc_;                       \
        ADASUM_LAUNCH(launch_expr);                             \
        rc_ = t_.end();                                         \
        if (rc_ != ADASUM_OK) return rc_;                       \
    } while (0)

// ---- common validation ---------------------------------------------------------

int check_operands(const void* const* ptrs, int count, int64_t N, int dtype) {
    if (ptrs == nullptr) return ADASUM_ERR_INVALID_ARG;
    for (int k = 0; k < count; ++k) {
        if (ptrs[k] == nullptr && N > 0) return ADASUM_ERR_INVALID_ARG;
        if (!aligned16(ptrs[k])) return ADASUM_ERR_MISALIGNED;
    }
    (void)dtype;
    return ADASUM_OK;
}

// ---- small layers, by the definition --------------------------------------------

// Before anything is written: the small layers of every worker (minus delta_start) and of
// delta_start itself go into the compact fp64 copy, kMaxPack workers per launch.
int small_gather(Plan* p, char* ws, const void* const* grads, int dtype, const Opts& o, void* stream) {
    if (p->n_small == 0) return ADASUM_OK;
    double* compact = reinterpret_cast<double*>(ws + p->lay.off_small);
    const int n_small = p->n_small;
    for (int k0 = 0; k0 < p->K; k0 += kMaxPack) {
        const int n = std::min(kMaxPack, p->K - k0);
        Operands ops;
        std::memset(&ops, 0, sizeof(ops));
        for (int j = 0; j < n; ++j) ops.pack[j] = grads[k0 + j];
        ADASUM_TIMED("small_gather", 0.0, stream,
                     launch_small_gather(dtype, ops, n, k0, p->d_small, n_small, p->lay.small_elems, o.delta_start,
                                         k0 == 0 && o.delta_start != nullptr, p->K, compact, stream));
    }
    return ADASUM_OK;
}

// After the passes: the small layers again, pair by pair in fp64, over what they wrote.
int small_reduce(Plan* p, char* ws, void* out, const Opts& o, void* stream) {
    if (p->n_small == 0) return ADASUM_OK;
    const double* compact = reinterpret_cast<const double*>(ws + p->lay.off_small);
    ADASUM_TIMED("small_layers", 0.0, stream,
                 launch_small_reduce(o.out_dtype, compact, p->K, p->d_small, p->n_small,
                                     p->lay.small_elems, o.order, o.delta_start != nullptr, p->K, out,
                                     o.layer_stats, stream));
    return ADASUM_OK;
}

// ---- the level scheduler -------------------------------------------------------

int run_tree(Plan* p, char* ws, const void* const* grads, int dtype, void* out, const Opts& o, void* stream) {
    const Layout& lay = p->lay;
    const int L = lay.n_layers;
    const int64_t N = lay.N;
    const TileSet gt = p->gram_tiles.view();
    char* slots = ws + lay.off_slots;
    double* partials = reinterpret_cast<double*>(ws + lay.off_partials);
    double* normparts = reinterpret_cast<double*>(ws + lay.off_normparts);
    double* normcoarse = reinterpret_cast<double*>(ws + lay.off_normcoarse);
    double* gram = reinterpret_cast<double*>(ws + lay.off_gram);
    double* weights = reinterpret_cast<double*>(ws + lay.off_weights);
    double* dotparts = reinterpret_cast<double*>(ws + lay.off_dotparts);
    const long long slot_bytes = static_cast<long long>(lay.slot_elems) * lay.node_bytes;
    char namebuf[48];
    // sibling-fused radix 2 (fuse_siblings): the combine of every level but the last also leaves the
    // dot products the next level needs
    const bool fuse = o.fuse != 0 && p->fuse != 0;
    bool dots_ready = false;   // the previous combine left this level's dot products
    // passes that feed the next one: the combine leaves the next pass's whole Gram matrix per tile
    const bool feed = p->feed != 0 && !fuse && o.delta_start == nullptr;
    double* nextparts = dotparts;   // (the two schemes exclude each other and share the section)
    bool fed = false;          // the previous combine left this level's Gram entries

    int nodes = virtual_leaves(p->radices);   // tree nodes alive before this pass (leaves: padded count)
    const int depth0 = first_depth(p->radices);   // the first pass's groups are the sub-trees of this depth
    int stride = 1;          // slot distance between consecutive alive nodes (passes >= 1)
    TileSet norm_tiles;      // the table the previous combine indexed its squared norms by
    const int n_levels = static_cast<int>(p->radices.size());
    // Resolve (and on first use build and upload) every tile table before the first launch:
    // nothing below may allocate, so the ladder can be captured into a graph.
    std::vector<TileSet> comb_sets(n_levels);
    for (int lv = 0; lv < n_levels; ++lv) {
        const int rc = p->comb_tiles_of(table_capacity(feed, p->radices, lv, lv == 0 ? dtype : node_dtype(dtype)),
                                        &comb_sets[lv]);
        if (rc != ADASUM_OK) return rc;
    }
    {
        const int rc = small_gather(p, ws, grads, dtype, o, stream);
        if (rc != ADASUM_OK) return rc;
    }
    for (int lv = 0; lv < n_levels; ++lv) {
        const int R = p->radices[lv];
        const int groups = nodes / R;
        const bool first = lv == 0, last = lv == n_levels - 1;
        const int in_dtype = first ? dtype : node_dtype(dtype);
        const int st_dtype = last ? o.out_dtype : node_dtype(dtype);
        // a wide pass walks the span table and leaves whole blocks per span; every other pass the Gram tiles
        const bool wide = wide_radix(R);
        const TileSet rt = wide ? p->wide_spans.view() : gt;
        const int np = wide ? gram_partial_entries(R) : gram_entries(R, first);
        const bool want_norm = !last || o.layer_stats != nullptr;
        const TileSet ct = comb_sets[lv];

        // groups per launch: the operand pointers travel by value in the kernel arguments
        const int batch = std::max(1, kMaxPack / R);
        // Section 4.1's delta form: the leaves are grads[k] - delta_start, the root adds delta_start back
        const void* sub_in = first ? o.delta_start : nullptr;
        const void* add_out = last ? o.delta_start : nullptr;
        // algorithmic bytes of a launch over `ng` groups with `leaves` distinct operands
        auto gram_bytes = [&](int leaves, int ng) {
            return static_cast<double>(leaves + (sub_in ? ng : 0)) * N * elem_bytes(in_dtype);
        };
        auto comb_bytes = [&](int leaves, int ng) {
            return static_cast<double>(N) * (static_cast<double>(leaves + (sub_in ? ng : 0)) * elem_bytes(in_dtype) +
                                             (add_out ? 2.0 : 1.0) * ng * elem_bytes(st_dtype));
        };

        // first pass: group g reads its sub-tree's leaves; a group with fewer than R leaves
        // (K not a power of two) repeats its first leaf, which the weights kernel zeroes
        auto fill_operands = [&](Operands& ops, int g0, int ng) {
            std::memset(&ops, 0, sizeof(ops));
            if (first) {
                for (int j = 0; j < ng; ++j) {
                    int lo, hi;
                    leaf_range(p->K, depth0, g0 + j, lo, hi);
                    for (int i = 0; i < R; ++i) ops.pack[j * R + i] = grads[lo + i < hi ? lo + i : lo];
                }
            } else {
                for (int i = 0; i < ng * R; ++i)
                    ops.pack[i] = slots + static_cast<long long>(g0 * R + i) * stride * slot_bytes;
            }
        };
        auto real_leaves = [&](int g0, int ng) {
            if (!first) return ng * R;
            int lo, hi, lo2, hi2;
            leaf_range(p->K, depth0, g0, lo, hi);
            leaf_range(p->K, depth0, g0 + ng - 1, lo2, hi2);
            return hi2 - lo;
        };

        // step 1: partial Gram entries -- from a pass over the operands, or (sibling-fused) already
        // left per combine tile by the combine that wrote them: one entry per pair, summed per Gram tile
        const bool feeds = feed && pass_feeds_next(p->radices, static_cast<size_t>(lv));
        if (fed) {
            // whole Gram matrices per combine tile, left by the combine below us: sum them per Gram tile
            ADASUM_TIMED("gram_from_combine", 0.0, stream,
                         launch_parts_coarsen(nextparts, groups, gram_entries(R, true), norm_tiles, gt, partials,
                                              stream));
        } else if (dots_ready) {
            ADASUM_TIMED("dot_coarsen", 0.0, stream,
                         launch_norm_coarsen(dotparts, groups, norm_tiles, gt, partials, stream));
        } else {
            for (int g0 = 0; g0 < groups; g0 += batch) {
                const int ng = std::min(batch, groups - g0);
                Operands ops;
                fill_operands(ops, g0, ng);
                kernel_name("gram", in_dtype, 0, R, first, namebuf, sizeof(namebuf));
                ADASUM_TIMED(namebuf, gram_bytes(real_leaves(g0, ng), ng), stream,
                             launch_gram(in_dtype, first, ops, rt, ng, R,
                                         partials + static_cast<int64_t>(g0) * np * rt.n_tiles, sub_in, stream));
            }
        }
        const bool fuse_here = fuse && R == 2 && !last && groups % 2 == 0;
        // step 2: finish the sums, then the tree's scalars
        if (!first && !fed) {
            ADASUM_TIMED("norm_coarsen", 0.0, stream,
                         launch_norm_coarsen(normparts, nodes, norm_tiles, gt, normcoarse, stream));
        }
        // (the tree's weights come out of the same launch; a fed pass has its diagonal in the partials)
        kernel_name("gram_finish", 0, 0, R, first || fed, namebuf, sizeof(namebuf));
        ADASUM_TIMED(namebuf, 0.0, stream,
                     launch_gram_finish(first || fed, rt, L, groups, R, partials, normcoarse, gram, weights, o.order,
                                        first ? p->K : 0, depth0, stream));
        if (first && o.layer_stats != nullptr) {
            ADASUM_LAUNCH(launch_trace_sums(gram, R, groups, L, p->K, depth0, 0, false, o.layer_stats + 1, 2, stream));
        }
        // step 3: apply
        for (int g0 = 0; g0 < groups; g0 += batch) {
            const int ng = std::min(batch, groups - g0);
            Operands ops;
            fill_operands(ops, g0, ng);
            Outputs outs;
            if (last) {
                outs.base = static_cast<char*>(out);
                outs.slot_bytes = 0;
                outs.stride = 0;
            } else {
                const int ostride = first ? 1 : R * stride;
                outs.base = slots + static_cast<long long>(g0) * ostride * slot_bytes;
                outs.slot_bytes = slot_bytes;
                outs.stride = ostride;
            }
            if (feeds) {
                const int R2 = p->radices[lv + 1];
                char base[40];
                kernel_name("combine", in_dtype, st_dtype, R, false, base, sizeof(base));
                std::snprintf(namebuf, sizeof(namebuf), "%s+gram%d", base, R2);
                ADASUM_TIMED(namebuf, comb_bytes(real_leaves(g0, ng), ng), stream,
                             launch_combine_feed(in_dtype, st_dtype, ops, outs, ct, L, ng, R, R2,
                                                 weights + static_cast<int64_t>(g0) * L * R,
                                                 nextparts + static_cast<int64_t>(g0 / R2) * ct.n_tiles *
                                                                 gram_entries(R2, true),
                                                 stream));
                continue;
            }
            if (fuse_here) {
                char base[40];
                kernel_name("combine", in_dtype, st_dtype, R, false, base, sizeof(base));
                std::snprintf(namebuf, sizeof(namebuf), "%s+dot", base);
                ADASUM_TIMED(namebuf, comb_bytes(real_leaves(g0, ng), ng), stream,
                             launch_combine_siblings(in_dtype, st_dtype, ops, outs, ct, L, ng,
                                                     weights + static_cast<int64_t>(g0) * L * R,
                                                     normparts + static_cast<int64_t>(g0) * ct.n_tiles,
                                                     dotparts + static_cast<int64_t>(g0 / 2) * ct.n_tiles, stream));
                continue;
            }
            kernel_name("combine", in_dtype, st_dtype, R, false, namebuf, sizeof(namebuf));
            ADASUM_TIMED(namebuf, comb_bytes(real_leaves(g0, ng), ng), stream,
                         launch_combine(in_dtype, st_dtype, ops, outs, ct, L, ng, R,
                                        weights + static_cast<int64_t>(g0) * L * R,
                                        want_norm ? normparts + static_cast<int64_t>(g0) * ct.n_tiles : nullptr,
                                        sub_in, add_out, stream));
        }
        dots_ready = fuse_here;
        fed = feeds;
        stride = first ? 1 : R * stride;
        nodes = groups;
        norm_tiles = ct;
    }
    if (o.layer_stats != nullptr) {
        ADASUM_LAUNCH(launch_norm_coarsen(normparts, 1, norm_tiles, gt, normcoarse, stream));
        ADASUM_LAUNCH(launch_layer_sums(normcoarse, 1, gt, L, o.layer_stats, 2, stream));
    }
    return small_reduce(p, ws, out, o, stream);
}

// Left-to-right order (Section 3.4, first recursion).  Pass 0 folds the first
// leaves; every later pass folds the running result (a node: fp32 or fp64, slot 0,
// operand 0, updated in place) with the next leaves, which are read in their own
// storage type.
int run_linear(Plan* p, char* ws, const void* const* grads, int dtype, void* out, const Opts& o, void* stream) {
    const Layout& lay = p->lay;
    const int L = lay.n_layers;
    const TileSet gt = p->gram_tiles.view();
    char* slots = ws + lay.off_slots;
    double* partials = reinterpret_cast<double*>(ws + lay.off_partials);
    double* gram = reinterpret_cast<double*>(ws + lay.off_gram);
    double* weights = reinterpret_cast<double*>(ws + lay.off_weights);
    double* normparts = reinterpret_cast<double*>(ws + lay.off_normparts);
    double* normcoarse = reinterpret_cast<double*>(ws + lay.off_normcoarse);
    const int n_passes = static_cast<int>(p->radices.size());
    const bool mixed = dtype != node_dtype(dtype);   // 16-bit leaves next to an fp32 running result

    // every table first: nothing below may allocate
    std::vector<TileSet> comb_sets(n_passes);
    for (int b = 0; b < n_passes; ++b) {
        const int rc = p->comb_tiles(dtype, p->radices[b], &comb_sets[b]);
        if (rc != ADASUM_OK) return rc;
    }

    {
        const int rc = small_gather(p, ws, grads, dtype, o, stream);
        if (rc != ADASUM_OK) return rc;
    }
    int next_leaf = 0;
    for (int b = 0; b < n_passes; ++b) {
        const int R = p->radices[b];
        const bool first = b == 0, last = b == n_passes - 1;
        const int st_dtype = last ? o.out_dtype : node_dtype(dtype);
        Operands ops;
        std::memset(&ops, 0, sizeof(ops));
        if (first) {
            for (int r = 0; r < R; ++r) ops.pack[r] = grads[next_leaf + r];
            next_leaf += R;
        } else {
            ops.pack[0] = slots;
            for (int r = 1; r < R; ++r) ops.pack[r] = grads[next_leaf + r - 1];
            next_leaf += R - 1;
        }
        const bool head32 = mixed && !first;
        // algorithmic bytes: R operands read, operand 0 of a later pass as a node
        const double read_bytes = static_cast<double>(lay.N) *
                                  ((first ? R : R - 1) * elem_bytes(dtype) + (first ? 0 : lay.node_bytes));
        char namebuf[64], base[48];
        kernel_name("gram", dtype, 0, R, true, base, sizeof(base));
        std::snprintf(namebuf, sizeof(namebuf), "%s%s", base, head32 ? "+f32 head" : "");
        if (head32) {
            ADASUM_TIMED(namebuf, read_bytes, stream, launch_gram_head32(dtype, ops, gt, R, partials, stream));
        } else {
            ADASUM_TIMED(namebuf, read_bytes, stream,
                         launch_gram(dtype, true, ops, gt, 1, R, partials, nullptr, stream));
        }
        kernel_name("gram_finish", 0, 0, R, true, namebuf, sizeof(namebuf));
        ADASUM_TIMED(namebuf, 0.0, stream,
                     launch_gram_finish(true, gt, L, 1, R, partials, nullptr, gram, weights, ADASUM_ORDER_LINEAR, 0, 0,
                                        stream));
        // statistics: every leaf's squared norm is a diagonal entry of exactly one pass (entry 0 of a
        // later pass is the running result)
        if (o.layer_stats != nullptr) {
            ADASUM_LAUNCH(launch_trace_sums(gram, R, 1, L, 0, 0, first ? 0 : 1, !first, o.layer_stats + 1, 2, stream));
        }
        Outputs outs;
        outs.base = last ? static_cast<char*>(out) : slots;
        outs.slot_bytes = 0;
        outs.stride = 0;
        double* np = last && o.layer_stats != nullptr ? normparts : nullptr;
        const double comb_bytes = read_bytes + static_cast<double>(lay.N) * elem_bytes(st_dtype);
        kernel_name("combine", dtype, st_dtype, R, false, base, sizeof(base));
        std::snprintf(namebuf, sizeof(namebuf), "%s%s", base, head32 ? "+f32 head" : "");
        if (head32) {
            ADASUM_TIMED(namebuf, comb_bytes, stream,
                         launch_combine_head32(dtype, st_dtype, ops, outs, comb_sets[b], L, R, weights, np, stream));
        } else {
            ADASUM_TIMED(namebuf, comb_bytes, stream,
                         launch_combine(dtype, st_dtype, ops, outs, comb_sets[b], L, 1, R, weights, np, nullptr,
                                        nullptr, stream));
        }
    }
    if (o.layer_stats != nullptr && n_passes > 0) {
        ADASUM_LAUNCH(launch_norm_coarsen(normparts, 1, comb_sets[n_passes - 1], gt, normcoarse, stream));
        ADASUM_LAUNCH(launch_layer_sums(normcoarse, 1, gt, L, o.layer_stats, 2, stream));
    }
    return small_reduce(p, ws, out, o, stream);
}

// K = 1: the result is the gradient itself, converted to the output dtype.
int run_copy(Plan* p, char* ws, const void* const* grads, int dtype, void* out, const Opts& o, void* stream) {
    const Layout& lay = p->lay;
    double* normparts = reinterpret_cast<double*>(ws + lay.off_normparts);
    TileSet ct;
    {
        const int rc = p->comb_tiles(dtype, 1, &ct);
        if (rc != ADASUM_OK) return rc;
    }
    Operands ops;
    std::memset(&ops, 0, sizeof(ops));
    ops.pack[0] = grads[0];
    Outputs outs;
    outs.base = static_cast<char*>(out);
    outs.slot_bytes = 0;
    outs.stride = 0;
    char namebuf[48];
    kernel_name("combine", dtype, o.out_dtype, 1, false, namebuf, sizeof(namebuf));
    // with delta_start the copy goes through the same arithmetic as any root: (x - start) + start
    const double copy_bytes = static_cast<double>(lay.N) * ((o.delta_start ? 2.0 : 1.0) * elem_bytes(dtype) +
                                                            (o.delta_start ? 2.0 : 1.0) * elem_bytes(o.out_dtype));
    ADASUM_TIMED(namebuf, copy_bytes, stream,
                 launch_combine(dtype, o.out_dtype, ops, outs, ct, lay.n_layers, 1, 1, nullptr,
                                o.layer_stats ? normparts : nullptr, o.delta_start, o.delta_start, stream));
    if (o.layer_stats != nullptr) {
        double* normcoarse = reinterpret_cast<double*>(ws + lay.off_normcoarse);
        const TileSet gt = p->gram_tiles.view();
        ADASUM_LAUNCH(launch_norm_coarsen(normparts, 1, ct, gt, normcoarse, stream));
        ADASUM_LAUNCH(launch_layer_sums(normcoarse, 1, gt, lay.n_layers, o.layer_stats, 2, stream));
        ADASUM_LAUNCH(launch_layer_sums(normcoarse, 1, gt, lay.n_layers, o.layer_stats + 1, 2, stream));
    }
    return ADASUM_OK;
}

// Builds and uploads every combine tile table a reduction with this plan reads, so that the
// launch ladder itself allocates nothing.
int prebuild_tables(Plan* p, int dtype, int order) {
    if (p->K == 1) {
        TileSet ct;
        return p->comb_tiles(dtype, 1, &ct);
    }
    for (size_t lv = 0; lv < p->radices.size(); ++lv) {
        TileSet ct;
        // (the left-to-right order reads leaves, in their storage type, in every pass)
        const bool leaves = lv == 0 || order == ADASUM_ORDER_LINEAR;
        const int rc = p->comb_tiles_of(table_capacity(p->feed != 0, p->radices, lv, leaves ? dtype : node_dtype(dtype)), &ct);
        if (rc != ADASUM_OK) return rc;
    }
    return ADASUM_OK;
}

// Replays the whole ladder as one hipGraph launch.  The graph is captured once
// per distinct set of buffers (kernel arguments are baked into its nodes) on a
// private stream and cached in the plan; a call with other buffers captures
// another one (at most kMaxGraphsPerPlan are kept, oldest dropped).
constexpr size_t kMaxGraphsPerPlan = 8;

int launch_as_graph(Plan* p, char* ws, const void* const* grads, int dtype, void* out, const Opts& o,
                    void* stream) {
    std::vector<uintptr_t> key;
    key.reserve(static_cast<size_t>(p->K) + 6);
    for (int k = 0; k < p->K; ++k) key.push_back(reinterpret_cast<uintptr_t>(grads[k]));
    key.push_back(reinterpret_cast<uintptr_t>(out));
    key.push_back(reinterpret_cast<uintptr_t>(ws));
    key.push_back(reinterpret_cast<uintptr_t>(o.layer_stats));
    key.push_back(reinterpret_cast<uintptr_t>(o.delta_start));
    key.push_back(static_cast<uintptr_t>(dtype));
    key.push_back(static_cast<uintptr_t>(o.out_dtype));
    key.push_back(static_cast<uintptr_t>(o.order));
    for (auto& g : p->graphs) {
        if (g.key == key) {
            ADASUM_HIP(hipGraphLaunch(g.exec, static_cast<hipStream_t>(stream)));
            return ADASUM_OK;
        }
    }
    if (p->capture_stream == nullptr) {
        ADASUM_HIP(hipStreamCreateWithFlags(&p->capture_stream, hipStreamNonBlocking));
    }
    // everything that allocates happens before the capture starts
    {
        const int rc = prebuild_tables(p, dtype, o.order);
        if (rc != ADASUM_OK) return rc;
    }
    ADASUM_HIP(hipStreamBeginCapture(p->capture_stream, hipStreamCaptureModeThreadLocal));
    const int rc = p->K == 1 ? run_copy(p, ws, grads, dtype, out, o, p->capture_stream)
                   : o.order == ADASUM_ORDER_LINEAR
                       ? run_linear(p, ws, grads, dtype, out, o, p->capture_stream)
                       : run_tree(p, ws, grads, dtype, out, o, p->capture_stream);
    hipGraph_t graph = nullptr;
    const hipError_t end = hipStreamEndCapture(p->capture_stream, &graph);
    if (rc != ADASUM_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (end != hipSuccess) {
        g_last_hip_error = static_cast<int>(end);
        return ADASUM_ERR_HIP;
    }
    hipGraphExec_t exec = nullptr;
    const hipError_t inst = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (inst != hipSuccess) {
        (void)hipGraphDestroy(graph);
        g_last_hip_error = static_cast<int>(inst);
        return inst == hipErrorOutOfMemory ? ADASUM_ERR_OUT_OF_MEMORY : ADASUM_ERR_HIP;
    }
    if (p->graphs.size() >= kMaxGraphsPerPlan) {
        (void)hipGraphExecDestroy(p->graphs.front().exec);
        (void)hipGraphDestroy(p->graphs.front().graph);
        p->graphs.erase(p->graphs.begin());
    }
    Plan::GraphEntry e;
    e.key = std::move(key);
    e.graph = graph;
    e.exec = exec;
    p->graphs.push_back(std::move(e));
    ADASUM_HIP(hipGraphLaunch(exec, static_cast<hipStream_t>(stream)));
    return ADASUM_OK;
}

// Checks of one call's buffers against a problem shape (no device work).
int check_call(const void* const* grads, int K, int64_t N, int dtype, void* out, const Opts& o) {
    int rc = check_operands(grads, K, N, dtype);
    if (rc != ADASUM_OK) return rc;
    if (out == nullptr && N > 0) return ADASUM_ERR_INVALID_ARG;
    if (!aligned16(out)) return ADASUM_ERR_MISALIGNED;
    if (N == 0) return ADASUM_OK;
    const size_t in_bytes = static_cast<size_t>(N) * elem_bytes(dtype);
    const size_t out_bytes = static_cast<size_t>(N) * elem_bytes(o.out_dtype);
    for (int k = 0; k < K; ++k)
        if (overlaps(grads[k], in_bytes, out, out_bytes)) return ADASUM_ERR_ALIAS;
    // out may BE delta_start (every element is read by the lane that then writes it) but not straddle it
    if (o.delta_start != nullptr && o.delta_start != out && overlaps(o.delta_start, in_bytes, out, out_bytes))
        return ADASUM_ERR_ALIAS;
    return ADASUM_OK;
}

// Device-side ordering of the calls that share a plan's workspace.  begin: a call that arrives
// on another stream than the previous one first waits for that call's event.  end: leaves the
// event on this call's stream.  A stream that is being captured into a caller's graph gets
// neither (the caller orders what it captures).  The caller holds the plan's lock or g_mutex.
int begin_on_stream(Plan* p, void* stream, bool* eager) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    *eager = false;
    if (p->done == nullptr) return ADASUM_OK;
    // (the default stream cannot be captured; asking about it could even disturb a capture that
    // another thread has under way in the global mode)
    if (st != nullptr) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        ADASUM_HIP(hipStreamIsCapturing(st, &cs));
        if (cs != hipStreamCaptureStatusNone) return ADASUM_OK;
    }
    *eager = true;
    if (p->has_last && p->last_stream != st) ADASUM_HIP(hipStreamWaitEvent(st, p->done, 0));
    return ADASUM_OK;
}

int end_on_stream(Plan* p, void* stream, bool eager, int rc) {
    if (!eager) return rc;
    // also after a failed enqueue: the launches before the failure may be in flight
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = hipEventRecord(p->done, st);
    if (e == hipSuccess) {
        p->last_stream = st;
        p->has_last = true;
    } else if (rc == ADASUM_OK) {
        g_last_hip_error = static_cast<int>(e);
        rc = ADASUM_ERR_HIP;
    }
    return rc;
}

// Enqueues one reduction with a plan.  The caller holds the plan's lock or g_mutex.
int execute_plan(Plan* p, const void* const* grads, int dtype, void* out, const Opts& o, void* stream) {
    char* ws = nullptr;
    int rc = plan_workspace(p, o, &ws);
    if (rc != ADASUM_OK) return rc;
    bool eager = false;
    rc = begin_on_stream(p, stream, &eager);
    if (rc != ADASUM_OK) return rc;
    if (o.use_graph && !g_profile) rc = launch_as_graph(p, ws, grads, dtype, out, o, stream);
    else if (p->K == 1) rc = run_copy(p, ws, grads, dtype, out, o, stream);
    else if (o.order == ADASUM_ORDER_LINEAR) rc = run_linear(p, ws, grads, dtype, out, o, stream);
    else rc = run_tree(p, ws, grads, dtype, out, o, stream);
    return end_on_stream(p, stream, eager, rc);
}

// The argument checks every reduce entry point starts with (no device work).  N receives the
// number of elements per gradient.
int check_reduce_args(const void* const* grads, int K, const int64_t* layer_offsets, int n_layers, int dtype,
                      void* out, const adasum_options* opts, Opts& o, int64_t& N) {
    if (K < 1) return ADASUM_ERR_INVALID_ARG;
    int rc = check_layer_table(layer_offsets, n_layers);
    if (rc != ADASUM_OK) return rc;
    if (!known_dtype(dtype)) return ADASUM_ERR_UNSUPPORTED;
    rc = read_opts(opts, dtype, o);
    if (rc != ADASUM_OK) return rc;
    if (K > (1 << 20)) return ADASUM_ERR_UNSUPPORTED;
    N = layer_offsets[n_layers];
    return check_call(grads, K, N, dtype, out, o);
}

int reduce_impl(const void* const* grads, int K, const int64_t* layer_offsets, int n_layers, int dtype,
                void* out, const adasum_options* opts, void* stream) {
    Opts o;
    int64_t N = 0;
    int rc = check_reduce_args(grads, K, layer_offsets, n_layers, dtype, out, opts, o, N);
    if (rc != ADASUM_OK || N == 0) return rc;

    std::lock_guard<std::mutex> lock(g_mutex);
    Plan* p = nullptr;
    rc = find_or_make_plan(K, o.radix == 0 ? default_radix(o) : o.radix, o.order, dtype, o.out_dtype,
                           o.delta_start != nullptr, o.fuse != 0, o.separate != 0, layer_offsets, n_layers, &p);
    if (rc != ADASUM_OK) return rc;
    return execute_plan(p, grads, dtype, out, o, stream);
}

// ---- the same reduction without any allocation -----------------------------------

// Hands out consecutive pieces of a region, each at the next multiple of `align` bytes.
struct Carver {
    size_t off = 0;
    size_t take(size_t bytes, size_t align = 256) {
        off = align_up(off, align);
        const size_t at = off;
        off += bytes;
        return at;
    }
};

// adasum_reduce_ex with tile tables and workspace inside the library's static device array:
// the layer table goes to the device in kernel arguments, the tables are built there, and the
// scheduler then runs on a plan that only borrows that memory.
int reduce_noalloc_impl(const void* const* grads, int K, const int64_t* layer_offsets, int n_layers, int dtype,
                        void* out, const adasum_options* opts, void* stream) {
    Opts o;
    int64_t N = 0;
    int rc = check_reduce_args(grads, K, layer_offsets, n_layers, dtype, out, opts, o, N);
    if (rc != ADASUM_OK) return rc;
    if (o.workspace != nullptr || o.use_graph) return ADASUM_ERR_INVALID_ARG;
    if (N == 0) return ADASUM_OK;

    const int L = n_layers;
    const int node_type = node_dtype(dtype);
    Plan plan;   // host-side description only; its device pointers point into the static array
    plan.borrowed = true;
    plan.K = K;
    plan.radix = o.radix == 0 ? default_radix(o) : o.radix;
    plan.order = o.order;
    plan.node_type = node_type;
    struct CombTable {
        int cap;
        int64_t n;
        size_t off_tiles, off_begin, off_index;
    };
    std::vector<CombTable> combs;
    Carver carve;
    size_t off_offsets = 0, off_gram_tiles = 0, off_gram_begin = 0, off_small = 0, off_ws = 0;
    size_t off_span_tiles = 0, off_span_begin = 0, off_span_parts = 0;
    int gcap = 0;
    int64_t n_gram = 0;
    try {
        rc = o.order == ADASUM_ORDER_LINEAR ? build_linear_passes(K, plan.radix, plan.radices)
                                            : build_levels(K, plan.radix, plan.radices);
        if (rc != ADASUM_OK) return rc;
        const int Kv = o.order == ADASUM_ORDER_LINEAR ? K : virtual_leaves(plan.radices);
        int64_t small_elems = 0;
        if (K > 1) {
            for (int l = 0; l < L; ++l) {
                const int64_t len = layer_offsets[l + 1] - layer_offsets[l];
                if (len >= 1 && len <= kSmallLayer) {
                    ++plan.n_small;
                    small_elems += len;
                }
            }
        }
        gcap = gram_tile_capacity(layer_offsets, L);
        n_gram = count_tiles(layer_offsets, L, gcap);
        plan.fuse = o.fuse;
        plan.feed = (o.order == ADASUM_ORDER_TREE && !o.fuse && !o.separate && o.delta_start == nullptr) ? 1 : 0;
        // the span table of a wide first pass is small (a few hundred entries): built here, on the host
        if (!plan.radices.empty() && wide_radix(plan.radices[0])) {
            plan.wide_spans.n_parts = wide_part_count(N);
            build_spans(layer_offsets, L, plan.wide_spans.n_parts, plan.wide_spans.tiles, plan.wide_spans.part_begin,
                        plan.wide_spans.layer_begin);
        }
        plan.lay = make_layout(Kv, N, L, n_gram, norm_entries_bound(Kv, layer_offsets, L, plan.radices, node_type),
                               plan.radices, o.order, K + 1, small_elems, node_type,
                               o.fuse      ? dot_entries_bound(Kv, layer_offsets, L, plan.radices, node_type)
                               : plan.feed ? next_entries_bound(Kv, layer_offsets, L, plan.radices, node_type)
                                           : 0,
                               static_cast<int64_t>(plan.wide_spans.tiles.size()));
        // the combine tables this reduction reads: one per distinct tile capacity
        std::vector<int> caps;
        if (K == 1) caps.push_back(combine_tile_capacity(dtype, 1));
        for (size_t lv = 0; lv < plan.radices.size(); ++lv) {
            const bool leaves = lv == 0 || o.order == ADASUM_ORDER_LINEAR;
            caps.push_back(table_capacity(plan.feed != 0, plan.radices, lv, leaves ? dtype : node_type));
        }
        off_offsets = carve.take(sizeof(int64_t) * (static_cast<size_t>(L) + 1));
        off_gram_tiles = carve.take(sizeof(adasum_tile) * static_cast<size_t>(n_gram));
        off_gram_begin = carve.take(sizeof(int32_t) * (static_cast<size_t>(L) + 1));
        for (int cap : caps) {
            bool seen = false;
            for (const CombTable& c : combs) seen = seen || c.cap == cap;
            if (seen) continue;
            if (cap < 1 || gcap % cap != 0) return ADASUM_ERR_INVALID_ARG;   // (never: powers of two below the Gram tile)
            CombTable c;
            c.cap = cap;
            c.n = count_tiles(layer_offsets, L, cap);
            c.off_tiles = carve.take(sizeof(adasum_tile) * static_cast<size_t>(c.n));
            c.off_begin = carve.take(sizeof(int32_t) * (static_cast<size_t>(L) + 1));
            c.off_index = carve.take(sizeof(int32_t) * (static_cast<size_t>(n_gram) + 1));
            combs.push_back(c);
        }
        off_small = carve.take(sizeof(SmallLayer) * static_cast<size_t>(plan.n_small));
        if (plan.wide_spans.n_parts > 0) {
            off_span_tiles = carve.take(sizeof(adasum_tile) * plan.wide_spans.tiles.size());
            off_span_begin = carve.take(sizeof(int64_t) * ((static_cast<size_t>(L) + 2) / 2));
            off_span_parts = carve.take(sizeof(int64_t) * ((static_cast<size_t>(plan.wide_spans.n_parts) + 2) / 2));
        }
        off_ws = carve.take(plan.lay.total);
    } catch (const std::bad_alloc&) {
        return ADASUM_ERR_OUT_OF_MEMORY;
    }
    if (carve.off > ADASUM_NOALLOC_SCRATCH_BYTES) return ADASUM_ERR_TOO_LARGE;

    char* base = nullptr;
    size_t have = 0;
    ADASUM_LAUNCH(static_scratch(&base, &have));
    if (carve.off > have) return ADASUM_ERR_TOO_LARGE;
    ADASUM_HIP(hipGetDevice(&plan.device));

    int64_t* d_offsets = reinterpret_cast<int64_t*>(base + off_offsets);
    ADASUM_LAUNCH(launch_put_offsets(layer_offsets, L, d_offsets, stream));
    plan.gram_tiles.capacity = gcap;
    plan.gram_tiles.n_borrowed = n_gram;
    plan.gram_tiles.d_tiles = reinterpret_cast<adasum_tile*>(base + off_gram_tiles);
    plan.gram_tiles.d_layer_begin = reinterpret_cast<int32_t*>(base + off_gram_begin);
    ADASUM_LAUNCH(launch_build_tiles(d_offsets, L, gcap, n_gram, plan.gram_tiles.d_tiles,
                                     plan.gram_tiles.d_layer_begin, stream));
    try {
        for (const CombTable& c : combs) {
            TileTable t;
            t.capacity = c.cap;
            t.n_borrowed = c.n;
            t.d_tiles = reinterpret_cast<adasum_tile*>(base + c.off_tiles);
            t.d_layer_begin = reinterpret_cast<int32_t*>(base + c.off_begin);
            t.d_first_in_gram = reinterpret_cast<int32_t*>(base + c.off_index);
            ADASUM_LAUNCH(launch_build_tiles(d_offsets, L, c.cap, c.n, t.d_tiles, t.d_layer_begin, stream));
            ADASUM_LAUNCH(launch_index_tiles(d_offsets, plan.gram_tiles.d_tiles, n_gram, c.cap, t.d_layer_begin, c.n,
                                             t.d_first_in_gram, stream));
            plan.comb_tables.emplace(c.cap, std::move(t));
        }
    } catch (const std::bad_alloc&) {
        return ADASUM_ERR_OUT_OF_MEMORY;
    }
    plan.d_small = reinterpret_cast<SmallLayer*>(base + off_small);
    ADASUM_LAUNCH(launch_build_small(d_offsets, L, plan.n_small, plan.d_small, stream));
    if (plan.wide_spans.n_parts > 0) {
        // the host-built span table travels like the layer table: as 8-byte words in kernel arguments
        TileTable& w = plan.wide_spans;
        w.n_borrowed = static_cast<int64_t>(w.tiles.size());
        w.d_tiles = reinterpret_cast<adasum_tile*>(base + off_span_tiles);
        w.d_layer_begin = reinterpret_cast<int32_t*>(base + off_span_begin);
        w.d_part_begin = reinterpret_cast<int32_t*>(base + off_span_parts);
        try {
            static_assert(sizeof(adasum_tile) == 2 * sizeof(int64_t), "a span is two words");
            std::vector<int64_t> words(2 * w.tiles.size());
            std::memcpy(words.data(), w.tiles.data(), words.size() * sizeof(int64_t));
            ADASUM_LAUNCH(launch_put_words(words.data(), words.size(), reinterpret_cast<int64_t*>(w.d_tiles), stream));
            auto put_ints = [&](const std::vector<int32_t>& v, int32_t* dst) -> int {
                std::vector<int64_t> packed((v.size() + 1) / 2, 0);
                std::memcpy(packed.data(), v.data(), v.size() * sizeof(int32_t));
                ADASUM_LAUNCH(launch_put_words(packed.data(), packed.size(), reinterpret_cast<int64_t*>(dst), stream));
                return ADASUM_OK;
            };
            rc = put_ints(w.layer_begin, w.d_layer_begin);
            if (rc != ADASUM_OK) return rc;
            rc = put_ints(w.part_begin, w.d_part_begin);
            if (rc != ADASUM_OK) return rc;
        } catch (const std::bad_alloc&) {
            return ADASUM_ERR_OUT_OF_MEMORY;
        }
    }

    // per-kernel timing would create events: not here
    struct NoProfile {
        NoProfile() { t_no_profile = true; }
        ~NoProfile() { t_no_profile = false; }
    } quiet;
    char* ws = base + off_ws;
    try {
        if (K == 1) return run_copy(&plan, ws, grads, dtype, out, o, stream);
        if (o.order == ADASUM_ORDER_LINEAR) return run_linear(&plan, ws, grads, dtype, out, o, stream);
        return run_tree(&plan, ws, grads, dtype, out, o, stream);
    } catch (const std::bad_alloc&) {
        return ADASUM_ERR_OUT_OF_MEMORY;
    }
}

}  // namespace
}  // namespace adasum

using namespace adasum;

// A plan the caller owns (adasum_plan_create): not part of the library's cache.
struct adasum_plan {
    std::unique_ptr<Plan> plan;   // null for an empty problem (N = 0)
    int dtype = ADASUM_F32;
    Opts opts{};                  // as fixed at creation; layer_stats / delta_start per execute
    bool for_delta = false;
};

extern "C" {

int adasum_plan_create(int K, const int64_t* layer_offsets, int n_layers, int dtype, const adasum_options* opts,
                       adasum_plan** plan) {
    if (plan == nullptr || K < 1) return ADASUM_ERR_INVALID_ARG;
    *plan = nullptr;
    int rc = check_layer_table(layer_offsets, n_layers);
    if (rc != ADASUM_OK) return rc;
    if (!known_dtype(dtype)) return ADASUM_ERR_UNSUPPORTED;
    Opts o;
    rc = read_opts(opts, dtype, o);
    if (rc != ADASUM_OK) return rc;
    if (K > (1 << 20)) return ADASUM_ERR_UNSUPPORTED;
    if (o.layer_stats != nullptr) return ADASUM_ERR_INVALID_ARG;   // given per execute
    std::unique_ptr<adasum_plan> h(new (std::nothrow) adasum_plan());
    if (!h) return ADASUM_ERR_OUT_OF_MEMORY;
    h->dtype = dtype;
    h->for_delta = o.delta_start != nullptr;
    h->opts = o;
    h->opts.radix = o.radix == 0 ? default_radix(o) : o.radix;
    h->opts.delta_start = nullptr;
    if (layer_offsets[n_layers] > 0) {
        rc = make_plan(K, h->opts.radix, o.order, node_dtype(dtype), o.fuse != 0, h->for_delta || o.separate != 0,
                       layer_offsets, n_layers, h->plan);
        if (rc != ADASUM_OK) return rc;
        if (o.workspace != nullptr && o.workspace_bytes < h->plan->lay.total) return ADASUM_ERR_WORKSPACE;
        // everything execute needs exists from here on: it allocates nothing
        rc = prebuild_tables(h->plan.get(), dtype, o.order);
        if (rc != ADASUM_OK) return rc;
        char* ws = nullptr;
        rc = plan_workspace(h->plan.get(), h->opts, &ws);
        if (rc != ADASUM_OK) return rc;
    }
    *plan = h.release();
    return ADASUM_OK;
}

int adasum_plan_execute(adasum_plan* plan, const void* const* grads, void* out, double* layer_stats,
                        const void* delta_start, void* stream) {
    if (plan == nullptr) return ADASUM_ERR_INVALID_ARG;
    Opts o = plan->opts;
    o.layer_stats = layer_stats;
    o.delta_start = delta_start;
    if (layer_stats != nullptr) {
        if ((reinterpret_cast<uintptr_t>(layer_stats) & 7u) != 0) return ADASUM_ERR_MISALIGNED;
    }
    if ((delta_start != nullptr) != plan->for_delta) return ADASUM_ERR_INVALID_ARG;
    if (delta_start != nullptr && !aligned16(delta_start)) return ADASUM_ERR_MISALIGNED;
    if (!plan->plan) return ADASUM_OK;   // N = 0
    Plan* p = plan->plan.get();
    const int rc = check_call(grads, p->K, p->lay.N, plan->dtype, out, o);
    if (rc != ADASUM_OK) return rc;
    // the plan's own lock: plans of different callers enqueue side by side
    std::lock_guard<std::mutex> lock(p->mu);
    return execute_plan(p, grads, plan->dtype, out, o, stream);
}

int adasum_plan_workspace_bytes(const adasum_plan* plan, size_t* bytes) {
    if (plan == nullptr || bytes == nullptr) return ADASUM_ERR_INVALID_ARG;
    *bytes = plan->plan ? plan->plan->lay.total : 0;
    return ADASUM_OK;
}

int adasum_plan_destroy(adasum_plan* plan) {
    if (plan == nullptr) return ADASUM_OK;
    delete plan;   // frees tables, graphs and the plan's own workspace (hipFree waits for work in flight)
    return ADASUM_OK;
}

int adasum_reduce(const void* const* grads, int K, const int64_t* layer_offsets, int n_layers, int dtype,
                  void* out, void* stream) {
    return reduce_impl(grads, K, layer_offsets, n_layers, dtype, out, nullptr, stream);
}

int adasum_reduce_ex(const void* const* grads, int K, const int64_t* layer_offsets, int n_layers, int dtype,
                     void* out, const adasum_options* opts, void* stream) {
    return reduce_impl(grads, K, layer_offsets, n_layers, dtype, out, opts, stream);
}

int adasum_reduce_noalloc(const void* const* grads, int K, const int64_t* layer_offsets, int n_layers, int dtype,
                          void* out, const adasum_options* opts, void* stream) {
    return reduce_noalloc_impl(grads, K, layer_offsets, n_layers, dtype, out, opts, stream);
}

int adasum_workspace_bytes(int K, const int64_t* layer_offsets, int n_layers, int dtype,
                           const adasum_options* opts, size_t* bytes) {
    if (bytes == nullptr || K < 1) return ADASUM_ERR_INVALID_ARG;
    int rc = check_layer_table(layer_offsets, n_layers);
    if (rc != ADASUM_OK) return rc;
    if (!known_dtype(dtype)) return ADASUM_ERR_UNSUPPORTED;
    Opts o;
    rc = read_opts(opts, dtype, o);
    if (rc != ADASUM_OK && rc != ADASUM_ERR_WORKSPACE) return rc;
    try {
        std::vector<int> radices;
        const int radix = o.radix == 0 ? default_radix(o) : o.radix;
        rc = o.order == ADASUM_ORDER_LINEAR ? build_linear_passes(K, radix, radices)
                                            : build_levels(K, radix, radices);
        if (rc != ADASUM_OK) return rc;
        const int Kv = o.order == ADASUM_ORDER_LINEAR ? K : virtual_leaves(radices);
        std::vector<SmallLayer> small;
        const int64_t small_elems = K > 1 ? find_small_layers(layer_offsets, n_layers, small) : 0;
        const Layout lay = make_layout(Kv, layer_offsets[n_layers], n_layers,
                                       count_tiles(layer_offsets, n_layers, gram_tile_capacity(layer_offsets, n_layers)),
                                       norm_entries_bound(Kv, layer_offsets, n_layers, radices, node_dtype(dtype)),
                                       radices, o.order, K + 1, small_elems, node_dtype(dtype),
                                       o.fuse ? dot_entries_bound(Kv, layer_offsets, n_layers, radices, node_dtype(dtype))
                                       : (o.order == ADASUM_ORDER_TREE && !o.separate && o.delta_start == nullptr)
                                           ? next_entries_bound(Kv, layer_offsets, n_layers, radices, node_dtype(dtype))
                                           : 0,
                                       !radices.empty() && wide_radix(radices[0])
                                           ? count_spans(layer_offsets, n_layers, wide_part_count(layer_offsets[n_layers]))
                                           : 0);
        *bytes = lay.total;
    } catch (const std::bad_alloc&) {
        return ADASUM_ERR_OUT_OF_MEMORY;
    }
    return ADASUM_OK;
}

static int step_common(const void* const* x, int R, const int64_t* layer_offsets, int n_layers, int dtype) {
    if (R != 2 && R != 4 && R != 8 && R != 16 && R != 32 && R != 64) return ADASUM_ERR_UNSUPPORTED;
    int rc = check_layer_table(layer_offsets, n_layers);
    if (rc != ADASUM_OK) return rc;
    if (!known_dtype(dtype) || R > max_radix(dtype)) return ADASUM_ERR_UNSUPPORTED;
    return check_operands(x, R, layer_offsets[n_layers], dtype);
}

int adasum_group_gram(const void* const* x, int R, const int64_t* layer_offsets, int n_layers, int dtype,
                      double* gram, void* stream) {
    int rc = step_common(x, R, layer_offsets, n_layers, dtype);
    if (rc != ADASUM_OK) return rc;
    if (gram == nullptr && n_layers > 0) return ADASUM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(gram) & 7u) != 0) return ADASUM_ERR_MISALIGNED;
    if (n_layers == 0) return ADASUM_OK;
    std::lock_guard<std::mutex> lock(g_mutex);
    Plan* p = nullptr;
    rc = find_or_make_plan(R, R, kStepPlans, dtype, dtype, false, false, false, layer_offsets, n_layers, &p);
    if (rc != ADASUM_OK) return rc;
    Opts o{};
    char* ws = nullptr;
    rc = plan_workspace(p, o, &ws);
    if (rc != ADASUM_OK) return rc;
    bool eager = false;
    rc = begin_on_stream(p, stream, &eager);
    if (rc != ADASUM_OK) return rc;
    auto enqueue = [&]() -> int {
        double* partials = reinterpret_cast<double*>(ws + p->lay.off_partials);
        const TileSet gt = wide_radix(R) ? p->wide_spans.view() : p->gram_tiles.view();
        Operands ops;
        std::memset(&ops, 0, sizeof(ops));
        for (int r = 0; r < R; ++r) ops.pack[r] = x[r];
        ADASUM_LAUNCH(launch_gram(dtype, true, ops, gt, 1, R, partials, nullptr, stream));
        ADASUM_LAUNCH(launch_gram_finish(true, gt, n_layers, 1, R, partials, nullptr, gram, nullptr, 0, 0, 0, stream));
        return ADASUM_OK;
    };
    return end_on_stream(p, stream, eager, enqueue());
}

int adasum_group_weights(const double* gram, int R, int n_layers, int order, double* weights, void* stream) {
    if (R != 2 && R != 4 && R != 8 && R != 16 && R != 32 && R != 64) return ADASUM_ERR_UNSUPPORTED;
    if (n_layers < 0) return ADASUM_ERR_INVALID_ARG;
    if (order != ADASUM_ORDER_TREE && order != ADASUM_ORDER_LINEAR) return ADASUM_ERR_UNSUPPORTED;
    if ((gram == nullptr || weights == nullptr) && n_layers > 0) return ADASUM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(gram) & 7u) != 0 || (reinterpret_cast<uintptr_t>(weights) & 7u) != 0)
        return ADASUM_ERR_MISALIGNED;
    if (n_layers == 0) return ADASUM_OK;
    ADASUM_LAUNCH(launch_weights(gram, R, n_layers, order, 1, 0, 0, weights, stream));
    return ADASUM_OK;
}

int adasum_group_combine(const void* const* x, int R, const int64_t* layer_offsets, int n_layers, int dtype,
                         const double* weights, void* out, int out_dtype, double* sqnorm, void* stream) {
    int rc = step_common(x, R, layer_offsets, n_layers, dtype);
    if (rc != ADASUM_OK) return rc;
    if (!dtype_pair_ok(dtype, out_dtype)) return ADASUM_ERR_UNSUPPORTED;
    const int64_t N = layer_offsets[n_layers];
    if ((weights == nullptr && n_layers > 0) || (out == nullptr && N > 0)) return ADASUM_ERR_INVALID_ARG;
    if (!aligned16(out) || (reinterpret_cast<uintptr_t>(weights) & 7u) != 0 ||
        (reinterpret_cast<uintptr_t>(sqnorm) & 7u) != 0)
        return ADASUM_ERR_MISALIGNED;
    if (n_layers == 0) return ADASUM_OK;
    const size_t in_bytes = static_cast<size_t>(N) * elem_bytes(dtype);
    const size_t out_bytes = static_cast<size_t>(N) * elem_bytes(out_dtype);
    for (int r = 0; r < R; ++r) {
        if (r == 0 && x[0] == out && dtype == out_dtype) continue;   // in place on operand 0
        if (N > 0 && overlaps(x[r], in_bytes, out, out_bytes)) return ADASUM_ERR_ALIAS;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    Plan* p = nullptr;
    rc = find_or_make_plan(R, R, kStepPlans, dtype, dtype, false, false, false, layer_offsets, n_layers, &p);
    if (rc != ADASUM_OK) return rc;
    Opts o{};
    char* ws = nullptr;
    rc = plan_workspace(p, o, &ws);
    if (rc != ADASUM_OK) return rc;
    TileSet ct;
    rc = p->comb_tiles(dtype, R, &ct);
    if (rc != ADASUM_OK) return rc;
    bool eager = false;
    rc = begin_on_stream(p, stream, &eager);
    if (rc != ADASUM_OK) return rc;
    auto enqueue = [&]() -> int {
        double* normparts = reinterpret_cast<double*>(ws + p->lay.off_normparts);
        Operands ops;
        std::memset(&ops, 0, sizeof(ops));
        for (int r = 0; r < R; ++r) ops.pack[r] = x[r];
        Outputs outs;
        outs.base = static_cast<char*>(out);
        outs.slot_bytes = 0;
        outs.stride = 0;
        ADASUM_LAUNCH(launch_combine(dtype, out_dtype, ops, outs, ct, n_layers, 1, R, weights,
                                     sqnorm ? normparts : nullptr, nullptr, nullptr, stream));
        if (sqnorm != nullptr) {
            double* normcoarse = reinterpret_cast<double*>(ws + p->lay.off_normcoarse);
            const TileSet gt = p->gram_tiles.view();
            ADASUM_LAUNCH(launch_norm_coarsen(normparts, 1, ct, gt, normcoarse, stream));
            ADASUM_LAUNCH(launch_layer_sums(normcoarse, 1, gt, n_layers, sqnorm, 1, stream));
        }
        return ADASUM_OK;
    };
    return end_on_stream(p, stream, eager, enqueue());
}

int adasum_tile_capacity(void) { return kTile; }

int adasum_plan_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity, adasum_tile* tiles,
                      int64_t cap, int64_t* n_tiles) {
    if (n_tiles == nullptr || cap < 0 || (tiles == nullptr && cap > 0)) return ADASUM_ERR_INVALID_ARG;
    if (capacity == 0) capacity = kTile;
    if (capacity < 1 || capacity > 0x7fffffff) return ADASUM_ERR_INVALID_ARG;
    int rc = check_layer_table(layer_offsets, n_layers);
    if (rc != ADASUM_OK) return rc;
    try {
        std::vector<adasum_tile> t;
        std::vector<int32_t> ltb;
        build_tiles(layer_offsets, n_layers, capacity, t, ltb);
        *n_tiles = static_cast<int64_t>(t.size());
        const int64_t n = std::min<int64_t>(cap, static_cast<int64_t>(t.size()));
        for (int64_t i = 0; i < n; ++i) tiles[i] = t[i];
    } catch (const std::bad_alloc&) {
        return ADASUM_ERR_OUT_OF_MEMORY;
    }
    return ADASUM_OK;
}

int adasum_plan_levels(int K, int radix, int* radices, int cap, int* n_levels) {
    if (n_levels == nullptr || cap < 0 || (radices == nullptr && cap > 0)) return ADASUM_ERR_INVALID_ARG;
    std::vector<int> r;
    int rc = build_levels(K, radix, r);
    if (rc != ADASUM_OK) return rc;
    *n_levels = static_cast<int>(r.size());
    for (int i = 0; i < std::min<int>(cap, static_cast<int>(r.size())); ++i) radices[i] = r[i];
    return ADASUM_OK;
}

int adasum_plan_groups(int K, int radix, int* first_worker, int cap, int* n_groups) {
    if (n_groups == nullptr || cap < 0 || (first_worker == nullptr && cap > 0)) return ADASUM_ERR_INVALID_ARG;
    std::vector<int> r;
    int rc = build_levels(K, radix, r);
    if (rc != ADASUM_OK) return rc;
    const int depth = first_depth(r);
    const int groups = 1 << depth;
    *n_groups = groups;
    for (int g = 0; g <= groups && g < cap; ++g) {
        int lo = K, hi = K;
        if (g < groups) leaf_range(K, depth, g, lo, hi);
        first_worker[g] = lo;
    }
    return ADASUM_OK;
}

int adasum_profile_enable(int on) {
    g_profile = on != 0;
    return ADASUM_OK;
}

int adasum_profile_collect(adasum_kernel_profile* out, int cap, int* n) {
    if (n == nullptr || cap < 0 || (out == nullptr && cap > 0)) return ADASUM_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    std::vector<adasum_kernel_profile> agg;
    for (auto& r : g_records) {
        ADASUM_HIP(hipEventSynchronize(r.stop));
        float ms = 0.f;
        ADASUM_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
        size_t i = 0;
        for (; i < agg.size(); ++i)
            if (r.name == agg[i].name) break;
        if (i == agg.size()) {
            adasum_kernel_profile k;
            std::memset(&k, 0, sizeof(k));
            std::snprintf(k.name, sizeof(k.name), "%s", r.name.c_str());
            agg.push_back(k);
        }
        agg[i].launches += 1;
        agg[i].total_ms += ms;
        agg[i].bytes += r.bytes;
        g_event_pool.push_back(r.start);
        g_event_pool.push_back(r.stop);
    }
    g_records.clear();
    *n = static_cast<int>(agg.size());
    for (int i = 0; i < std::min<int>(cap, *n); ++i) out[i] = agg[i];
    return ADASUM_OK;
}

const char* adasum_strerror(int code) {
    switch (code) {
        case ADASUM_OK: return "ok";
        case ADASUM_ERR_INVALID_ARG: return "invalid argument";
        case ADASUM_ERR_UNSUPPORTED: return "unsupported (dtype f32/bf16/f16/f64; output the input type or f32, f64 only with f64; radix 2/4/8/16, f64 up to 8, 32/64 for bf16/f16 in tree order without the delta form; the delta form only in tree order)";
        case ADASUM_ERR_MISALIGNED: return "device pointer not 16-byte aligned";
        case ADASUM_ERR_OUT_OF_MEMORY: return "out of memory";
        case ADASUM_ERR_HIP: return "HIP call failed (see adasum_last_hip_error)";
        case ADASUM_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
        case ADASUM_ERR_ALIAS: return "output overlaps an input";
        case ADASUM_ERR_TOO_LARGE: return "adasum_reduce_noalloc: tile tables and workspace of this problem exceed the static scratch (ADASUM_NOALLOC_SCRATCH_BYTES); use adasum_reduce_ex or a plan";
        default: return "unknown error";
    }
}

int adasum_last_hip_error(void) { return g_last_hip_error; }

const char* adasum_version(void) { return "libadasum 0.3.0 (gfx950)"; }

int adasum_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mutex);
    g_plans.clear();
    std::lock_guard<std::mutex> prof_lock(g_prof_mutex);
    for (auto& r : g_records) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_records.clear();
    for (auto e : g_event_pool) (void)hipEventDestroy(e);
    g_event_pool.clear();
    return ADASUM_OK;
}

}  // extern "C"
