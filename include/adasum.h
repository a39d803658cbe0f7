/*
 * libadasum -- the Adasum tree combiner on one AMD MI355X (gfx950).
 *
 * Operation (arXiv 2006.02924):
 *   - two-gradient operator, Section 1 / Section 3:
 *       Adasum(g1, g2) = (1 - g1.g2 / (2 |g1|^2)) g1 + (1 - g1.g2 / (2 |g2|^2)) g2
 *   - K gradients: recursive halving, Section 3.4 (second recursion) -- for a power
 *     of two a balanced binary tree whose level-0 pairs are workers (2j, 2j+1); any
 *     other K splits every node [lo, hi) at lo + (hi - lo) / 2;
 *   - the operator's scalars are taken per layer of the fused gradient buffer,
 *     Section 3.6 (last paragraph) and Section 4.4.3 (boundary bookkeeping);
 *   - dot products and squared norms: each lane accumulates a short run in fp32,
 *     a wave adds its lanes in fp32, everything above that (and the ragged
 *     head/tail elements of a layer) is summed in fp64; the operator's scalars
 *     are computed in fp64 (Section 4.4.1 asks for double accumulation).  fp64
 *     inputs are reduced in fp64 throughout;
 *   - layers of at most 16 elements are reduced by the definition itself, pair by
 *     pair in fp64 over all K workers with nothing stored in between: vectors that
 *     short can nearly cancel at a tree node, where stored fp32 nodes lose digits.
 * Reading where the paper is silent: an operand whose squared norm is exactly 0
 * gets coefficient 1, so Adasum(0, g) = g and Adasum(0, 0) = 0.
 *
 * Supported magnitudes.  Products of two stored values are formed and summed in fp32
 * lanes (fp64 for fp64 storage), so for fp32 and bf16 storage a layer's values must
 * keep their squares inside the fp32 range: root-mean-square magnitude of a layer
 * between about 1e-17 and 1e+17 (checked against the oracle at 1e-15 and 1e+15; a first
 * pass of radix 32 or 64 sums up to 2^18 products in fp32 before it widens them: 1e+16).
 * fp16 storage cannot leave that range; fp64 storage has fp64's (1e-150 .. 1e+150).
 * Outside it the result of THAT layer is not the operator's: squares that underflow
 * to zero put the layer on (or near) the zero-norm convention, a plain sum of the
 * workers; squares that overflow make it NaN.  Other layers are unaffected.  Gradients, with
 * or without loss scaling, are many orders of magnitude inside the range.
 *
 * Conventions for every entry point
 *   - returns ADASUM_OK (0) or a negative ADASUM_ERR_* code; never throws,
 *     aborts or prints.  All argument validation happens before any device
 *     work, so the error paths need no GPU.
 *   - "HOST" / "DEVICE" says where a pointer must live.  DEVICE pointers must be
 *     16-byte aligned.  The caller owns every buffer it passes; inputs are never
 *     modified; host arrays are copied during the call and may be freed at return.
 *   - work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns without synchronising.
 *   - thread-safe.  Calls with the same K, dtypes, radix, order, delta form and
 *     layer table share one cached plan and its workspace; the library orders
 *     them on the device: a call issued on another stream than the previous call
 *     with that plan first waits for it (an event wait, no host blocking).  So
 *     the same model shape may be reduced from several host threads and streams
 *     at once and every result is right, but those calls run one after another;
 *     callers that want them to overlap hold one plan each (adasum_plan_create).
 *     No ordering is inserted on a stream that is being captured into a graph:
 *     what a caller captures, it orders.
 *   - results are deterministic: identical inputs give bit-identical outputs
 *     (no atomics anywhere on the path).
 */
#ifndef ADASUM_H
#define ADASUM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* the library exports the entry points below and nothing else */
#define ADASUM_API __attribute__((visibility("default")))

/* element storage types */
#define ADASUM_F32  0   /* IEEE binary32 */
#define ADASUM_BF16 1   /* bfloat16; stores round to nearest even */
#define ADASUM_F16  2   /* IEEE binary16; stores round to nearest even (no loss scaling here:
                           values must fit the format, as Section 4.4.1's dynamic scaling ensures) */
#define ADASUM_F64  3   /* IEEE binary64: reduced in fp64 throughout (lanes, tree nodes, output);
                           only to an fp64 result, radix at most 8 (default 8) */

/* error codes */
#define ADASUM_OK                 0
#define ADASUM_ERR_INVALID_ARG   -1  /* null pointer, K < 1, n_layers < 0, bad layer table, bad option */
#define ADASUM_ERR_UNSUPPORTED   -2  /* unknown dtype / radix / order, or a combination not offered */
#define ADASUM_ERR_MISALIGNED    -3  /* a DEVICE pointer is not 16-byte aligned */
#define ADASUM_ERR_OUT_OF_MEMORY -4  /* device or host allocation failed */
#define ADASUM_ERR_HIP           -5  /* a HIP call failed; see adasum_last_hip_error() */
#define ADASUM_ERR_WORKSPACE     -6  /* caller-provided workspace too small or misaligned */
#define ADASUM_ERR_ALIAS         -7  /* `out` overlaps an input buffer */
#define ADASUM_ERR_TOO_LARGE     -8  /* adasum_reduce_noalloc: the problem needs more than the static scratch */

/* tree order (Section 3.4 gives both recursions; they give different results) */
#define ADASUM_ORDER_TREE   0   /* recursive halving -- the one the paper uses in practice */
#define ADASUM_ORDER_LINEAR 1   /* left-to-right fold */

/*
 * Options for adasum_reduce_ex.  Zero-initialise, set struct_bytes = sizeof,
 * then set what differs from the defaults.
 */
typedef struct adasum_options {
    uint32_t struct_bytes;     /* sizeof(adasum_options) as the caller compiled it */
    int32_t  out_dtype;        /* the input dtype or ADASUM_F32 (any 16- or 32-bit storage type
                                  when the input is fp32; fp64 goes with fp64 only);
                                  -1 = same as the input dtype */
    int32_t  radix;            /* how many binary tree levels one pass over the data fuses:
                                  2 = one level per pass (reduce pass + combine pass per level),
                                  4 / 8 / 16 = two / three / four levels per pass (the pass
                                  computes the group's Gram matrix, the tree's scalars follow
                                  from it);
                                  32 / 64 = five / six levels in the first pass, for bf16 and fp16
                                  inputs in ADASUM_ORDER_TREE without delta_start (else
                                  ADASUM_ERR_UNSUPPORTED): with 528 or 2080 entries per group the
                                  Gram matrix is a dense contraction X X^T and is computed on the
                                  matrix cores (exact 16-bit products, summed in fp32 within a
                                  workgroup's span of a layer, fp64 above); K = 64 is then a single
                                  pass.  Later passes, over fp32 nodes, stay at 16 or less;
                                  0 = library default (16; 8 for fp64 and the delta form).
                                  The result is the same binary tree. */
    int32_t  order;            /* ADASUM_ORDER_TREE (default) | ADASUM_ORDER_LINEAR */
    int32_t  use_graph;        /* 1 = replay the level ladder as one hipGraph launch: captured
                                  once per distinct set of buffers (grads, out, workspace,
                                  layer_stats), cached in the plan, relaunched while they match */
    int32_t  fuse_siblings;    /* radix 2, ADASUM_ORDER_TREE, no delta_start (else ADASUM_ERR_UNSUPPORTED):
                                  1 = the combine of a level handles the two sibling pairs of an element
                                  range together and also leaves the dot product of the two nodes it
                                  writes (Section 3.4's recursion taken one level ahead), so only the
                                  first level makes a reduce pass of its own.  Same tree, same result up
                                  to rounding, a quarter fewer bytes than plain radix 2.  (This field was
                                  reserved and had to be 0 before.) */
    void*    workspace;        /* DEVICE, 256-byte aligned, or NULL = library-owned, cached per plan */
    size_t   workspace_bytes;  /* size of `workspace`; see adasum_workspace_bytes */
    double*  layer_stats;      /* DEVICE or NULL: n_layers x 2 doubles written per call,
                                  [l][0] = |Adasum(g_1..g_K)|^2 of layer l (of the value before
                                  it is rounded to the output type), [l][1] = sum_i |g_i|^2; their ratio
                                  is the orthogonality metric of Section 3.6 (in either order: the
                                  first entry is the norm of whatever `order` computes) */
    const void* delta_start;   /* DEVICE or NULL.  Section 4.1 (Adasum applied after the optimizer):
                                  N elements of the input dtype, 16-byte aligned -- the model
                                  parameters before the workers' local optimizer steps.  When set,
                                  grads[k] holds worker k's parameters AFTER its local step; the
                                  library reduces the effective gradients grads[k] - delta_start
                                  (formed on the fly, never stored) and writes
                                  out = delta_start + Adasum(...), the new parameters.
                                  layer_stats then describe the effective gradients.  Needs
                                  out_dtype == the input dtype and ADASUM_ORDER_TREE
                                  (else ADASUM_ERR_UNSUPPORTED).  `out` may be the very same
                                  buffer as delta_start (in-place parameter update); any other
                                  overlap is ADASUM_ERR_ALIAS.  A struct_bytes that ends before
                                  this field (the struct as it was without it) reads as NULL. */
    int32_t  separate_passes;  /* 0 (default): in the tree order, the combine of a pass also leaves the
                                  Gram matrix of the next pass's group (it handles the sibling groups of
                                  a tile in one workgroup, one wave each, and the waves exchange what they
                                  wrote), so that only the first pass reads its operands twice;
                                  1: every pass makes a reduce pass of its own over its operands (for
                                  measurements; the result is the same up to rounding).  A struct_bytes
                                  that ends before this field reads as 0. */
    int32_t  reserved1;        /* must be 0 */
} adasum_options;

/*
 * The combiner.  Reduces K per-worker gradients to one, per layer, up the
 * binary tree (Sections 3, 3.4, 3.6).
 *
 *   grads          HOST array of K DEVICE pointers; grads[k] is worker k's flat
 *                  fused buffer of N = layer_offsets[n_layers] elements of `dtype`
 *   K              number of workers, >= 1 (K = 1 copies).  Any count: the node over
 *                  workers [lo, hi) splits at lo + (hi - lo) / 2, which is the paper's
 *                  recursion g_[0,n/2) | g_[n/2,n] read literally (the left part takes
 *                  floor(count / 2) workers) and the balanced tree for a power of two
 *   layer_offsets  HOST, n_layers + 1 entries in element units, [0] = 0,
 *                  non-decreasing; layer l is [layer_offsets[l], layer_offsets[l+1]);
 *                  empty layers are allowed; N = 0 is a no-op
 *   dtype          ADASUM_F32 | ADASUM_BF16 | ADASUM_F16 | ADASUM_F64: storage type of grads AND of out
 *   out            DEVICE, N elements of `dtype`; must not overlap any input
 *   stream         hipStream_t
 *
 * Intermediate tree nodes are kept in fp32 for 16- and 32-bit storage types (fp64
 * for fp64); the only rounding to bf16 / fp16 is the final store.  Uses a
 * library-owned workspace cached with the plan for (K, radix, order, node type,
 * layer table); the first call with a new shape allocates.  At most 64 plans are
 * kept; making a 65th frees the least recently used one (and waits for the device).
 */
ADASUM_API int adasum_reduce(const void* const* grads, int K,
                  const int64_t* layer_offsets, int n_layers,
                  int dtype, void* out, void* stream);

/* Same operation with options (output dtype, radix, order, caller workspace,
 * per-layer statistics).  opts == NULL means all defaults. */
ADASUM_API int adasum_reduce_ex(const void* const* grads, int K,
                     const int64_t* layer_offsets, int n_layers,
                     int dtype, void* out, const adasum_options* opts, void* stream);

/* Bytes of DEVICE workspace adasum_reduce_ex needs for this problem (intermediate
 * tree nodes, per-tile partial sums, coefficient tables, the compact copy of the
 * small layers).  Depends on dtype, radix, order, fuse_siblings, separate_passes and on
 * whether delta_start is set (any non-NULL value).  Host-only. */
ADASUM_API int adasum_workspace_bytes(int K, const int64_t* layer_offsets, int n_layers,
                           int dtype, const adasum_options* opts, size_t* bytes);

/* ---- plans the caller owns ----
 *
 * adasum_reduce(_ex) look their plan up in a cache by shape on every call.  A caller
 * that reduces the same shape again and again can hold the plan itself: tile tables
 * on the current device, the pass schedule, captured graphs and (unless a workspace is
 * given) the plan's own workspace.  All of it is allocated by adasum_plan_create:
 * adasum_plan_execute with use_graph = 0 and profiling off only launches kernels
 * (no allocation, no copy, no synchronisation), so it may be issued on a stream the
 * caller is capturing into a hipGraph of its own.
 *
 *   opts   as for adasum_reduce_ex; out_dtype, radix, order, use_graph and
 *          workspace / workspace_bytes are fixed for the plan's lifetime;
 *          layer_stats must be NULL here (it is an argument of execute);
 *          delta_start != NULL (any 16-byte aligned value) plans for the delta form of
 *          Section 4.1: every execute must then pass a delta_start, else none may
 *   plan   receives the handle; destroy it with adasum_plan_destroy (waits for the
 *          device).  adasum_shutdown does not touch it.
 * Executes on one plan share its workspace and are ordered like the calls above (a
 * different stream than the previous execute waits for it; none while capturing).
 * Executes on different plans take no common lock and may overlap.
 */
typedef struct adasum_plan adasum_plan;
ADASUM_API int adasum_plan_create(int K, const int64_t* layer_offsets, int n_layers, int dtype,
                                  const adasum_options* opts, adasum_plan** plan);
/* grads: HOST array of K DEVICE pointers; out, layer_stats (or NULL), delta_start (or
 * NULL): DEVICE, as in adasum_reduce_ex.  Same checks, same errors. */
ADASUM_API int adasum_plan_execute(adasum_plan* plan, const void* const* grads, void* out,
                                   double* layer_stats, const void* delta_start, void* stream);
/* Bytes of workspace the plan uses (what adasum_workspace_bytes reports for its shape). */
ADASUM_API int adasum_plan_workspace_bytes(const adasum_plan* plan, size_t* bytes);
ADASUM_API int adasum_plan_destroy(adasum_plan* plan);

/* ---- for callers that cannot allocate ----
 *
 * Code under HIP graph capture, tight serving loops and harnesses that forbid device
 * allocation cannot use the entry points above on a new shape (their first call with a
 * shape allocates tile tables and a workspace with hipMalloc).  adasum_reduce_noalloc is
 * adasum_reduce_ex for them: same arguments, same kernels, same result bit for bit, but it
 * calls no hipMalloc / hipFree / hipMemcpy and no other allocating or synchronising routine.
 * The layer table travels to the device in kernel arguments, the tile tables are built there,
 * and tables plus workspace live in one static device array of
 * ADASUM_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until the process
 * ends.  Per-kernel timing (adasum_profile_enable) does not cover it.
 *
 *   opts   as for adasum_reduce_ex, except workspace must be NULL and use_graph 0
 *          (ADASUM_ERR_INVALID_ARG otherwise); NULL = all defaults
 * Limit: tables + workspace of the problem (about adasum_workspace_bytes() plus 16 bytes per
 * 256 to 512 elements) must fit the array, else ADASUM_ERR_TOO_LARGE and nothing is enqueued.  That
 * holds for e.g. ResNet-50 (25.6 M elements) at K <= 16, or 3 M elements at K = 64 -- and, since a
 * single pass keeps no intermediate nodes, for BERT-Large (335 M elements) at K <= 64 with radix 64.
 * Every call on one GPU uses the same array and finds the previous call's contents there:
 * each call rebuilds all it reads (nothing needs to start at zero), and two calls that
 * overlap in time on one GPU -- on different streams without an ordering between them -- race.
 * Calls on one stream, or ordered by events, are safe.
 */
#define ADASUM_NOALLOC_SCRATCH_BYTES (64u << 20)
ADASUM_API int adasum_reduce_noalloc(const void* const* grads, int K,
                          const int64_t* layer_offsets, int n_layers,
                          int dtype, void* out, const adasum_options* opts, void* stream);

/* ---- the steps of one tree level, exposed so that each can be checked alone ---- */

/*
 * Step 1 (Algorithm 1, "partial dot products"): per layer, the Gram matrix of R
 * operands, G[i][j] = x_i . x_j (the pair case R = 2 is the triple
 * [a.b, a.a, b.b]).
 *   x      HOST array of R DEVICE pointers (N elements of `dtype` each)
 *   R      2, 4, 8 or 16 (fp64: up to 8); 32 or 64 for bf16 and fp16 operands
 *   gram   DEVICE, n_layers x R x R doubles, row-major per layer, symmetric
 */
ADASUM_API int adasum_group_gram(const void* const* x, int R,
                      const int64_t* layer_offsets, int n_layers,
                      int dtype, double* gram, void* stream);

/*
 * Step 2 (Algorithm 1, "finish dot products" + the scalars of "apply Adasum"):
 * per layer, the weights w with  tree(x_0..x_{R-1}) = sum_r w_r x_r,  obtained
 * from the Gram matrix by walking the binary tree over the R leaves bottom-up;
 * R = 2 gives w = (1 - d/(2 n1), 1 - d/(2 n2)).  fp64 arithmetic and result.
 *   gram     DEVICE, n_layers x R x R doubles (as written by adasum_group_gram)
 *   weights  DEVICE, n_layers x R doubles
 */
ADASUM_API int adasum_group_weights(const double* gram, int R, int n_layers, int order,
                         double* weights, void* stream);

/*
 * Step 3 (Algorithm 1, "apply Adasum"): out = sum_r w[layer][r] * x_r element
 * by element (fp32 fused multiply-adds with the weights rounded to fp32, one
 * rounding at the store; the few elements of a layer's ragged head and tail are
 * done in fp64), and in the same pass the squared norm of the result per layer.
 *   weights    DEVICE, n_layers x R doubles
 *   out        DEVICE, N elements of out_dtype; may be x[0] itself (in place)
 *              when out_dtype == dtype, must not overlap any other operand
 *   sqnorm     DEVICE, n_layers doubles, or NULL
 */
ADASUM_API int adasum_group_combine(const void* const* x, int R,
                         const int64_t* layer_offsets, int n_layers,
                         int dtype, const double* weights,
                         void* out, int out_dtype, double* sqnorm, void* stream);

/* ---- host-side planning, exposed for inspection and tests (no GPU needed) ---- */

typedef struct adasum_tile {
    int64_t start;   /* first element (global index into the fused buffer) */
    int32_t len;     /* 1 .. tile capacity; a tile never crosses a layer boundary */
    int32_t layer;
} adasum_tile;

/* Elements one workgroup of the Gram pass covers at most (a layer table with fewer
 * than 2048 such tiles is cut into tiles of 16384 instead).  (The combine pass
 * uses finer tables: one 16-byte load per lane and operand, 64 to 256 lanes.) */
ADASUM_API int adasum_tile_capacity(void);

/* Writes the tile table for a layer table: consecutive runs of at most
 * `capacity` elements (0 = adasum_tile_capacity()) whose boundaries fall on
 * global multiples of the capacity and on layer boundaries, so a tile never
 * crosses a layer.  *n_tiles receives the number of tiles; at most `cap` entries
 * are written to `tiles` (tiles may be NULL with cap = 0 to query the count).
 * Tiles are ordered by start; empty layers get no tile. */
ADASUM_API int adasum_plan_tiles(const int64_t* layer_offsets, int n_layers, int64_t capacity,
                      adasum_tile* tiles, int64_t cap, int64_t* n_tiles);

/* Writes the radix of every pass of the tree order for K workers, e.g. K = 64,
 * radix 8 -> {8, 8}; K = 128 -> {8, 8, 2}.  Their product is K for a power of
 * two, else the next power of two: the first pass's groups are then sub-trees
 * with fewer leaves than its radix (see adasum_plan_groups), e.g. K = 12,
 * radix 8 -> {8, 2} with two groups of 6.  *n_levels receives the count; at
 * most `cap` entries are written. */
ADASUM_API int adasum_plan_levels(int K, int radix, int* radices, int cap, int* n_levels);

/* The groups of the first pass of the tree order: group g reduces workers
 * first_worker[g] .. first_worker[g+1]-1, a whole sub-tree of the recursion of
 * Section 3.4 (split at lo + (hi - lo) / 2).  *n_groups receives the number of
 * groups G; at most `cap` of the G + 1 boundaries are written. */
ADASUM_API int adasum_plan_groups(int K, int radix, int* first_worker, int cap, int* n_groups);

/* ---- per-kernel timing (HIP events on the caller's stream) ---- */

typedef struct adasum_kernel_profile {
    char     name[48];        /* e.g. "combine<bf16,f32,R=2>" */
    int64_t  launches;
    double   total_ms;        /* sum of event-measured durations */
    double   bytes;           /* algorithmic bytes summed over those launches:
                                 operands read once + outputs written once */
} adasum_kernel_profile;

/* on != 0: every kernel launched by adasum_reduce(_ex) is bracketed by a pair
 * of HIP events on its stream.  Off by default. */
ADASUM_API int adasum_profile_enable(int on);
/* Synchronises the recorded events, aggregates by kernel name, writes at most
 * `cap` entries, sets *n to the number of distinct kernels, and clears the log. */
ADASUM_API int adasum_profile_collect(adasum_kernel_profile* out, int cap, int* n);

/* ---- housekeeping ---- */
ADASUM_API const char* adasum_strerror(int code);
ADASUM_API int         adasum_last_hip_error(void);   /* hipError_t of the last failing HIP call in this thread */
ADASUM_API const char* adasum_version(void);
/* Frees every cached plan and library-owned workspace.  The caller must have
 * synchronised the streams it used. */
ADASUM_API int adasum_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* ADASUM_H */
