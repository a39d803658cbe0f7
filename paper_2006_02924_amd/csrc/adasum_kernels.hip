// gfx950 (CDNA4) kernels of the Adasum tree combiner (arXiv 2006.02924).
//
// One pass over a group of R sibling tree nodes does what Algorithm 1 does for
// a pair: "partial dot products" (gram_kernel), "finish dot products"
// (gram_finish_kernel, which also walks the scalars of the Section 3 operator up
// the tree of Section 3.4 over the group's R leaves: wave_tree_weights), and
// "apply Adasum" (combine_kernel), which also accumulates the squared norm of
// what it writes so the next pass needs only the cross dot products.  Layers
// of a few elements are redone by the definition in fp64 (small_*_kernel).
//
// The work is HBM-bound streaming on the vector units; only the opt-in wide first pass
// (radix 32 and 64, gram_wide_kernel below), whose Gram matrix is a dense contraction,
// uses the matrix cores.  Every workgroup owns one
// tile (consecutive elements inside one layer): a long one (kTile elements) in
// the read-only Gram pass, where a workgroup's start-up and its reduction must
// be amortised, and a short one (one 16-byte load per lane and operand, or per
// pair of operands) in the combine pass, where short-lived workgroups keep the
// mixed read/write stream near sequential.  64-wide waves issue 16-byte
// non-temporal loads that cover 1 KiB of one operand per instruction (the
// 16-operand combine of 16-bit inputs: 512 bytes of each of two operands);
// partial sums go lane (fp32; fp64 for
// fp64 storage) -> wave (shuffles) -> workgroup (fp64 via LDS) -> per-tile fp64
// partial in memory, summed later in a fixed order; no atomics anywhere.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "adasum_host.h"

// Tuning knobs (compile-time): 16-byte loads a lane issues before consuming any,
// and whether streaming loads / stores carry the non-temporal hint.
#ifndef ADASUM_INFLIGHT
#define ADASUM_INFLIGHT 8
#endif
#ifndef ADASUM_NT_LOAD
#define ADASUM_NT_LOAD 1
#endif
#ifndef ADASUM_NT_STORE
#define ADASUM_NT_STORE 1
#endif
// bf16 Gram entries through v_dot2c_f32_bf16: 0 = never (unpack + fp32 FMA), 1 = only at
// radix 16, where 136 entries per lane would otherwise be bound by the vector ALUs
// (14.8 ms instead of 7.0 ms on the K=64 BERT-Large case), 2 = always.  The instruction
// adds two exact bf16 products to the fp32 accumulator but, unlike an FMA, does not round
// to nearest (measured: 1585 of 65536 probes differ from the FMA chain, all one ulp toward zero).
#ifndef ADASUM_BF16_DOT2
#define ADASUM_BF16_DOT2 1
#endif

// Blocks the wide Gram pass (radix 32, 64) loads ahead of the one it multiplies: 1 or 2.  Measured
// alike (6.21 and 6.24 ms on the K = 64 BERT-Large case); 1 leaves the compiler 32 registers more.
#ifndef ADASUM_WIDE_AHEAD
#define ADASUM_WIDE_AHEAD 1
#endif

// Scratch memory of the entry point that allocates nothing (adasum_reduce_noalloc): tile
// tables and workspace of one reduction.  One copy per GPU, held until the process ends; its
// device address comes from hipGetSymbolAddress (static_scratch below), never from this name.
static __device__ __align__(256) unsigned char scratch[ADASUM_NOALLOC_SCRATCH_BYTES];

namespace adasum {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

struct bf16_t { unsigned short v; };
struct f16_t { unsigned short v; };   // IEEE binary16
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

// VEC: elements per 16-byte granule; acc_t: the type lanes compute in (fp64 storage is
// reduced in fp64 throughout, everything else in fp32 lanes with fp64 above the wave)
template <typename T> struct Traits;
template <> struct Traits<float>  { static constexpr int VEC = 4; typedef float acc_t; };
template <> struct Traits<bf16_t> { static constexpr int VEC = 8; typedef float acc_t; };
template <> struct Traits<f16_t>  { static constexpr int VEC = 8; typedef float acc_t; };
template <> struct Traits<double> { static constexpr int VEC = 2; typedef double acc_t; };

__device__ __forceinline__ float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }

// round to nearest even; NaN stays NaN (quiet), overflow rounds to infinity
__device__ __forceinline__ unsigned int f32_to_bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// G consecutive elements of T held as raw 32-bit words (8, 16 or 32 bytes)
template <typename T, int G>
struct Granule {
    static constexpr int NW = G * (int)sizeof(T) / 4;
    static_assert(NW == 2 || NW == 4 || NW == 8, "granule must be 8, 16 or 32 bytes");
    unsigned int w[NW];
};

template <typename V>
__device__ __forceinline__ V stream_load(const V* p) {
#if ADASUM_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

template <bool NT, typename V>
__device__ __forceinline__ void stream_store(V v, V* p) {
    if constexpr (NT && ADASUM_NT_STORE) {
        __builtin_nontemporal_store(v, p);
    } else {
        *p = v;
    }
}

// p must be aligned to the granule size (to 16 bytes for a 32-byte granule)
template <typename T, int G>
__device__ __forceinline__ void load_raw(Granule<T, G>& r, const T* p) {
    constexpr int NW = Granule<T, G>::NW;
    if constexpr (NW == 2) {
        const u32x2 q = stream_load(reinterpret_cast<const u32x2*>(p));
        r.w[0] = q.x;
        r.w[1] = q.y;
    } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i) {
            const u32x4 q = stream_load(reinterpret_cast<const u32x4*>(p) + i);
            r.w[4 * i + 0] = q.x;
            r.w[4 * i + 1] = q.y;
            r.w[4 * i + 2] = q.z;
            r.w[4 * i + 3] = q.w;
        }
    }
}

template <int G>
__device__ __forceinline__ void unpack(const Granule<float, G>& r, float (&v)[G]) {
#pragma unroll
    for (int i = 0; i < G; ++i) v[i] = __uint_as_float(r.w[i]);
}

template <int G>
__device__ __forceinline__ void unpack(const Granule<bf16_t, G>& r, float (&v)[G]) {
#pragma unroll
    for (int i = 0; i < G / 2; ++i) {
        v[2 * i + 0] = __uint_as_float(r.w[i] << 16);
        v[2 * i + 1] = __uint_as_float(r.w[i] & 0xffff0000u);
    }
}

template <int G>
__device__ __forceinline__ void unpack(const Granule<f16_t, G>& r, float (&v)[G]) {
#pragma unroll
    for (int i = 0; i < G / 2; ++i) {
        const f16x2_t h = __builtin_bit_cast(f16x2_t, r.w[i]);
        v[2 * i + 0] = static_cast<float>(h.x);
        v[2 * i + 1] = static_cast<float>(h.y);
    }
}

template <int G>
__device__ __forceinline__ void unpack(const Granule<double, G>& r, double (&v)[G]) {
#pragma unroll
    for (int i = 0; i < G; ++i)
        v[i] = __longlong_as_double((static_cast<long long>(r.w[2 * i + 1]) << 32) |
                                    static_cast<long long>(r.w[2 * i]));
}

// fp32 -> binary16, round to nearest even (the conversion instruction's default mode)
__device__ __forceinline__ unsigned int f32_to_f16_bits(float f) {
    const _Float16 h = static_cast<_Float16>(f);
    return static_cast<unsigned int>(__builtin_bit_cast(unsigned short, h));
}

template <bool NT, int NW>
__device__ __forceinline__ void store_words(void* p, const unsigned int (&w)[NW]) {
    if constexpr (NW == 2) {
        u32x2 q;
        q.x = w[0];
        q.y = w[1];
        stream_store<NT>(q, reinterpret_cast<u32x2*>(p));
    } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i) {
            u32x4 q;
            q.x = w[4 * i + 0];
            q.y = w[4 * i + 1];
            q.z = w[4 * i + 2];
            q.w = w[4 * i + 3];
            stream_store<NT>(q, reinterpret_cast<u32x4*>(p) + i);
        }
    }
}

template <bool NT, int G>
__device__ __forceinline__ void store_granule(float* p, const float (&v)[G]) {
    unsigned int w[G];
#pragma unroll
    for (int i = 0; i < G; ++i) w[i] = __float_as_uint(v[i]);
    store_words<NT>(p, w);
}

template <bool NT, int G>
__device__ __forceinline__ void store_granule(bf16_t* p, const float (&v)[G]) {
    unsigned int w[G / 2];
#pragma unroll
    for (int i = 0; i < G / 2; ++i) w[i] = f32_to_bf16_rne(v[2 * i]) | (f32_to_bf16_rne(v[2 * i + 1]) << 16);
    store_words<NT>(p, w);
}

template <bool NT, int G>
__device__ __forceinline__ void store_granule(f16_t* p, const float (&v)[G]) {
    unsigned int w[G / 2];
#pragma unroll
    for (int i = 0; i < G / 2; ++i) w[i] = f32_to_f16_bits(v[2 * i]) | (f32_to_f16_bits(v[2 * i + 1]) << 16);
    store_words<NT>(p, w);
}

template <bool NT, int G>
__device__ __forceinline__ void store_granule(double* p, const double (&v)[G]) {
    unsigned int w[2 * G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const long long b = __double_as_longlong(v[i]);
        w[2 * i] = static_cast<unsigned int>(b);
        w[2 * i + 1] = static_cast<unsigned int>(b >> 32);
    }
    store_words<NT>(p, w);
}

__device__ __forceinline__ double load_elem(const double* p) { return *p; }
__device__ __forceinline__ void store_elem(double* p, double v) { *p = v; }
__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const f16_t* p) {
    return static_cast<float>(__builtin_bit_cast(_Float16, p->v));
}
__device__ __forceinline__ void store_elem(f16_t* p, float v) {
    p->v = static_cast<unsigned short>(f32_to_f16_bits(v));
}
__device__ __forceinline__ float load_elem(const bf16_t* p) {
    return __uint_as_float(static_cast<unsigned int>(p->v) << 16);
}
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(bf16_t* p, float v) {
    p->v = static_cast<unsigned short>(f32_to_bf16_rne(v));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Sums every one of N per-lane values over the 64 lanes of a wave with N + N/2 + ... shuffles
// instead of 6 N: at the step with mask m a lane whose bit m is clear keeps the even-indexed
// values and hands the odd-indexed ones to its partner (and the other way round), so each step
// halves the number of values a lane carries.  On return lane l holds in v[i] the complete sum
// of value number l + 64 i (values past N are padding).  Fixed order: bit-identical reruns.
template <typename A, int N>
__device__ __forceinline__ void wave_sum_scatter(A (&v)[N], int lane) {
    static_assert(N >= 1, "");
    int n = N;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const bool upper = (lane & m) != 0;
        const int half = (n + 1) / 2;
#pragma unroll
        for (int i = 0; i < (N + 1) / 2; ++i) {
            if (i < half) {
                const A a = v[2 * i];
                const A b = (2 * i + 1 < n) ? v[2 * i + 1] : static_cast<A>(0);
                const A keep = upper ? b : a, send = upper ? a : b;
                v[i] = keep + __shfl_xor(send, m, 64);
            }
        }
        n = half;
    }
}

template <int R>
__device__ __forceinline__ const void* operand_ptr(const Operands& ops, int g, int r) {
    return ops.pack[g * R + r];
}

// The tile split every kernel uses: [start, hs) scalar head, [bs, be) whole
// granules aligned to G elements of the global index, [ts, end) scalar tail.
struct Split {
    long long start, end, bs, hs, ts;
    int ng, nh, nt;
};

template <int G>
__device__ __forceinline__ Split split_tile(const adasum_tile& t) {
    Split s;
    s.start = t.start;
    s.end = t.start + t.len;
    s.bs = (s.start + (G - 1)) / G * G;
    const long long be = s.end / G * G;
    s.hs = s.bs < s.end ? s.bs : s.end;
    s.ts = be > s.hs ? be : s.hs;
    s.ng = be > s.bs ? static_cast<int>((be - s.bs) / G) : 0;
    s.nh = static_cast<int>(s.hs - s.start);
    s.nt = static_cast<int>(s.end - s.ts);
    return s;
}

// ---------------------------------------------------------------------------
// Step 1: per-tile partial Gram entries of R operands.
// Entry order: for i < R, for j from (DIAG ? i : i+1) to R-1.
// partials[(group * n_tiles + tile) * NP + entry]: one workgroup's entries side by side (written
// entry-major, 136 scattered 8-byte stores per workgroup cost the radix-16 pass 9 %)
// ---------------------------------------------------------------------------
// DELTA: the operands are x_r - start (the "effective gradient" of Section 4.1:
// parameters after the local step minus the parameters before it), formed on
// the fly; `start` has the operands' type.
// HEAD32: operand 0 is stored as fp32 while the others are 16-bit (the running result of the
// left-to-right order folded with the next leaves).
template <typename T, int R, bool DIAG, bool DELTA, int TILE, bool HEAD32 = false>
__global__ void __launch_bounds__(kThreads)
gram_kernel(const Operands ops, const adasum_tile* __restrict__ tiles, int n_tiles,
            double* __restrict__ partials, const T* __restrict__ start) {
    static_assert(!HEAD32 || (sizeof(T) == 2 && DIAG && !DELTA), "fp32 head: 16-bit leaves, full Gram matrix");
    constexpr int G = Traits<T>::VEC;
    typedef typename Traits<T>::acc_t acc_t;
    constexpr int NP = R * (R - 1) / 2 + (DIAG ? R : 0);
    constexpr int ITERS = TILE / G / kThreads;
    constexpr int U0 = (R >= ADASUM_INFLIGHT) ? 1 : (ADASUM_INFLIGHT / R);   // granule-steps loaded ahead
    constexpr int U = U0 > ITERS ? ITERS : U0;
    static_assert(ITERS % U == 0, "unroll must divide the trip count");

    const int tid = threadIdx.x;
    const int tile_id = static_cast<int>(blockIdx.x % static_cast<unsigned>(n_tiles));
    const int g = static_cast<int>(blockIdx.x / static_cast<unsigned>(n_tiles));
    const adasum_tile t = tiles[tile_id];
    const Split s = split_tile<G>(t);

    const T* x[R];
#pragma unroll
    for (int r = 0; r < R; ++r) x[r] = static_cast<const T*>(operand_ptr<R>(ops, g, r));
    const float* x0 = static_cast<const float*>(operand_ptr<R>(ops, g, 0));   // used with HEAD32 only

    acc_t acc[NP];
#pragma unroll
    for (int e = 0; e < NP; ++e) acc[e] = 0;

    constexpr bool kDot2 = !DELTA && sizeof(T) == 2 && (ADASUM_BF16_DOT2 == 2 || (ADASUM_BF16_DOT2 == 1 && R >= 16));
    auto dot2 = [&](const Granule<T, G>& a, const Granule<T, G>& b, acc_t& sum) {
#pragma unroll
        for (int k = 0; k < Granule<T, G>::NW; ++k) {
            if constexpr (std::is_same<T, bf16_t>::value) {
                sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w[k]),
                                                      __builtin_bit_cast(bf16x2_t, b.w[k]), sum, false);
            } else if constexpr (std::is_same<T, f16_t>::value) {
                sum = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a.w[k]), __builtin_bit_cast(f16x2_t, b.w[k]),
                                             sum, false);
            }
        }
    };
    // raw[0] is not loaded with HEAD32: `head` holds operand 0 instead
    auto consume = [&](const Granule<T, G> (&raw)[R], const Granule<float, G>& head, long long idx) {
        (void)idx;
        (void)head;
        if constexpr (HEAD32) {
            // row 0 (the fp32 operand against everything) in fp32 FMAs; the 16-bit rows as usual
            float v0[G];
            unpack(head, v0);
#pragma unroll
            for (int k = 0; k < G; ++k) acc[0] = fma_t(v0[k], v0[k], acc[0]);
#pragma unroll
            for (int j = 1; j < R; ++j) {
                float vj[G];
                unpack(raw[j], vj);
#pragma unroll
                for (int k = 0; k < G; ++k) acc[j] = fma_t(v0[k], vj[k], acc[j]);
            }
            int e = R;
#pragma unroll
            for (int i = 1; i < R; ++i) {
#pragma unroll
                for (int j = i; j < R; ++j) {
                    if constexpr (kDot2) {
                        dot2(raw[i], raw[j], acc[e]);
                    } else {
                        float vi[G], vj[G];
                        unpack(raw[i], vi);
                        unpack(raw[j], vj);
#pragma unroll
                        for (int k = 0; k < G; ++k) acc[e] = fma_t(vi[k], vj[k], acc[e]);
                    }
                    ++e;
                }
            }
        } else if constexpr (kDot2) {
            // two 16-bit products and the fp32 accumulate in one instruction, straight
            // from the packed words (bf16 x bf16 and f16 x f16 are exact in fp32)
            int e = 0;
#pragma unroll
            for (int i = 0; i < R; ++i) {
#pragma unroll
                for (int j = (DIAG ? i : i + 1); j < R; ++j) {
                    dot2(raw[i], raw[j], acc[e]);
                    ++e;
                }
            }
        } else {
            acc_t v[R][G];
#pragma unroll
            for (int r = 0; r < R; ++r) unpack(raw[r], v[r]);
            if constexpr (DELTA) {
                Granule<T, G> sraw;
                load_raw(sraw, start + idx);
                acc_t sv[G];
                unpack(sraw, sv);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int k = 0; k < G; ++k) v[r][k] -= sv[k];
            }
            int e = 0;
#pragma unroll
            for (int i = 0; i < R; ++i) {
#pragma unroll
                for (int j = (DIAG ? i : i + 1); j < R; ++j) {
#pragma unroll
                    for (int k = 0; k < G; ++k) acc[e] = fma_t(v[i][k], v[j][k], acc[e]);
                    ++e;
                }
            }
        }
    };

    if (s.ng == TILE / G) {
        for (int it0 = 0; it0 < ITERS; it0 += U) {
            Granule<T, G> raw[U][R];
            Granule<float, G> head[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long idx = s.bs + (static_cast<long long>(it0 + u) * kThreads + tid) * G;
                if constexpr (HEAD32) load_raw(head[u], x0 + idx);
#pragma unroll
                for (int r = HEAD32 ? 1 : 0; r < R; ++r) load_raw(raw[u][r], x[r] + idx);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                consume(raw[u], head[u], s.bs + (static_cast<long long>(it0 + u) * kThreads + tid) * G);
        }
    } else {
        for (int j = tid; j < s.ng; j += kThreads) {
            Granule<T, G> raw[R];
            Granule<float, G> head;
            const long long idx = s.bs + static_cast<long long>(j) * G;
            if constexpr (HEAD32) load_raw(head, x0 + idx);
#pragma unroll
            for (int r = HEAD32 ? 1 : 0; r < R; ++r) load_raw(raw[r], x[r] + idx);
            consume(raw, head, idx);
        }
    }
    // Whole granules went through fp32 lanes.  The at most 2*(G-1) elements of a
    // ragged head/tail are multiplied and summed in fp64 by wave 0: layers of a
    // few elements (which are all head/tail) then get exact products, so the
    // scalars of nearly cancelling tiny layers do not lose digits here.
    __shared__ double sh[kThreads / 64][NP];
    __shared__ double sh_edge[NP];
    const int lane = tid & 63, wave = tid >> 6;
    const int nedge = s.nh + s.nt;
    if (nedge > 0 && wave == 0) {
        double v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = 0.0;
        if (lane < nedge) {
            const long long idx = lane < s.nh ? s.start + lane : s.ts + (lane - s.nh);
#pragma unroll
            for (int r = HEAD32 ? 1 : 0; r < R; ++r) v[r] = static_cast<double>(load_elem(x[r] + idx));
            if constexpr (HEAD32) v[0] = static_cast<double>(x0[idx]);
            if constexpr (DELTA) {
                const double sv = static_cast<double>(load_elem(start + idx));
#pragma unroll
                for (int r = 0; r < R; ++r) v[r] -= sv;
            }
        }
        int e = 0;
#pragma unroll
        for (int i = 0; i < R; ++i) {
#pragma unroll
            for (int j = (DIAG ? i : i + 1); j < R; ++j) {
                const double p = wave_sum(v[i] * v[j]);
                if (lane == 0) sh_edge[e] = p;
                ++e;
            }
        }
    }
    // the wave's lanes added in the lanes' precision; lane l ends up with entries l, l + 64, ...
    wave_sum_scatter(acc, lane);
#pragma unroll
    for (int i = 0; i < (NP + 63) / 64; ++i) {
        const int e = lane + 64 * i;
        if (e < NP) sh[wave][e] = static_cast<double>(acc[i]);
    }
    __syncthreads();
    if (tid < NP) {
        double tot = sh[0][tid];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) tot += sh[w][tid];
        if (nedge > 0) tot += sh_edge[tid];
        partials[(static_cast<long long>(g) * n_tiles + tile_id) * NP + tid] = tot;
    }
}

// ---------------------------------------------------------------------------
// Step 2a: sum the per-tile partials of every (group, layer) into a full
// symmetric R x R Gram matrix, in a fixed order.  When !DIAG the diagonal comes
// from the squared norms the previous combine left per (node, tile).
// One workgroup per (group, layer).
// ---------------------------------------------------------------------------
__device__ __forceinline__ double block_sum(double v, double* sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_sum(v);
    __syncthreads();                 // sh may still be read from the previous call
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    double tot = sh[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) tot += sh[w];
    return tot;
}

// The combine pass leaves one squared norm per (node, combine tile); combine
// tiles are short, so a big layer has tens of thousands of them.  This kernel
// sums them to one value per (node, Gram tile): first_in_gram[t] .. [t+1] are the
// combine tiles inside Gram tile t.  One wave per (node, Gram tile).
__global__ void __launch_bounds__(64)
norm_coarsen_kernel(const double* __restrict__ fine, int n_fine_tiles,
                    const int32_t* __restrict__ first_in_gram, int n_gram_tiles,
                    double* __restrict__ coarse) {
    const int t = static_cast<int>(blockIdx.x % static_cast<unsigned>(n_gram_tiles));
    const int node = static_cast<int>(blockIdx.x / static_cast<unsigned>(n_gram_tiles));
    const int b = first_in_gram[t], e = first_in_gram[t + 1];
    const double* row = fine + static_cast<long long>(node) * n_fine_tiles;
    double v = 0.0;
    for (int i = b + static_cast<int>(threadIdx.x); i < e; i += 64) v += row[i];
    v = wave_sum(v);
    if (threadIdx.x == 0) coarse[static_cast<long long>(node) * n_gram_tiles + t] = v;
}

// Entry e of the Gram kernel's order -> (i, j).
template <int R, bool DIAG>
__device__ __forceinline__ void entry_to_ij(int e, int& i, int& j) {
    i = 0;
    int rowlen = DIAG ? R : R - 1;
    while (e >= rowlen) {
        e -= rowlen;
        ++i;
        --rowlen;
    }
    j = (DIAG ? i : i + 1) + e;
}

// The tree's weights from one Gram matrix, computed by one wave (64 lanes): every node of
// the tree is a combination of its leaves, node = sum_p w_p x_p; for two sibling nodes A and
// B the operator of Section 3 needs d = A.B = sum_{p in A, q in B} w_p w_q G_pq, n1 = |A|^2,
// n2 = |B|^2 (quadratic forms whose terms are spread over the lanes and summed in a fixed
// order) and scales A's weights by 1 - d/(2 n1), B's by 1 - d/(2 n2); a zero squared norm
// gives coefficient 1.  G and w live in LDS; r leaves are real, the rest get weight 0.
template <int R>
__device__ __forceinline__ double wave_quadratic(const double* G, const double* w, int a0, int a1, int b0, int b1,
                                                 int lane) {
    const int nb = b1 - b0, n = (a1 - a0) * nb;
    double v = 0.0;
    for (int i = lane; i < n; i += 64) {
        const int p = a0 + i / nb, q = b0 + i % nb;
        v += w[p] * w[q] * G[p * R + q];
    }
    return wave_sum(v);
}

template <int R>
__device__ __forceinline__ void wave_merge(const double* G, double* w, int a0, int a1, int b0, int b1, int lane) {
    const double n1 = wave_quadratic<R>(G, w, a0, a1, a0, a1, lane);
    const double n2 = wave_quadratic<R>(G, w, b0, b1, b0, b1, lane);
    const double d = wave_quadratic<R>(G, w, a0, a1, b0, b1, lane);
    const double ca = n1 > 0.0 ? 1.0 - d / (2.0 * n1) : 1.0;
    const double cb = n2 > 0.0 ? 1.0 - d / (2.0 * n2) : 1.0;
    if (lane >= a0 && lane < a1) w[lane] *= ca;
    if (lane >= b0 && lane < b1) w[lane] *= cb;
}

template <int R>
__device__ __forceinline__ void wave_tree_weights(const double* G, double* w, int r, int order, int lane) {
    if (lane < R) w[lane] = lane < r ? 1.0 : 0.0;
    if (order == ADASUM_ORDER_LINEAR) {
        for (int k = 1; k < r; ++k) wave_merge<R>(G, w, 0, k, k, k + 1, lane);
        return;
    }
    // the halving tree over r leaves, deepest nodes first: children before parents
    int levels = 0;
    while ((1 << levels) < r) ++levels;
    for (int d = levels - 1; d >= 0; --d) {
        for (int j = 0; j < (1 << d); ++j) {
            int lo, hi;
            leaf_range(r, d, j, lo, hi);
            if (hi - lo >= 2) {
                const int mid = lo + (hi - lo) / 2;
                wave_merge<R>(G, w, lo, mid, mid, hi, lane);
            }
        }
    }
}

// The same walk by a whole workgroup of NW waves (the wide first pass: 63 merges of up to 32 x 32 terms
// are slow one after the other): the nodes of one depth are independent, so their 3 quadratic forms
// each are spread over the waves, then every leaf takes its node's coefficient.  Tree order only.
// Every thread of the workgroup must call it; q is LDS scratch of 3 * R / 2 doubles.
template <int R, int NW>
__device__ __forceinline__ void block_tree_weights(const double* G, double* w, double* q, int r) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < R) w[tid] = tid < r ? 1.0 : 0.0;
    int levels = 0;
    while ((1 << levels) < r) ++levels;
    for (int d = levels - 1; d >= 0; --d) {
        __syncthreads();
        const int nodes = 1 << d;
        for (int job = wave; job < 3 * nodes; job += NW) {
            const int j = job / 3, what = job - 3 * j;
            int lo, hi;
            leaf_range(r, d, j, lo, hi);
            const int mid = lo + (hi - lo) / 2;
            double v = 0.0;
            if (hi - lo >= 2)
                v = what == 0   ? wave_quadratic<R>(G, w, lo, mid, lo, mid, lane)
                    : what == 1 ? wave_quadratic<R>(G, w, mid, hi, mid, hi, lane)
                                : wave_quadratic<R>(G, w, lo, mid, mid, hi, lane);
            if (lane == 0) q[job] = v;
        }
        __syncthreads();
        if (tid < r) {
            // the node of this depth that holds leaf tid: walk down from the root
            int lo = 0, hi = r, j = 0;
            for (int b = 0; b < d; ++b) {
                const int mid = lo + (hi - lo) / 2;
                j = 2 * j + (tid >= mid ? 1 : 0);
                if (tid >= mid) lo = mid; else hi = mid;
            }
            if (hi - lo >= 2) {
                const int mid = lo + (hi - lo) / 2;
                const double n1 = q[3 * j], n2 = q[3 * j + 1], dd = q[3 * j + 2];
                const double ca = n1 > 0.0 ? 1.0 - dd / (2.0 * n1) : 1.0;
                const double cb = n2 > 0.0 ? 1.0 - dd / (2.0 * n2) : 1.0;
                w[tid] *= tid < mid ? ca : cb;
            }
        }
    }
    __syncthreads();
}

// One workgroup per (group, layer).  When !DIAG the diagonal comes from the
// coarsened squared norms normparts[(group * R + i) * n_tiles + tile].
// Threads of a finish workgroup: enough rows of entries side by side to keep many loads in
// flight (radix 16 has 136 entries per tile row).
constexpr int finish_threads(int R) { return R >= 16 ? 1024 : kThreads; }

template <int R, bool DIAG>
__global__ void __launch_bounds__(finish_threads(R))
gram_finish_kernel(const double* __restrict__ partials, const double* __restrict__ normparts,
                   const int32_t* __restrict__ layer_tile_begin, int n_tiles, int n_layers,
                   double* __restrict__ gram, double* __restrict__ weights, int order, int K_leaves, int depth) {
    constexpr int NP = R * (R - 1) / 2 + (DIAG ? R : 0);
    constexpr int THREADS = finish_threads(R);
    constexpr int NW = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l = static_cast<int>(blockIdx.x % static_cast<unsigned>(n_layers));
    const int g = static_cast<int>(blockIdx.x / static_cast<unsigned>(n_layers));
    const int tb = layer_tile_begin[l], te = layer_tile_begin[l + 1];
    double* out = gram + (static_cast<long long>(g) * n_layers + l) * (R * R);
    __shared__ double shG[R * R];
    __shared__ double shW[R];

    // partials[(group * n_tiles + tile) * NP + entry]: the layer's tiles form one contiguous run
    // of NP-entry rows.  Thread (row, e) adds entry e of the tiles row, row + ROWS, ... (kAhead of
    // them in flight together); consecutive threads read consecutive addresses.  The ROWS sums of
    // an entry are then added in a fixed order.
    constexpr int ROWS = THREADS / NP;   // tiles handled side by side (NP <= 136)
    constexpr int kAhead = 16;   // loads in flight per thread (one workgroup sums all tiles of a layer)
    static_assert(ROWS >= 1, "more entries than threads");
    __shared__ double shP[ROWS * NP];
    {
        const int row = static_cast<int>(threadIdx.x) / NP, e = static_cast<int>(threadIdx.x) % NP;
        if (row < ROWS) {
            double v = 0.0;
            const double* base = partials + static_cast<long long>(g) * n_tiles * NP + e;
            for (int t0 = tb + row; t0 < te; t0 += ROWS * kAhead) {
                // branch-free so that the loads of a round are issued together: a tile past the
                // end re-reads the layer's last tile and its value is dropped
                double x[kAhead];
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int t = t0 + u * ROWS;
                    x[u] = base[static_cast<long long>(t < te ? t : te - 1) * NP];
                }
#pragma unroll
                for (int u = 0; u < kAhead; ++u) v += (t0 + u * ROWS < te) ? x[u] : 0.0;
            }
            shP[row * NP + e] = v;
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < NP; e += THREADS) {
        double tot = shP[e];
#pragma unroll
        for (int k = 1; k < ROWS; ++k) tot += shP[k * NP + e];
        int i, j;
        entry_to_ij<R, DIAG>(e, i, j);
        out[i * R + j] = tot;
        out[j * R + i] = tot;
        shG[i * R + j] = tot;
        shG[j * R + i] = tot;
    }
    if (!DIAG) {
        for (int i = wave; i < R; i += NW) {
            const double* row = normparts + (static_cast<long long>(g) * R + i) * n_tiles;
            double v = 0.0;
            for (int t = tb + lane; t < te; t += 64) v += row[t];
            v = wave_sum(v);
            if (lane == 0) {
                out[i * R + i] = v;
                shG[i * R + i] = v;
            }
        }
    }
    // Step 2b in the same launch: the weights of this (group, layer), by wave 0
    if (weights != nullptr) {
        __syncthreads();
        if (wave == 0) {
            int r = R;
            if (K_leaves > 0) {
                int lo, hi;
                leaf_range(K_leaves, depth, g, lo, hi);
                r = hi - lo;
            }
            wave_tree_weights<R>(shG, shW, r, order, lane);
            if (lane < R) weights[(static_cast<long long>(g) * n_layers + l) * R + lane] = shW[lane];
        }
    }
}

// ---------------------------------------------------------------------------
// Step 2b on its own (the step entry point): Gram matrices -> weights of the tree over R
// leaves, one wave per (group, layer) item, the same routine the finish kernel runs.
// ---------------------------------------------------------------------------
template <int R>
__global__ void __launch_bounds__(64)
weights_kernel(const double* __restrict__ gram, long long n_items, int order, int n_layers, int K_leaves,
               int depth, double* __restrict__ weights) {
    __shared__ double shG[R * R];
    __shared__ double shW[R];
    const long long item = blockIdx.x;
    const int lane = threadIdx.x;
    if (item >= n_items) return;
    for (int i = lane; i < R * R; i += 64) shG[i] = gram[item * (R * R) + i];
    __builtin_amdgcn_wave_barrier();
    // leaves this group really holds (its first r operands; the rest is padding)
    int r = R;
    if (K_leaves > 0) {
        int lo, hi;
        leaf_range(K_leaves, depth, static_cast<int>(item / n_layers), lo, hi);
        r = hi - lo;
    }
    wave_tree_weights<R>(shG, shW, r, order, lane);
    if (lane < R) weights[item * R + lane] = shW[lane];
}

// The R weights of a (group, layer) item, or ones without a table: one branch, so that the loads are
// issued together.
template <int R, typename A>
__device__ __forceinline__ void load_weights(const double* __restrict__ wp, double (&wd)[R], A (&w)[R]) {
    if (wp != nullptr) {
#pragma unroll
        for (int r = 0; r < R; ++r) wd[r] = wp[r];
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) wd[r] = 1.0;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) w[r] = static_cast<A>(wd[r]);
}

// ---------------------------------------------------------------------------
// Step 3: out = sum_r w_r x_r per element, squared norm of the result per tile.
// One workgroup per combine tile: combine_threads(R) granules of 16 input bytes, i.e. one
// 16-byte load per lane and operand, then the workgroup ends.  Short-lived
// workgroups that walk memory in launch order keep the mixed read/write stream
// close to sequential, worth 10-20 % of bandwidth over long-lived workgroups.
// Sixteen 16-bit operands (combine_pairs_operands): 32 granules per tile and two operands per
// load instruction, so that the wave ends after 8 loads and one store.
// normparts[group * n_tiles + tile].  weights == nullptr: unit weights.
// ---------------------------------------------------------------------------
// HEAD32: operand 0 is stored as fp32 while the others are 16-bit (left-to-right order).
template <typename TI, typename TO, int R, bool SUB, bool HEAD32 = false>
__global__ void __launch_bounds__(combine_threads(R))
combine_kernel(const Operands ops, const Outputs outs, const adasum_tile* __restrict__ tiles,
               int n_tiles, int n_layers, const double* __restrict__ weights,
               double* __restrict__ normparts, const TI* __restrict__ sub_in, const TO* add_out) {
    static_assert(!HEAD32 || (sizeof(TI) == 2 && !SUB), "fp32 head: 16-bit leaves, no delta form");
    constexpr int G = 16 / (int)sizeof(TI);   // tile capacity is THREADS * G
    constexpr int THREADS = combine_threads(R);
    typedef typename Traits<TI>::acc_t acc_t;     // fp64 storage is combined in fp64
    typedef typename Traits<TO>::acc_t out_acc_t; // what the stored value is rounded from
    // Non-temporal stores pay off except where the output is half of the traffic
    // and every lane issues two of them (bf16 pair -> fp32): measured, 13.4 vs 16.4 ms.
    constexpr bool NTS = !(sizeof(TI) == 2 && sizeof(TO) == 4 && R <= 2);
    constexpr bool PAIR = combine_pairs_operands(sizeof(TI), R);

    // grid: (tile, group), tiles fastest -- a group's tiles are walked in memory order
    const int tid = threadIdx.x;
    const int tile_id = static_cast<int>(blockIdx.x);
    const int g = static_cast<int>(blockIdx.y);
    const TI* x[R];
#pragma unroll
    for (int r = 0; r < R; ++r) x[r] = static_cast<const TI*>(operand_ptr<R>(ops, g, r));
    const float* x0 = static_cast<const float*>(operand_ptr<R>(ops, g, 0));   // used with HEAD32 only
    const adasum_tile t = tiles[tile_id];
    const Split s = split_tile<G>(t);
    TO* out = reinterpret_cast<TO*>(outs.base + static_cast<long long>(g) * outs.stride * outs.slot_bytes);
    const double* wp = weights ? weights + (static_cast<long long>(g) * n_layers + t.layer) * R : nullptr;

    acc_t nacc = 0;
    // fp64 weights as computed; the streaming body uses them rounded to fp32
    // (fetched after the operand loads are in flight)
    double wd[R];
    acc_t w[R];
    if constexpr (PAIR) {
        // Two operands per load instruction: lanes 0-31 hold the tile's granules of the operands of one
        // parity, lanes 32-63 of the other.  Each half sums what it holds, the halves exchange the four
        // columns the other one stores, and half h stores columns 4 h .. 4 h + 3 of its granule.
        constexpr int H = G / 2;
        constexpr int R0 = HEAD32 ? 1 : 0;            // operands from R0 on are paired
        constexpr int NL = (R - R0 + 1) / 2;          // loads per lane
        const int half = tid >> 5, c = tid & 31;
        const bool upper = half != 0;
        const bool active = c < s.ng;
        const long long idx = s.bs + static_cast<long long>(c) * G;
        Granule<TI, G> raw[NL];
        Granule<float, H> head;
        if (active) {
            if constexpr (HEAD32) load_raw(head, x0 + idx + H * half);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                // (an odd count leaves the last operand to the lower half; the upper half's copy is not used)
                const int r = R0 + 2 * i, r1 = r + 1 < R ? r + 1 : r;
                load_raw(raw[i], (upper ? x[r1] : x[r]) + idx);
            }
        }
        load_weights<R>(wp, wd, w);
        acc_t z[G];
#pragma unroll
        for (int k = 0; k < G; ++k) z[k] = 0;
        if (active) {
            acc_t sv[G];
            if constexpr (SUB) {
                Granule<TI, G> sraw;
                load_raw(sraw, sub_in + idx);
                unpack(sraw, sv);
            }
            if constexpr (HEAD32) {
                acc_t hv[H];
                unpack(head, hv);
#pragma unroll
                for (int k = 0; k < H; ++k) {
                    const acc_t pz = w[0] * hv[k];
                    z[k] = upper ? static_cast<acc_t>(0) : pz;
                    z[H + k] = upper ? pz : static_cast<acc_t>(0);
                }
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int r = R0 + 2 * i, r1 = r + 1 < R ? r + 1 : r;
                const bool both = r + 1 < R;
                const acc_t ws = upper ? w[r1] : w[r];
                acc_t v[G];
                unpack(raw[i], v);
                if (both || !upper) {
#pragma unroll
                    for (int k = 0; k < G; ++k) {
                        const acc_t e = SUB ? v[k] - sv[k] : v[k];
                        z[k] = (i == 0 && !HEAD32) ? ws * e : fma_t(ws, e, z[k]);
                    }
                }
            }
        }
        acc_t mine[H];
#pragma unroll
        for (int k = 0; k < H; ++k) {
            const acc_t send = upper ? z[k] : z[H + k];
            const acc_t keep = upper ? z[H + k] : z[k];
            mine[k] = keep + __shfl_xor(send, 32, 64);
        }
        if (active) {
#pragma unroll
            for (int k = 0; k < H; ++k) nacc = fma_t(mine[k], mine[k], nacc);
            if (add_out != nullptr) {
                Granule<TO, H> araw;
                load_raw(araw, add_out + idx + H * half);
                acc_t av[H];
                unpack(araw, av);
#pragma unroll
                for (int k = 0; k < H; ++k) mine[k] += av[k];
            }
            store_granule<NTS>(out + idx + H * half, mine);
        }
    } else {
    const long long idx = s.bs + static_cast<long long>(tid) * G;
    Granule<TI, G> raw[R];
    Granule<float, G> head;
    if (tid < s.ng) {
        if constexpr (HEAD32) load_raw(head, x0 + idx);
#pragma unroll
        for (int r = HEAD32 ? 1 : 0; r < R; ++r) load_raw(raw[r], x[r] + idx);
    }

    load_weights<R>(wp, wd, w);

    // Section 4.1's delta form: with SUB the operands are x_r - sub_in (the parameters
    // before the local step); with add_out the stored result is add_out + z.  The
    // squared norm is that of z either way.
    if (tid < s.ng) {
        acc_t sv[G];
        if constexpr (SUB) {
            Granule<TI, G> sraw;
            load_raw(sraw, sub_in + idx);
            unpack(sraw, sv);
        }
        acc_t z[G];
        {
            acc_t v[G];
            if constexpr (HEAD32) unpack(head, v);
            else unpack(raw[0], v);
#pragma unroll
            for (int k = 0; k < G; ++k) z[k] = w[0] * (SUB ? v[k] - sv[k] : v[k]);
        }
#pragma unroll
        for (int r = 1; r < R; ++r) {
            acc_t v[G];
            unpack(raw[r], v);
#pragma unroll
            for (int k = 0; k < G; ++k) z[k] = fma_t(w[r], SUB ? v[k] - sv[k] : v[k], z[k]);
        }
#pragma unroll
        for (int k = 0; k < G; ++k) nacc = fma_t(z[k], z[k], nacc);
        if (add_out != nullptr) {
            Granule<TO, G> araw;
            load_raw(araw, add_out + idx);
            acc_t av[G];
            unpack(araw, av);
#pragma unroll
            for (int k = 0; k < G; ++k) z[k] += av[k];
        }
        store_granule<NTS>(out + idx, z);
    }
    }

    // ragged head/tail elements: fp64 arithmetic, one rounding at the store
    const int lane = tid & 63, wave = tid >> 6;
    const int nedge = s.nh + s.nt;
    double enorm = 0.0;
    if (nedge > 0 && wave == 0) {
        if (lane < nedge) {
            const long long idx = lane < s.nh ? s.start + lane : s.ts + (lane - s.nh);
            const double sd = SUB ? static_cast<double>(load_elem(sub_in + idx)) : 0.0;
            double first;
            if constexpr (HEAD32) first = static_cast<double>(x0[idx]);
            else first = static_cast<double>(load_elem(x[0] + idx));
            double z = wd[0] * (first - sd);
#pragma unroll
            for (int r = 1; r < R; ++r)
                z = __builtin_fma(wd[r], static_cast<double>(load_elem(x[r] + idx)) - sd, z);
            const out_acc_t zs = static_cast<out_acc_t>(z);
            enorm = static_cast<double>(zs) * static_cast<double>(zs);
            if (add_out != nullptr) z += static_cast<double>(load_elem(add_out + idx));
            store_elem(out + idx, static_cast<out_acc_t>(z));
        }
        if (normparts != nullptr) enorm = wave_sum(enorm);
    }

    if (normparts != nullptr) {
        __shared__ double sh[THREADS / 64];
        const acc_t ws = wave_sum(nacc);
        if (lane == 0) sh[wave] = static_cast<double>(ws);
        __syncthreads();
        if (tid == 0) {
            double tot = sh[0];
#pragma unroll
            for (int k = 1; k < THREADS / 64; ++k) tot += sh[k];
            if (nedge > 0) tot += enorm;
            normparts[static_cast<long long>(g) * n_tiles + tile_id] = tot;
        }
    }
}

// ---------------------------------------------------------------------------
// Step 3 for two sibling pairs at once (radix 2 with fuse_siblings): the recursion of Section 3.4
// taken one level ahead.  Workgroup (tile, j) reads the tile of operands A, B (group 2j) and C, D
// (group 2j+1), writes P = a A + b B and Q = c C + d D, and leaves |P|^2, |Q|^2 and P.Q of the
// tile, so the level above -- whose operands are exactly P and Q -- needs no pass over them
// before its own combine.  Tile capacity: 256 lanes x one 16-byte load per operand.
// normparts[(2j | 2j+1) * n_tiles + tile], dotparts[j * n_tiles + tile].
// ---------------------------------------------------------------------------
template <typename TI, typename TO>
__global__ void __launch_bounds__(combine_threads(2))
combine_siblings_kernel(const Operands ops, const Outputs outs, const adasum_tile* __restrict__ tiles, int n_tiles,
                        int n_layers, const double* __restrict__ weights, double* __restrict__ normparts,
                        double* __restrict__ dotparts) {
    constexpr int G = 16 / (int)sizeof(TI);
    constexpr int THREADS = combine_threads(2);
    typedef typename Traits<TI>::acc_t acc_t;
    typedef typename Traits<TO>::acc_t out_acc_t;
    // plain stores where half of the traffic is written (16-bit leaves -> fp32 nodes), as in the pair
    // kernel; measured on the K = 64 BERT-Large case: 16.5 ms against 18.1 ms with non-temporal ones
    constexpr bool NTS = !(sizeof(TI) == 2 && sizeof(TO) == 4);

    const int tid = threadIdx.x;
    const unsigned v = blockIdx.x;
    const int tile_id = static_cast<int>(v % static_cast<unsigned>(n_tiles));
    const int j = static_cast<int>(v / static_cast<unsigned>(n_tiles));
    const adasum_tile t = tiles[tile_id];
    const Split s = split_tile<G>(t);

    const TI* x[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) x[r] = static_cast<const TI*>(ops.pack[4 * j + r]);
    TO* out[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
        out[h] = reinterpret_cast<TO*>(outs.base + static_cast<long long>(2 * j + h) * outs.stride * outs.slot_bytes);

    const long long idx = s.bs + static_cast<long long>(tid) * G;
    Granule<TI, G> raw[4];
    if (tid < s.ng) {
#pragma unroll
        for (int r = 0; r < 4; ++r) load_raw(raw[r], x[r] + idx);
    }
    // weights[(group * n_layers + layer) * 2 + operand], groups 2j and 2j+1
    double wd[4];
    acc_t w[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        wd[r] = weights[(static_cast<long long>(2 * j + (r >> 1)) * n_layers + t.layer) * 2 + (r & 1)];
        w[r] = static_cast<acc_t>(wd[r]);
    }

    acc_t acc[3] = {0, 0, 0};   // |P|^2, |Q|^2, P.Q
    if (tid < s.ng) {
        acc_t z[2][G];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            acc_t a[G], b[G];
            unpack(raw[2 * h], a);
            unpack(raw[2 * h + 1], b);
#pragma unroll
            for (int k = 0; k < G; ++k) z[h][k] = fma_t(w[2 * h + 1], b[k], w[2 * h] * a[k]);
        }
#pragma unroll
        for (int k = 0; k < G; ++k) {
            acc[0] = fma_t(z[0][k], z[0][k], acc[0]);
            acc[1] = fma_t(z[1][k], z[1][k], acc[1]);
            acc[2] = fma_t(z[0][k], z[1][k], acc[2]);
        }
        store_granule<NTS>(out[0] + idx, z[0]);
        store_granule<NTS>(out[1] + idx, z[1]);
    }

    // ragged head/tail elements: fp64 arithmetic, one rounding at the store
    const int lane = tid & 63, wave = tid >> 6;
    const int nedge = s.nh + s.nt;
    double edge[3] = {0.0, 0.0, 0.0};
    if (nedge > 0 && wave == 0) {
        if (lane < nedge) {
            const long long e = lane < s.nh ? s.start + lane : s.ts + (lane - s.nh);
            double zs[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const double z = __builtin_fma(wd[2 * h + 1], static_cast<double>(load_elem(x[2 * h + 1] + e)),
                                               wd[2 * h] * static_cast<double>(load_elem(x[2 * h] + e)));
                const out_acc_t stored = static_cast<out_acc_t>(z);
                zs[h] = static_cast<double>(stored);
                store_elem(out[h] + e, stored);
            }
            edge[0] = zs[0] * zs[0];
            edge[1] = zs[1] * zs[1];
            edge[2] = zs[0] * zs[1];
        }
#pragma unroll
        for (int q = 0; q < 3; ++q) edge[q] = wave_sum(edge[q]);
    }

    __shared__ double sh[3][THREADS / 64];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        const acc_t ws = wave_sum(acc[q]);
        if (lane == 0) sh[q][wave] = static_cast<double>(ws);
    }
    __syncthreads();
    if (tid < 3) {
        double tot = sh[tid][0];
#pragma unroll
        for (int k = 1; k < THREADS / 64; ++k) tot += sh[tid][k];
        // (threads 0..2 are lanes of wave 0, every lane of which holds the edge sums)
        if (nedge > 0) tot += tid == 0 ? edge[0] : (tid == 1 ? edge[1] : edge[2]);
        if (tid < 2) normparts[static_cast<long long>(2 * j + tid) * n_tiles + tile_id] = tot;
        else dotparts[static_cast<long long>(j) * n_tiles + tile_id] = tot;
    }
}

// ---------------------------------------------------------------------------
// Step 3 of a pass that feeds the next one.  Workgroup (tile, s) has R2 waves; wave w combines
// group s * R2 + w for the tile exactly as combine_kernel does (one 16-byte load per lane and
// operand or pair of operands, fp64 edges), then the waves put what they wrote into LDS and wave w forms, for every
// sibling b >= w, the dot product of its node with b's over the tile (b = w: the squared norm).
// Those R2 (R2 + 1) / 2 sums are the tile's share of the next pass's Gram matrix, in the Gram
// pass's entry order: nextparts[(s * n_tiles + tile) * NP2 + entry].  The next pass starts from
// them and reads its operands only once, in its own combine.
// ---------------------------------------------------------------------------
template <typename TI, typename TO, int R, int R2>
__global__ void __launch_bounds__(kFeedLanes * R2)
combine_feed_kernel(const Operands ops, const Outputs outs, const adasum_tile* __restrict__ tiles, int n_tiles,
                    int n_layers, const double* __restrict__ weights, double* __restrict__ nextparts) {
    constexpr int G = 16 / (int)sizeof(TI);
    constexpr int NP2 = R2 * (R2 + 1) / 2;
    typedef typename Traits<TI>::acc_t acc_t;
    typedef typename Traits<TO>::acc_t out_acc_t;
    static_assert(std::is_same<acc_t, out_acc_t>::value, "the nodes of a pass that is not the last have the node type");
    constexpr bool NTS = !(sizeof(TI) == 2 && sizeof(TO) == 4 && R <= 2);   // as combine_kernel
    constexpr bool PAIR = combine_pairs_operands(sizeof(TI), R);

    const int lane = threadIdx.x & 63;
    // the wave's number, as a scalar: the group's operand pointers and weights then live in scalar
    // registers, as in combine_kernel (60 vector registers fewer, one more wave per SIMD)
    const int w = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    // grid: (tile, set of R2 sibling groups), tiles fastest
    const int tile_id = static_cast<int>(blockIdx.x);
    const int super = static_cast<int>(blockIdx.y);
    const int g = super * R2 + w;
    const TI* x[R];
#pragma unroll
    for (int r = 0; r < R; ++r) x[r] = static_cast<const TI*>(operand_ptr<R>(ops, g, r));
    const adasum_tile t = tiles[tile_id];
    const Split s = split_tile<G>(t);
    TO* out = reinterpret_cast<TO*>(outs.base + static_cast<long long>(g) * outs.stride * outs.slot_bytes);

    // what a lane keeps of the node it wrote: its granule, or with paired operands (as in combine_kernel)
    // the half of it that the lane stored
    constexpr int NK = PAIR ? G / 2 : G;
    __shared__ acc_t sh[R2][NK][kFeedLanes];
    __shared__ double sh_edge[R2][kFeedLanes];
    double wd[R];
    acc_t wt[R];
    acc_t z[NK];
    if constexpr (PAIR) {
        constexpr int NL = R / 2;
        const int half = lane >> 5, c = lane & 31;
        const bool upper = half != 0;
        const bool active = c < s.ng;
        const long long idx = s.bs + static_cast<long long>(c) * G;
        Granule<TI, G> raw[NL];
        if (active) {
#pragma unroll
            for (int i = 0; i < NL; ++i) load_raw(raw[i], (upper ? x[2 * i + 1] : x[2 * i]) + idx);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            wd[r] = weights[(static_cast<long long>(g) * n_layers + t.layer) * R + r];
            wt[r] = static_cast<acc_t>(wd[r]);
        }
        acc_t part[G];
#pragma unroll
        for (int k = 0; k < G; ++k) part[k] = 0;
        if (active) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const acc_t ws = upper ? wt[2 * i + 1] : wt[2 * i];
                acc_t a[G];
                unpack(raw[i], a);
#pragma unroll
                for (int k = 0; k < G; ++k) part[k] = i == 0 ? ws * a[k] : fma_t(ws, a[k], part[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < NK; ++k) {
            const acc_t send = upper ? part[k] : part[NK + k];
            const acc_t keep = upper ? part[NK + k] : part[k];
            z[k] = keep + __shfl_xor(send, 32, 64);
        }
        if (active) store_granule<NTS>(out + idx + NK * half, z);
    } else {
        const long long idx = s.bs + static_cast<long long>(lane) * G;
        Granule<TI, G> raw[R];
        if (lane < s.ng) {
#pragma unroll
            for (int r = 0; r < R; ++r) load_raw(raw[r], x[r] + idx);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            wd[r] = weights[(static_cast<long long>(g) * n_layers + t.layer) * R + r];
            wt[r] = static_cast<acc_t>(wd[r]);
        }
#pragma unroll
        for (int k = 0; k < G; ++k) z[k] = 0;
        if (lane < s.ng) {
            {
                acc_t a[G];
                unpack(raw[0], a);
#pragma unroll
                for (int k = 0; k < G; ++k) z[k] = wt[0] * a[k];
            }
#pragma unroll
            for (int r = 1; r < R; ++r) {
                acc_t a[G];
                unpack(raw[r], a);
#pragma unroll
                for (int k = 0; k < G; ++k) z[k] = fma_t(wt[r], a[k], z[k]);
            }
            store_granule<NTS>(out + idx, z);
        }
    }
#pragma unroll
    for (int k = 0; k < NK; ++k) sh[w][k][lane] = z[k];

    // ragged head/tail elements: fp64 arithmetic, one rounding at the store; the stored value goes
    // into the sums
    const int nedge = s.nh + s.nt;
    double ze = 0.0;
    if (nedge > 0) {
        if (lane < nedge) {
            const long long e = lane < s.nh ? s.start + lane : s.ts + (lane - s.nh);
            double acc = wd[0] * static_cast<double>(load_elem(x[0] + e));
#pragma unroll
            for (int r = 1; r < R; ++r) acc = __builtin_fma(wd[r], static_cast<double>(load_elem(x[r] + e)), acc);
            const out_acc_t stored = static_cast<out_acc_t>(acc);
            store_elem(out + e, stored);
            ze = static_cast<double>(stored);
        }
        sh_edge[w][lane] = ze;
    }
    __syncthreads();

    // entry (i, j), i <= j, of the Gram pass's order with the diagonal: i * R2 - i (i - 1) / 2 + (j - i)
    double* dst = nextparts + (static_cast<long long>(super) * n_tiles + tile_id) * NP2 + (w * R2 - w * (w - 1) / 2);
    for (int b = w; b < R2; ++b) {
        acc_t acc = 0;
#pragma unroll
        for (int k = 0; k < NK; ++k) acc = fma_t(z[k], sh[b][k][lane], acc);
        double tot = static_cast<double>(wave_sum(acc));
        if (nedge > 0) tot += wave_sum(ze * sh_edge[b][lane]);
        if (lane == 0) dst[b - w] = tot;
    }
}

// rows of NP Gram entries per combine tile -> per Gram tile.  One wave per (row set, Gram tile).  The wave
// holds S = 64 / NP slices of NP lanes (one slice and a loop over the entries when NP > 32): slice s sums
// entry q over every S-th combine tile of the Gram tile, starting at the s-th, then the slices are added
// up in order.  Consecutive lanes read consecutive doubles; the order is fixed.
__global__ void __launch_bounds__(64)
parts_coarsen_kernel(const double* __restrict__ fine, int n_fine_tiles, const int32_t* __restrict__ first_in_gram,
                     int n_gram_tiles, int NP, double* __restrict__ coarse) {
    const int t = static_cast<int>(blockIdx.x % static_cast<unsigned>(n_gram_tiles));
    const int row = static_cast<int>(blockIdx.x / static_cast<unsigned>(n_gram_tiles));
    const int b = first_in_gram[t], e = first_in_gram[t + 1];
    const double* src = fine + static_cast<long long>(row) * n_fine_tiles * NP;
    double* dst = coarse + (static_cast<long long>(row) * n_gram_tiles + t) * NP;
    const int lane = threadIdx.x;
    const int S = NP <= 32 ? 64 / NP : 1;
    __shared__ double sh[64];
    const int slice = lane / NP;                       // (>= S: a lane with nothing to do when S > 1)
    for (int q0 = 0; q0 < NP; q0 += 64) {              // one round unless NP > 64
        const int q = S > 1 ? lane - slice * NP : q0 + lane;
        const bool active = S > 1 ? slice < S : q < NP;
        double v0 = 0.0, v1 = 0.0, v2 = 0.0, v3 = 0.0;   // four chains so that loads overlap; fixed order
        if (active) {
            int i = b + (S > 1 ? slice : 0);
            for (; i + 3 * S < e; i += 4 * S) {
                v0 += src[static_cast<long long>(i) * NP + q];
                v1 += src[static_cast<long long>(i + S) * NP + q];
                v2 += src[static_cast<long long>(i + 2 * S) * NP + q];
                v3 += src[static_cast<long long>(i + 3 * S) * NP + q];
            }
            for (; i < e; i += S) v0 += src[static_cast<long long>(i) * NP + q];
        }
        const double mine = (v0 + v1) + (v2 + v3);
        if (S > 1) {
            sh[lane] = mine;
            __syncthreads();
            if (lane < NP) {
                double tot = sh[lane];
                for (int k = 1; k < S; ++k) tot += sh[k * NP + lane];
                dst[lane] = tot;
            }
        } else if (active) {
            dst[q] = mine;
        }
    }
}

// ---------------------------------------------------------------------------
// Wide first pass (radix 32 and 64, 16-bit leaves): with 528 or 2080 Gram entries per group the
// "partial dot products" step is a dense contraction, G = X X^T over a tile of R rows, more
// multiply-adds per byte than the vector units have at the memory's speed, so it runs on the
// matrix cores.  v_mfma_f32_32x32x16 takes, per lane, eight consecutive 16-bit elements of row
// lane % 32 (k-half lane / 32) for either operand -- the layout a 16-byte load of one row yields
// -- and multiplying a block of rows with itself or with the other block gives a 32 x 32 block
// of G.  R = 64: rows 0..31 are P, rows 32..63 are Q, blocks P P^T, P Q^T, Q Q^T; R = 32: P P^T only.
//
// The elements are cut into as many equal parts as the chip holds workgroups of this kernel (two
// per compute unit; more, of at most 2^20 elements, for very long buffers), and a part into spans at
// the layer boundaries; a workgroup (four waves) takes one part and leaves one set of blocks per span.  (Per fixed-size tile, as the other passes do it,
// the pass would write 24 KB every 8 MB it reads: 0.3 % of the traffic, and yet stores sprinkled
// over a stream of loads cost it 9 % of its speed, 6.9 instead of 6.3 ms on the K = 64 BERT-Large
// case.  With spans the stores are as few as they can be.)
// A span is walked in blocks of R rows x 2048 / R granules (32 KB).  How the rows are read decides
// the speed as well: a wave that fetches 128 bytes of each of 64 rows per step streams at 6.0 TB/s,
// one that fetches 512 bytes or more of 16 rows at 7.0 (measured on the bare access pattern), so
// wave w loads rows w, w + 4, ... of the block, 512 bytes or 1 KB of a row per load instruction,
// one block ahead of the multiplies.  The block goes through LDS (two buffers, one barrier per
// block) to reach the operand layout; every wave then multiplies its quarter of the block's columns
// for all rows.  The products are exact; the matrix cores add the 64 of a wave's quarter in fp32,
// the blocks' sums are added with ordinary fp32 additions (round to nearest), fp64 above the wave.
// partials[(group * n_spans + span) * NPW + (block * 16 + v) * 64 + lane], NPW = blocks * 1024:
// accumulator v of a lane is row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32 of the block.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// A 16-byte streaming load through a pointer that was kept in LDS: such a pointer has lost its
// address space, and a load through it would be a flat one, which counts against the LDS counter
// too and makes every wait for LDS a wait for all of memory.  These pointers are device memory.
typedef const u32x4 __attribute__((address_space(1)))* global_u32x4_ptr;
__device__ __forceinline__ u32x4 stream_load_global(const void* p) {
#if ADASUM_NT_LOAD
    return __builtin_nontemporal_load((global_u32x4_ptr)p);
#else
    return *(global_u32x4_ptr)p;
#endif
}

template <typename T>
__device__ __forceinline__ f32x16_t mfma_rows(const u32x4& a, const u32x4& b, const f32x16_t& c) {
    if constexpr (std::is_same<T, bf16_t>::value)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                       c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b),
                                                      c, 0, 0, 0);
}

template <typename T, int R>
__global__ void __launch_bounds__(kThreads, 2)   // (second figure: waves per SIMD the register budget must allow)
gram_wide_kernel(const Operands ops, const adasum_tile* __restrict__ spans, const int32_t* __restrict__ part_begin,
                 int n_parts, int n_spans, double* __restrict__ partials) {
    static_assert(sizeof(T) == 2 && (R == 32 || R == 64), "16-bit leaves, 32 or 64 rows");
    static_assert(kThreads == 256, "four waves per tile");
    constexpr int G = 8;                          // elements per 16-byte granule
    constexpr int NB = wide_blocks(R);            // 32 x 32 blocks of the matrix a wave accumulates
    constexpr int CH = 2048 / R;                  // granules per row and block: 32 (R = 64) or 64 (R = 32)
    constexpr int RPI = 64 / CH;                  // rows one load instruction covers: 2 or 1
    constexpr int NLD = R / 4 / RPI;              // load instructions per wave and block: 8
    constexpr int KW = CH / 8;                    // 16-element multiply steps per wave and block: 4 or 8
    constexpr int AHEAD = ADASUM_WIDE_AHEAD;      // blocks whose loads are in flight while one is multiplied
    static_assert(AHEAD == 1 || AHEAD == 2, "");
    constexpr int PITCH = CH * 16 + 16;           // bytes per row in LDS (padded: conflict-free operand reads)
    constexpr int BUF = R * PITCH;
    constexpr int NPW = NB * 1024;
    static_assert(NLD == 8 && 2 * BUF >= 4 * NPW * (int)sizeof(float), "LDS is reused for the waves' sums");

    __shared__ __align__(16) unsigned char lds[2 * BUF];
    __shared__ const T* rowptr[R];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int part = static_cast<int>(blockIdx.x % static_cast<unsigned>(n_parts));
    const int g = static_cast<int>(blockIdx.x / static_cast<unsigned>(n_parts));

    if (tid == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) rowptr[r] = static_cast<const T*>(operand_ptr<R>(ops, g, r));
    }
    __syncthreads();

    // what this lane loads: granule `chunk` of rows (lrow + RPI i) * 4 + wave, i = 0 .. NLD - 1
    const int chunk = lane % CH, lrow = lane / CH;
    const int wr = (lrow * 4 + wave) * PITCH + chunk * 16;
    // what it multiplies: row m of P (and of Q), k-half h of the wave's multiply steps
    const int m = lane & 31, h = lane >> 5;
    const int rdP = m * PITCH + (2 * KW * wave + h) * 16;
    const int rdQ = rdP + 32 * PITCH;

    float sum[NB][16];

    auto multiply_add = [&](const u32x4& p, const u32x4& q, f32x16_t (&acc)[NB]) {
        acc[0] = mfma_rows<T>(p, p, acc[0]);
        if constexpr (NB == 3) {
            acc[1] = mfma_rows<T>(p, q, acc[1]);
            acc[2] = mfma_rows<T>(q, q, acc[2]);
        }
    };
    auto flush = [&](f32x16_t (&acc)[NB]) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                sum[b][v] += acc[b][v];
                acc[b][v] = 0.f;
            }
    };

    for (int sp = part_begin[part]; sp < part_begin[part + 1]; ++sp) {   // (uniform: the barriers below match)
        const Split s = split_tile<G>(spans[sp]);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[b][v] = 0.f;
        // Blocks start at multiples of the block length in the fused buffer, so that a lane group's
        // 512 bytes or 1 KB of a row are whole 128-byte lines whatever the layer's offset: the span's
        // granules are numbers g0 .. g0 + ng - 1 of that grid.
        const long long base = s.bs / (CH * G) * (CH * G);
        const int g0 = static_cast<int>((s.bs - base) / G), g1 = g0 + s.ng;
        const int nsteps = s.ng > 0 ? (g1 + CH - 1) / CH : 0;   // the same for every wave
        u32x4 stage[AHEAD][NLD];                      // the loads of AHEAD blocks in flight per wave
        // No branch around a load (the waits between loads and their use are then counted exactly, and
        // younger loads stay in flight): a lane outside the span's granules re-reads the nearest one,
        // and what it fetched is replaced by zeros when it is stored to LDS.
        // (the row pointers are read from LDS every time: eight more registers per lane would spill)
        auto fetch = [&](u32x4 (&into)[NLD], int step) {
            const int gi = step * CH + chunk;
            const long long off = base + static_cast<long long>(gi < g0 ? g0 : gi < g1 ? gi : g1 - 1) * G;
#pragma unroll
            for (int i = 0; i < NLD; ++i) into[i] = stream_load_global(rowptr[(i * RPI + lrow) * 4 + wave] + off);
        };
        auto store_block = [&](unsigned char* buf, const u32x4 (&from)[NLD], int step) {
            const int gi = step * CH + chunk;
            const bool live = gi >= g0 && gi < g1;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                u32x4 v = from[i];
                v.x = live ? v.x : 0u;
                v.y = live ? v.y : 0u;
                v.z = live ? v.z : 0u;
                v.w = live ? v.w : 0u;
                *reinterpret_cast<u32x4*>(buf + wr + i * (RPI * 4 * PITCH)) = v;
            }
        };
        f32x16_t acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

        if (nsteps > 0) {
#pragma unroll
            for (int a = 0; a < AHEAD; ++a) fetch(stage[a], a);
        }
        for (int step0 = 0; step0 < nsteps; step0 += 2) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                // block step0 + a (one past the end multiplies zeros) through buffer a: the buffer's last
                // readers, two blocks back, passed the barrier of the block in between
                unsigned char* buf = lds + a * BUF;
                store_block(buf, stage[a % AHEAD], step0 + a);
                fetch(stage[a % AHEAD], step0 + a + AHEAD);
                __syncthreads();
#pragma unroll
                for (int j = 0; j < KW; ++j) {
                    const u32x4 p = *reinterpret_cast<const u32x4*>(buf + rdP + j * 32);
                    u32x4 q = p;
                    if constexpr (NB == 3) q = *reinterpret_cast<const u32x4*>(buf + rdQ + j * 32);
                    multiply_add(p, q, acc);
                }
                flush(acc);
            }
        }

        // the at most 2 * 7 elements of a ragged head and tail: one more multiply step by wave 0, the
        // elements fetched one by one straight into the operand layout (k = 8 h .. 8 h + 7)
        const int nedge = s.nh + s.nt;
        if (nedge > 0 && wave == 0) {
            unsigned int pw[4] = {0u, 0u, 0u, 0u}, qw[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int e = 8 * h + k;
                if (e < nedge) {
                    const long long idx = e < s.nh ? s.start + e : s.ts + (e - s.nh);
                    pw[k / 2] |= static_cast<unsigned int>(rowptr[m][idx].v) << (16 * (k & 1));
                    if constexpr (NB == 3) qw[k / 2] |= static_cast<unsigned int>(rowptr[32 + m][idx].v) << (16 * (k & 1));
                }
            }
            u32x4 p, q;
            p.x = pw[0]; p.y = pw[1]; p.z = pw[2]; p.w = pw[3];
            q.x = qw[0]; q.y = qw[1]; q.z = qw[2]; q.w = qw[3];
            multiply_add(p, q, acc);
            flush(acc);
        }

        // the four waves' sums go through LDS (the staging area, now free) and are added in a fixed
        // order, in fp64, by all lanes: entry e of wave w sits at w * NPW + e
        float* red = reinterpret_cast<float*>(lds);
        double* out = partials + (static_cast<long long>(g) * n_spans + sp) * NPW;
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave * NPW + (b * 16 + v) * 64 + lane] = sum[b][v];
        __syncthreads();
        for (int e = tid; e < NPW; e += kThreads)
            out[e] = ((static_cast<double>(red[e]) + static_cast<double>(red[NPW + e])) +
                      static_cast<double>(red[2 * NPW + e])) + static_cast<double>(red[3 * NPW + e]);
        __syncthreads();   // (the next span stages into the same memory)
    }
}

// Step 2 after a wide first pass: sums the per-tile blocks of a (group, layer) in a fixed order,
// spreads them into the full R x R matrix and walks the tree (wave_tree_weights).
template <int R>
__global__ void __launch_bounds__(1024)
gram_finish_wide_kernel(const double* __restrict__ partials, const int32_t* __restrict__ layer_tile_begin, int n_tiles,
                        int n_layers, double* __restrict__ gram, double* __restrict__ weights, int order, int K_leaves,
                        int depth) {
    constexpr int NB = wide_blocks(R);
    constexpr int NPW = NB * 1024;
    constexpr int kAhead = 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l = static_cast<int>(blockIdx.x % static_cast<unsigned>(n_layers));
    const int g = static_cast<int>(blockIdx.x / static_cast<unsigned>(n_layers));
    const int tb = layer_tile_begin[l], te = layer_tile_begin[l + 1];
    double* out = gram + (static_cast<long long>(g) * n_layers + l) * (R * R);
    __shared__ double shG[R * R];
    __shared__ double shW[R];

    // thread tid owns accumulator v = tid / 64 of lane tid % 64 in every block; one workgroup sums all
    // tiles of a layer, so it keeps many loads in flight (branch-free: a tile past the end re-reads the
    // layer's last tile and its value is dropped)
    const double* base = partials + static_cast<long long>(g) * n_tiles * NPW + tid;
    double tots[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) tots[b] = 0.0;
    for (int t0 = tb; t0 < te; t0 += kAhead) {
        double x[NB][kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int t = t0 + u;
            const double* row = base + static_cast<long long>(t < te ? t : te - 1) * NPW;
#pragma unroll
            for (int b = 0; b < NB; ++b) x[b][u] = row[b * 1024];
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
#pragma unroll
            for (int b = 0; b < NB; ++b) tots[b] += (t0 + u < te) ? x[b][u] : 0.0;
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const double tot = tots[b];
        const int v = wave, i = 8 * (v / 4) + 4 * (lane / 32) + v % 4, j = lane % 32;
        // block 0: rows and columns 0..31; block 1: rows 0..31 against 32..63; block 2: rows and columns 32..63
        const int row = b == 2 ? 32 + i : i, col = b == 0 ? j : 32 + j;
        shG[row * R + col] = tot;
        out[row * R + col] = tot;
        if (b == 1) {
            shG[col * R + row] = tot;
            out[col * R + row] = tot;
        }
    }
    if (weights != nullptr) {
        __shared__ double shQ[3 * R / 2];
        int r = R;
        if (K_leaves > 0) {
            int lo, hi;
            leaf_range(K_leaves, depth, g, lo, hi);
            r = hi - lo;
        }
        (void)order;   // (a wide pass exists in the tree order only)
        block_tree_weights<R, 16>(shG, shW, shQ, r);
        if (tid < R) weights[(static_cast<long long>(g) * n_layers + l) * R + tid] = shW[tid];
    }
}

// Step 3 after a wide first pass: out = sum_r w_r x_r over R = 32 or 64 16-bit operands, sixteen at a
// time (as many loads in flight per lane as the radix-16 combine has), one 16-byte granule per lane, one
// wave per tile.  normparts[group * n_tiles + tile] (or null).
template <typename TI, typename TO, int R>
__global__ void __launch_bounds__(64)
combine_wide_kernel(const Operands ops, const Outputs outs, const adasum_tile* __restrict__ tiles, int n_tiles,
                    int n_layers, const double* __restrict__ weights, double* __restrict__ normparts) {
    static_assert(sizeof(TI) == 2 && (R == 32 || R == 64), "16-bit leaves, 32 or 64 operands");
    constexpr int G = 8, C = 16;
    typedef typename Traits<TO>::acc_t out_acc_t;
    const int lane = threadIdx.x;
    const int tile_id = static_cast<int>(blockIdx.x);   // grid: (tile, group)
    const int g = static_cast<int>(blockIdx.y);
    const adasum_tile t = tiles[tile_id];
    const Split s = split_tile<G>(t);
    TO* out = reinterpret_cast<TO*>(outs.base + static_cast<long long>(g) * outs.stride * outs.slot_bytes);
    const double* wl = weights + (static_cast<long long>(g) * n_layers + t.layer) * R;
    const long long idx = s.bs + static_cast<long long>(lane) * G;

    float nacc = 0.f;
    if (lane < s.ng) {
        float z[G];
#pragma unroll
        for (int k = 0; k < G; ++k) z[k] = 0.f;
#pragma unroll 1
        for (int c = 0; c < R / C; ++c) {
            Granule<TI, G> raw[C];
#pragma unroll
            for (int r = 0; r < C; ++r) load_raw(raw[r], static_cast<const TI*>(ops.pack[g * R + c * C + r]) + idx);
#pragma unroll
            for (int r = 0; r < C; ++r) {
                const float w = static_cast<float>(wl[c * C + r]);
                float v[G];
                unpack(raw[r], v);
#pragma unroll
                for (int k = 0; k < G; ++k) z[k] = fma_t(w, v[k], z[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < G; ++k) nacc = fma_t(z[k], z[k], nacc);
        store_granule<true>(out + idx, z);
    }
    // ragged head/tail elements: fp64 arithmetic, one rounding at the store
    const int nedge = s.nh + s.nt;
    double enorm = 0.0;
    if (nedge > 0) {
        if (lane < nedge) {
            const long long e = lane < s.nh ? s.start + lane : s.ts + (lane - s.nh);
            double z = 0.0;
#pragma unroll 1
            for (int r = 0; r < R; ++r)
                z = __builtin_fma(wl[r], static_cast<double>(load_elem(static_cast<const TI*>(ops.pack[g * R + r]) + e)), z);
            const out_acc_t zs = static_cast<out_acc_t>(z);
            enorm = static_cast<double>(zs) * static_cast<double>(zs);
            store_elem(out + e, zs);
        }
        if (normparts != nullptr) enorm = wave_sum(enorm);
    }
    if (normparts != nullptr) {
        const float ws = wave_sum(nacc);
        if (lane == 0) normparts[static_cast<long long>(g) * n_tiles + tile_id] = static_cast<double>(ws) + enorm;
    }
}

// ---------------------------------------------------------------------------
// Small layers (at most kSmallLayer elements), by the definition itself: the
// operator of Section 3 applied pair by pair over all K workers in fp64, in the
// order of Section 3.4's recursion, nothing stored in between.
// ---------------------------------------------------------------------------
// compact[(leaf0 + j)][coff + e] = ops.pack[j][start + e] (- delta[start + e]); with
// stash_start also compact[start_row][coff + e] = delta[start + e].
template <typename T>
__global__ void __launch_bounds__(kThreads)
small_gather_kernel(const Operands ops, int n_leaves, int leaf0, const SmallLayer* __restrict__ small,
                    long long small_elems, const T* __restrict__ delta, int stash_start, int start_row,
                    double* __restrict__ compact) {
    const SmallLayer s = small[blockIdx.x];
    const int rows = n_leaves + (stash_start ? 1 : 0);
    for (int i = threadIdx.x; i < rows * s.len; i += kThreads) {
        const int j = i / s.len, e = i - j * s.len;
        const long long idx = s.start + e;
        if (j < n_leaves) {
            double v = static_cast<double>(load_elem(static_cast<const T*>(ops.pack[j]) + idx));
            if (delta != nullptr) v -= static_cast<double>(load_elem(delta + idx));
            compact[static_cast<long long>(leaf0 + j) * small_elems + s.coff + e] = v;
        } else {
            compact[static_cast<long long>(start_row) * small_elems + s.coff + e] =
                static_cast<double>(load_elem(delta + idx));
        }
    }
}

// One lane per element; lanes past the layer's length hold zeros.  A one-element layer needs no
// sums over the lanes (lane 0 has the only products; the other lanes scale their zeros).
__device__ __forceinline__ double small_pair(double a, double b, bool single) {
    const double d = single ? a * b : wave_sum(a * b);
    const double n1 = single ? a * a : wave_sum(a * a);
    const double n2 = single ? b * b : wave_sum(b * b);
    const double ca = n1 > 0.0 ? 1.0 - d / (2.0 * n1) : 1.0;
    const double cb = n2 > 0.0 ? 1.0 - d / (2.0 * n2) : 1.0;
    return ca * a + cb * b;
}

// How many nodes of the halving tree over K leaves end with leaf k (k is their last leaf)?  Walking the
// leaves left to right with a stack of finished sub-trees, that many merges of the two topmost follow
// the push of leaf k.
__device__ __forceinline__ int merges_after_leaf(int K, int k) {
    int a = 0, b = K, count = 0;
    while (b - a >= 2) {
        if (b == k + 1) ++count;
        const int mid = a + (b - a) / 2;
        if (k < mid) b = mid; else a = mid;
    }
    return count;
}

template <typename TO>
__global__ void __launch_bounds__(64)
small_reduce_kernel(const double* __restrict__ compact, int K, const SmallLayer* __restrict__ small,
                    long long small_elems, int order, int add_start, int start_row, TO* out,
                    double* __restrict__ stats) {
    constexpr int kDepth = 34;   // a stack of complete sub-trees of distinct depths: at most log2(K) + 2
    constexpr int kAhead = 8;    // leaves fetched together (the fetches are what takes the time)
    __shared__ double vstack[kDepth][64];
    __shared__ int merges[64];   // per leaf of the current run of 64: merges that follow its push
    const SmallLayer s = small[blockIdx.x];
    const int lane = threadIdx.x;
    const bool live = lane < s.len;
    const bool single = s.len == 1;
    const bool linear = order == ADASUM_ORDER_LINEAR;
    const double* col = compact + s.coff + lane;
    double leafsq = 0.0, r = 0.0;
    int sp = 0;
    for (int k0 = 0; k0 < K; k0 += kAhead) {
        if ((k0 & 63) == 0 && !linear) {
            __syncthreads();
            merges[lane] = k0 + lane < K ? merges_after_leaf(K, k0 + lane) : 0;
            __syncthreads();
        }
        double leaf[kAhead];
        int todo[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            leaf[u] = (live && k0 + u < K) ? col[static_cast<long long>(k0 + u) * small_elems] : 0.0;
            todo[u] = linear ? 0 : merges[(k0 & 63) + u];
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int k = k0 + u;
            if (k >= K) break;
            const double v = leaf[u];
            leafsq += v * v;
            if (linear) {
                r = k == 0 ? v : small_pair(r, v, single);
                continue;
            }
            // tree order: the top of the stack stays in a register; each merge pops one sub-tree
            if (k > 0) vstack[sp++][lane] = r;
            r = v;
            for (int m = 0; m < todo[u]; ++m) r = small_pair(vstack[--sp][lane], r, single);
        }
    }
    // tree order: sp == 0 and r is the root [0, K)
    const double rsq = wave_sum(r * r);
    leafsq = wave_sum(leafsq);
    if (stats != nullptr && lane == 0) {
        stats[2 * s.layer + 0] = rsq;
        stats[2 * s.layer + 1] = leafsq;
    }
    if (live) {
        double z = r;
        if (add_start) z += compact[static_cast<long long>(start_row) * small_elems + s.coff + lane];
        store_elem(out + s.start + lane, static_cast<typename Traits<TO>::acc_t>(z));
    }
}

// ---------------------------------------------------------------------------
// Per-layer statistics helpers (orthogonality metric of Section 3.6).
// ---------------------------------------------------------------------------
// out[l * out_stride] = sum over rows and the tiles of layer l of parts[row][tile]
__global__ void __launch_bounds__(kThreads)
layer_sums_kernel(const double* __restrict__ parts, int n_rows,
                  const int32_t* __restrict__ layer_tile_begin, int n_tiles,
                  double* __restrict__ out, int out_stride) {
    __shared__ double sh[kThreads / 64];
    const int l = blockIdx.x;
    const int tb = layer_tile_begin[l], te = layer_tile_begin[l + 1];
    double v = 0.0;
    for (int r = 0; r < n_rows; ++r) {
        const double* row = parts + static_cast<long long>(r) * n_tiles;
        for (int t = tb + threadIdx.x; t < te; t += kThreads) v += row[t];
    }
    v = block_sum(v, sh);
    if (threadIdx.x == 0) out[static_cast<long long>(l) * out_stride] = v;
}

// out[l * out_stride] (+)= sum over groups of the diagonal entries first_entry.. of gram[group][l], over
// each group's real leaves
__global__ void __launch_bounds__(64)
trace_sums_kernel(const double* __restrict__ gram, int R, int n_groups, int n_layers, int K_leaves, int depth,
                  int first_entry, int accumulate, double* __restrict__ out, int out_stride) {
    const int l = blockIdx.x * 64 + threadIdx.x;
    if (l >= n_layers) return;
    double v = accumulate ? out[static_cast<long long>(l) * out_stride] : 0.0;
    for (int g = 0; g < n_groups; ++g) {
        const double* G = gram + (static_cast<long long>(g) * n_layers + l) * (R * R);
        int r = R;
        if (K_leaves > 0) {
            int lo, hi;
            leaf_range(K_leaves, depth, g, lo, hi);
            r = hi - lo;
        }
        for (int i = first_entry; i < r; ++i) v += G[i * R + i];
    }
    out[static_cast<long long>(l) * out_stride] = v;
}

// ---------------------------------------------------------------------------
// Set-up without allocation: the layer table arrives in kernel arguments and the
// tile tables are built on the device (the twins of build_tiles / index_against /
// find_small_layers on the host).
// ---------------------------------------------------------------------------
constexpr int kOffsetsPerLaunch = 384;
struct OffsetChunk {
    long long v[kOffsetsPerLaunch];
};

__global__ void __launch_bounds__(kOffsetsPerLaunch)
put_offsets_kernel(const OffsetChunk c, int n, long long* __restrict__ dst) {
    const int i = threadIdx.x;
    if (i < n) dst[i] = c.v[i];
}

constexpr int kScanThreads = 1024;

// Exclusive prefix sums of one value per thread over a workgroup of kScanThreads; returns the
// sum of the values of the threads before this one, *total gets the sum over all threads.
__device__ __forceinline__ long long block_exclusive_scan(long long v, long long* sh, long long* total) {
    const int tid = threadIdx.x;
    __syncthreads();   // sh may still be read from a previous scan
    sh[tid] = v;
    __syncthreads();
    for (int d = 1; d < kScanThreads; d <<= 1) {
        const long long add = tid >= d ? sh[tid - d] : 0;
        __syncthreads();
        sh[tid] += add;
        __syncthreads();
    }
    *total = sh[kScanThreads - 1];
    return sh[tid] - v;
}

__device__ __forceinline__ long long tiles_of_layer(long long lo, long long hi, long long cap) {
    return hi > lo ? (hi - 1) / cap - lo / cap + 1 : 0;
}

// layer_begin[l] = tiles of the layers before l; layer_begin[n_layers] = all tiles.  One workgroup:
// every thread takes a run of consecutive layers.
__global__ void __launch_bounds__(kScanThreads)
tile_scan_kernel(const long long* __restrict__ offs, int n_layers, long long cap, int32_t* __restrict__ layer_begin) {
    __shared__ long long sh[kScanThreads];
    const int tid = threadIdx.x;
    const int per = (n_layers + kScanThreads - 1) / kScanThreads;
    const long long first = static_cast<long long>(tid) * per;
    const int l0 = first < n_layers ? static_cast<int>(first) : n_layers;
    const int l1 = first + per < n_layers ? static_cast<int>(first + per) : n_layers;
    long long mine = 0;
    for (int l = l0; l < l1; ++l) mine += tiles_of_layer(offs[l], offs[l + 1], cap);
    long long total;
    long long run = block_exclusive_scan(mine, sh, &total);
    for (int l = l0; l < l1; ++l) {
        layer_begin[l] = static_cast<int32_t>(run);
        run += tiles_of_layer(offs[l], offs[l + 1], cap);
    }
    if (tid == 0) layer_begin[n_layers] = static_cast<int32_t>(total);
}

// Tile t of the table: its layer is the last one whose first tile is at or before t; inside the
// layer the boundaries are the global multiples of the capacity.
__global__ void __launch_bounds__(kThreads)
tile_fill_kernel(const long long* __restrict__ offs, int n_layers, long long cap,
                 const int32_t* __restrict__ layer_begin, int n_tiles, adasum_tile* __restrict__ tiles) {
    const int t = static_cast<int>(blockIdx.x) * kThreads + static_cast<int>(threadIdx.x);
    if (t >= n_tiles) return;
    int lo = 0, hi = n_layers - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) / 2;
        if (layer_begin[mid] <= t) lo = mid;
        else hi = mid - 1;
    }
    const long long a = offs[lo], b = offs[lo + 1];
    const long long j = t - layer_begin[lo];
    const long long s = j == 0 ? a : (a / cap + j) * cap;
    const long long stop = (a / cap + j + 1) * cap;
    adasum_tile r;
    r.start = s;
    r.len = static_cast<int32_t>((stop < b ? stop : b) - s);
    r.layer = lo;
    tiles[t] = r;
}

// A Gram tile starts at its layer's first element or at a global multiple of the Gram capacity,
// which the combine capacity divides: the combine tile that starts there is found by counting.
__global__ void __launch_bounds__(kThreads)
tile_index_kernel(const long long* __restrict__ offs, const adasum_tile* __restrict__ gram_tiles, int n_gram,
                  long long ccap, const int32_t* __restrict__ comb_layer_begin, int n_comb,
                  int32_t* __restrict__ first_in_gram) {
    const int t = static_cast<int>(blockIdx.x) * kThreads + static_cast<int>(threadIdx.x);
    if (t > n_gram) return;
    if (t == n_gram) {
        first_in_gram[t] = n_comb;
        return;
    }
    const adasum_tile g = gram_tiles[t];
    const long long a = offs[g.layer];
    first_in_gram[t] = comb_layer_begin[g.layer] + static_cast<int32_t>(g.start / ccap - a / ccap);
}

// The table of the layers of 1 .. kSmallLayer elements, in layer order, with each one's place in
// a row of the compact copy.  One workgroup, as tile_scan_kernel.
__global__ void __launch_bounds__(kScanThreads)
small_table_kernel(const long long* __restrict__ offs, int n_layers, SmallLayer* __restrict__ small) {
    __shared__ long long sh[kScanThreads];
    const int tid = threadIdx.x;
    const int per = (n_layers + kScanThreads - 1) / kScanThreads;
    const long long first = static_cast<long long>(tid) * per;
    const int l0 = first < n_layers ? static_cast<int>(first) : n_layers;
    const int l1 = first + per < n_layers ? static_cast<int>(first + per) : n_layers;
    long long count = 0, elems = 0;
    for (int l = l0; l < l1; ++l) {
        const long long len = offs[l + 1] - offs[l];
        if (len >= 1 && len <= kSmallLayer) {
            ++count;
            elems += len;
        }
    }
    long long total;
    long long idx = block_exclusive_scan(count, sh, &total);
    long long coff = block_exclusive_scan(elems, sh, &total);
    for (int l = l0; l < l1; ++l) {
        const long long len = offs[l + 1] - offs[l];
        if (len >= 1 && len <= kSmallLayer) {
            SmallLayer s;
            s.start = offs[l];
            s.len = static_cast<int32_t>(len);
            s.layer = l;
            s.coff = static_cast<int32_t>(coff);
            s.pad = 0;
            small[idx] = s;
            ++idx;
            coff += len;
        }
    }
}

inline int check_launch() { return static_cast<int>(hipGetLastError()); }

inline bool grid_fits(long long blocks) { return blocks > 0 && blocks <= 0x7fffffffLL; }
constexpr int kMaxGridY = 65535;   // second grid dimension (groups)

template <typename T, bool DIAG, bool DELTA>
int launch_gram_r(const Operands& ops, const TileSet& gt, int n_groups, int R, double* partials, const void* start,
                  hipStream_t st) {
    const long long blocks = gt.n_tiles * static_cast<long long>(n_groups);
    if (!grid_fits(blocks)) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    const int nt = static_cast<int>(gt.n_tiles);
    const T* s0 = static_cast<const T*>(start);
    if (gt.capacity != kTile && gt.capacity != kTileSmall) return static_cast<int>(hipErrorInvalidValue);
    const bool small = gt.capacity == kTileSmall;
#define ADASUM_GRAM(RR)                                                                               \
    do {                                                                                              \
        if (small)                                                                                    \
            hipLaunchKernelGGL((gram_kernel<T, RR, DIAG, DELTA, kTileSmall>), grid, block, 0, st, ops, \
                               gt.tiles, nt, partials, s0);                                           \
        else                                                                                          \
            hipLaunchKernelGGL((gram_kernel<T, RR, DIAG, DELTA, kTile>), grid, block, 0, st, ops,     \
                               gt.tiles, nt, partials, s0);                                           \
    } while (0)
    switch (R) {
        case 2: ADASUM_GRAM(2); break;
        case 4: ADASUM_GRAM(4); break;
        case 8: ADASUM_GRAM(8); break;
        case 16:
            // 136 fp64 accumulators per lane do not fit the register file
            if constexpr (std::is_same<T, double>::value) return static_cast<int>(hipErrorInvalidValue);
            else ADASUM_GRAM(16);
            break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef ADASUM_GRAM
    return check_launch();
}

template <typename T>
int launch_gram_t(bool diag, const Operands& ops, const TileSet& gt, int n_groups, int R, double* partials,
                  const void* start, hipStream_t st) {
    if (start != nullptr) {
        if (!diag) return static_cast<int>(hipErrorInvalidValue);   // the delta form exists for the leaves only
        return launch_gram_r<T, true, true>(ops, gt, n_groups, R, partials, start, st);
    }
    return diag ? launch_gram_r<T, true, false>(ops, gt, n_groups, R, partials, nullptr, st)
                : launch_gram_r<T, false, false>(ops, gt, n_groups, R, partials, nullptr, st);
}

template <typename TI, typename TO>
int launch_combine_r(const Operands& ops, const Outputs& outs, const TileSet& ct, int n_layers, int n_groups,
                     int R, const double* weights, double* normparts, const void* sub_in, const void* add_out,
                     hipStream_t st) {
    if (!grid_fits(ct.n_tiles) || n_groups < 1 || n_groups > kMaxGridY) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(ct.n_tiles), static_cast<unsigned>(n_groups)), block(combine_threads(R));
    const int nt = static_cast<int>(ct.n_tiles);
#define ADASUM_COMBINE_AS(RR, SUB)                                                                   \
    hipLaunchKernelGGL((combine_kernel<TI, TO, RR, SUB>), grid, block, 0, st, ops, outs, ct.tiles,  \
                       nt, n_layers, weights, normparts, static_cast<const TI*>(sub_in),            \
                       static_cast<const TO*>(add_out))
    // the subtracting form exists where the delta form can use it: the first pass of several
    // (fp32 nodes out) and a single pass (output of the input's type)
    constexpr bool kSubOk = std::is_same<TO, float>::value || std::is_same<TI, TO>::value;
#define ADASUM_COMBINE(RR)                                                                           \
    do {                                                                                             \
        if (sub_in == nullptr) {                                                                     \
            ADASUM_COMBINE_AS(RR, false);                                                            \
        } else if constexpr (kSubOk) {                                                               \
            ADASUM_COMBINE_AS(RR, true);                                                             \
        } else {                                                                                     \
            return static_cast<int>(hipErrorInvalidValue);                                           \
        }                                                                                            \
    } while (0)
    switch (R) {
        case 1: ADASUM_COMBINE(1); break;
        case 2: ADASUM_COMBINE(2); break;
        case 4: ADASUM_COMBINE(4); break;
        case 8: ADASUM_COMBINE(8); break;
        case 16:
            if constexpr (std::is_same<TI, double>::value) return static_cast<int>(hipErrorInvalidValue);
            else ADASUM_COMBINE(16);
            break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef ADASUM_COMBINE_AS
#undef ADASUM_COMBINE
    return check_launch();
}

// Operand 0 stored as fp32, operands 1.. as T (16-bit): one group, the full Gram matrix.
template <typename T>
int launch_gram_head32_t(const Operands& ops, const TileSet& gt, int R, double* partials, hipStream_t st) {
    if (!grid_fits(gt.n_tiles)) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(gt.n_tiles)), block(kThreads);
    const int nt = static_cast<int>(gt.n_tiles);
    if (gt.capacity != kTile && gt.capacity != kTileSmall) return static_cast<int>(hipErrorInvalidValue);
    const bool small = gt.capacity == kTileSmall;
#define ADASUM_GRAM_HEAD32(RR)                                                                              \
    do {                                                                                                    \
        if (small)                                                                                          \
            hipLaunchKernelGGL((gram_kernel<T, RR, true, false, kTileSmall, true>), grid, block, 0, st, ops, \
                               gt.tiles, nt, partials, static_cast<const T*>(nullptr));                     \
        else                                                                                                \
            hipLaunchKernelGGL((gram_kernel<T, RR, true, false, kTile, true>), grid, block, 0, st, ops,     \
                               gt.tiles, nt, partials, static_cast<const T*>(nullptr));                     \
    } while (0)
    switch (R) {
        case 2: ADASUM_GRAM_HEAD32(2); break;
        case 4: ADASUM_GRAM_HEAD32(4); break;
        case 8: ADASUM_GRAM_HEAD32(8); break;
        case 16: ADASUM_GRAM_HEAD32(16); break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef ADASUM_GRAM_HEAD32
    return check_launch();
}

template <typename TI, typename TO>
int launch_combine_head32_r(const Operands& ops, const Outputs& outs, const TileSet& ct, int n_layers, int R,
                            const double* weights, double* normparts, hipStream_t st) {
    if (!grid_fits(ct.n_tiles)) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(ct.n_tiles)), block(combine_threads(R));
    const int nt = static_cast<int>(ct.n_tiles);
#define ADASUM_COMBINE_HEAD32(RR)                                                                           \
    hipLaunchKernelGGL((combine_kernel<TI, TO, RR, false, true>), grid, block, 0, st, ops, outs, ct.tiles,  \
                       nt, n_layers, weights, normparts, static_cast<const TI*>(nullptr),                   \
                       static_cast<const TO*>(nullptr))
    switch (R) {
        case 2: ADASUM_COMBINE_HEAD32(2); break;
        case 4: ADASUM_COMBINE_HEAD32(4); break;
        case 8: ADASUM_COMBINE_HEAD32(8); break;
        case 16: ADASUM_COMBINE_HEAD32(16); break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef ADASUM_COMBINE_HEAD32
    return check_launch();
}

template <typename TI, typename TO>
int launch_combine_siblings_t(const Operands& ops, const Outputs& outs, const TileSet& ct, int n_layers, int n_groups,
                              const double* weights, double* normparts, double* dotparts, hipStream_t st) {
    const long long blocks = ct.n_tiles * static_cast<long long>(n_groups / 2);
    if (!grid_fits(blocks)) return static_cast<int>(hipErrorInvalidConfiguration);
    hipLaunchKernelGGL((combine_siblings_kernel<TI, TO>), dim3(static_cast<unsigned>(blocks)), dim3(combine_threads(2)),
                       0, st, ops, outs, ct.tiles, static_cast<int>(ct.n_tiles), n_layers, weights, normparts, dotparts);
    return check_launch();
}

template <typename TI, typename TO, int R>
int launch_combine_feed_r(const Operands& ops, const Outputs& outs, const TileSet& ct, int n_layers, int n_groups,
                          int R2, const double* weights, double* nextparts, hipStream_t st) {
    if (!grid_fits(ct.n_tiles) || n_groups / R2 > kMaxGridY) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(ct.n_tiles), static_cast<unsigned>(n_groups / R2));
    const int nt = static_cast<int>(ct.n_tiles);
#define ADASUM_FEED(RR2)                                                                                   \
    hipLaunchKernelGGL((combine_feed_kernel<TI, TO, R, RR2>), grid, dim3(kFeedLanes * RR2), 0, st, ops, outs, \
                       ct.tiles, nt, n_layers, weights, nextparts)
    switch (R2) {
        case 2: ADASUM_FEED(2); break;
        case 4: ADASUM_FEED(4); break;
        case 8: ADASUM_FEED(8); break;
        case 16:
            if constexpr (R * 16 <= kMaxPack) ADASUM_FEED(16);
            else return static_cast<int>(hipErrorInvalidValue);
            break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef ADASUM_FEED
    return check_launch();
}

template <typename TI, typename TO>
int launch_combine_feed_t(const Operands& ops, const Outputs& outs, const TileSet& ct, int n_layers, int n_groups,
                          int R, int R2, const double* weights, double* nextparts, hipStream_t st) {
    switch (R) {
        case 2: return launch_combine_feed_r<TI, TO, 2>(ops, outs, ct, n_layers, n_groups, R2, weights, nextparts, st);
        case 4: return launch_combine_feed_r<TI, TO, 4>(ops, outs, ct, n_layers, n_groups, R2, weights, nextparts, st);
        case 8: return launch_combine_feed_r<TI, TO, 8>(ops, outs, ct, n_layers, n_groups, R2, weights, nextparts, st);
        case 16:
            if constexpr (std::is_same<TI, double>::value) return static_cast<int>(hipErrorInvalidValue);
            else return launch_combine_feed_r<TI, TO, 16>(ops, outs, ct, n_layers, n_groups, R2, weights, nextparts, st);
        default: return static_cast<int>(hipErrorInvalidValue);
    }
}

// The wide first pass (gram_wide_kernel and what follows it): 16-bit leaves, R = 32 or 64.
template <typename T>
int launch_gram_wide_t(const Operands& ops, const TileSet& spans, int n_groups, int R, double* partials, hipStream_t st) {
    if (spans.part_begin == nullptr || spans.n_parts < 1) return static_cast<int>(hipErrorInvalidValue);   // not a span table
    const long long blocks = spans.n_parts * static_cast<long long>(n_groups);
    if (!grid_fits(blocks) || n_groups * R > kMaxPack) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    const int ns = static_cast<int>(spans.n_tiles);
    if (R == 64)
        hipLaunchKernelGGL((gram_wide_kernel<T, 64>), grid, block, 0, st, ops, spans.tiles, spans.part_begin, spans.n_parts,
                           ns, partials);
    else if (R == 32)
        hipLaunchKernelGGL((gram_wide_kernel<T, 32>), grid, block, 0, st, ops, spans.tiles, spans.part_begin, spans.n_parts,
                           ns, partials);
    else return static_cast<int>(hipErrorInvalidValue);
    return check_launch();
}

template <typename TI, typename TO>
int launch_combine_wide_t(const Operands& ops, const Outputs& outs, const TileSet& ct, int n_layers, int n_groups, int R,
                          const double* weights, double* normparts, hipStream_t st) {
    if (!grid_fits(ct.n_tiles) || n_groups < 1 || n_groups * R > kMaxPack) return static_cast<int>(hipErrorInvalidConfiguration);
    if (weights == nullptr || ct.capacity != combine_tile_capacity(ADASUM_BF16, R)) return static_cast<int>(hipErrorInvalidValue);
    const dim3 grid(static_cast<unsigned>(ct.n_tiles), static_cast<unsigned>(n_groups)), block(64);
    const int nt = static_cast<int>(ct.n_tiles);
    if (R == 64)
        hipLaunchKernelGGL((combine_wide_kernel<TI, TO, 64>), grid, block, 0, st, ops, outs, ct.tiles, nt, n_layers, weights,
                           normparts);
    else if (R == 32)
        hipLaunchKernelGGL((combine_wide_kernel<TI, TO, 32>), grid, block, 0, st, ops, outs, ct.tiles, nt, n_layers, weights,
                           normparts);
    else return static_cast<int>(hipErrorInvalidValue);
    return check_launch();
}

}  // namespace

int launch_combine_feed(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                        int n_layers, int n_groups, int R, int R2, const double* weights, double* nextparts,
                        void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ct.n_tiles == 0 || n_groups == 0) return 0;
    if (R2 < 2 || n_groups % R2 != 0 || n_groups * R > kMaxPack || weights == nullptr || nextparts == nullptr ||
        ct.capacity != feed_tile_capacity(dtype, R))
        return static_cast<int>(hipErrorInvalidValue);
    // the nodes such a pass writes are never the root: always the node type of the input
    if (dtype == ADASUM_F64 && out_dtype == ADASUM_F64)
        return launch_combine_feed_t<double, double>(ops, out, ct, n_layers, n_groups, R, R2, weights, nextparts, st);
    if (out_dtype != ADASUM_F32) return static_cast<int>(hipErrorInvalidValue);
    if (dtype == ADASUM_BF16)
        return launch_combine_feed_t<bf16_t, float>(ops, out, ct, n_layers, n_groups, R, R2, weights, nextparts, st);
    if (dtype == ADASUM_F16)
        return launch_combine_feed_t<f16_t, float>(ops, out, ct, n_layers, n_groups, R, R2, weights, nextparts, st);
    if (dtype == ADASUM_F32)
        return launch_combine_feed_t<float, float>(ops, out, ct, n_layers, n_groups, R, R2, weights, nextparts, st);
    return static_cast<int>(hipErrorInvalidValue);
}

int launch_parts_coarsen(const double* fine, int n_rows, int NP, const TileSet& ct, const TileSet& gt, double* coarse,
                         void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const long long blocks = static_cast<long long>(n_rows) * gt.n_tiles;
    if (blocks == 0) return 0;
    if (!grid_fits(blocks) || ct.first_in_gram == nullptr || NP < 1) return static_cast<int>(hipErrorInvalidConfiguration);
    hipLaunchKernelGGL(parts_coarsen_kernel, dim3(static_cast<unsigned>(blocks)), dim3(64), 0, st, fine,
                       static_cast<int>(ct.n_tiles), ct.first_in_gram, static_cast<int>(gt.n_tiles), NP, coarse);
    return check_launch();
}

int launch_combine_siblings(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                            int n_layers, int n_groups, const double* weights, double* normparts, double* dotparts,
                            void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ct.n_tiles == 0 || n_groups == 0) return 0;
    if (n_groups % 2 != 0 || 2 * n_groups > kMaxPack || weights == nullptr || normparts == nullptr || dotparts == nullptr ||
        ct.capacity != combine_tile_capacity(dtype, 2))
        return static_cast<int>(hipErrorInvalidValue);
    // the nodes a fused level writes are never the root: always the node type of the input
    if (dtype == ADASUM_F64 && out_dtype == ADASUM_F64)
        return launch_combine_siblings_t<double, double>(ops, out, ct, n_layers, n_groups, weights, normparts, dotparts, st);
    if (out_dtype != ADASUM_F32) return static_cast<int>(hipErrorInvalidValue);
    if (dtype == ADASUM_BF16)
        return launch_combine_siblings_t<bf16_t, float>(ops, out, ct, n_layers, n_groups, weights, normparts, dotparts, st);
    if (dtype == ADASUM_F16)
        return launch_combine_siblings_t<f16_t, float>(ops, out, ct, n_layers, n_groups, weights, normparts, dotparts, st);
    if (dtype == ADASUM_F32)
        return launch_combine_siblings_t<float, float>(ops, out, ct, n_layers, n_groups, weights, normparts, dotparts, st);
    return static_cast<int>(hipErrorInvalidValue);
}

int launch_gram_head32(int dtype, const Operands& ops, const TileSet& gt, int R, double* partials, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (gt.n_tiles == 0) return 0;
    if (dtype == ADASUM_BF16) return launch_gram_head32_t<bf16_t>(ops, gt, R, partials, st);
    if (dtype == ADASUM_F16) return launch_gram_head32_t<f16_t>(ops, gt, R, partials, st);
    return static_cast<int>(hipErrorInvalidValue);
}

int launch_combine_head32(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                          int n_layers, int R, const double* weights, double* normparts, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ct.n_tiles == 0) return 0;
    if (ct.capacity != combine_tile_capacity(dtype, R)) return static_cast<int>(hipErrorInvalidValue);
    if (dtype == ADASUM_BF16 && out_dtype == ADASUM_BF16)
        return launch_combine_head32_r<bf16_t, bf16_t>(ops, out, ct, n_layers, R, weights, normparts, st);
    if (dtype == ADASUM_BF16 && out_dtype == ADASUM_F32)
        return launch_combine_head32_r<bf16_t, float>(ops, out, ct, n_layers, R, weights, normparts, st);
    if (dtype == ADASUM_F16 && out_dtype == ADASUM_F16)
        return launch_combine_head32_r<f16_t, f16_t>(ops, out, ct, n_layers, R, weights, normparts, st);
    if (dtype == ADASUM_F16 && out_dtype == ADASUM_F32)
        return launch_combine_head32_r<f16_t, float>(ops, out, ct, n_layers, R, weights, normparts, st);
    return static_cast<int>(hipErrorInvalidValue);
}

int launch_gram(int dtype, bool diag, const Operands& ops, const TileSet& gt, int n_groups, int R,
                double* partials, const void* delta_start, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (gt.n_tiles == 0 || n_groups == 0) return 0;
    if (wide_radix(R)) {
        // leaves only: the whole matrix, no delta form
        if (!diag || delta_start != nullptr) return static_cast<int>(hipErrorInvalidValue);
        if (dtype == ADASUM_BF16) return launch_gram_wide_t<bf16_t>(ops, gt, n_groups, R, partials, st);
        if (dtype == ADASUM_F16) return launch_gram_wide_t<f16_t>(ops, gt, n_groups, R, partials, st);
        return static_cast<int>(hipErrorInvalidValue);
    }
    if (dtype == ADASUM_BF16) return launch_gram_t<bf16_t>(diag, ops, gt, n_groups, R, partials, delta_start, st);
    if (dtype == ADASUM_F16) return launch_gram_t<f16_t>(diag, ops, gt, n_groups, R, partials, delta_start, st);
    if (dtype == ADASUM_F64) return launch_gram_t<double>(diag, ops, gt, n_groups, R, partials, delta_start, st);
    return launch_gram_t<float>(diag, ops, gt, n_groups, R, partials, delta_start, st);
}

int launch_norm_coarsen(const double* fine, int n_nodes, const TileSet& ct, const TileSet& gt, double* coarse,
                        void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const long long blocks = static_cast<long long>(n_nodes) * gt.n_tiles;
    if (blocks == 0) return 0;
    if (!grid_fits(blocks) || ct.first_in_gram == nullptr) return static_cast<int>(hipErrorInvalidConfiguration);
    hipLaunchKernelGGL(norm_coarsen_kernel, dim3(static_cast<unsigned>(blocks)), dim3(64), 0, st, fine,
                       static_cast<int>(ct.n_tiles), ct.first_in_gram, static_cast<int>(gt.n_tiles), coarse);
    return check_launch();
}

int launch_gram_finish(bool diag, const TileSet& gt, int n_layers, int n_groups, int R,
                       const double* partials, const double* normparts, double* gram, double* weights, int order,
                       int K_leaves, int depth, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const long long blocks = static_cast<long long>(n_groups) * n_layers;
    if (blocks == 0) return 0;
    if (!grid_fits(blocks)) return static_cast<int>(hipErrorInvalidConfiguration);
    const int ngt = static_cast<int>(gt.n_tiles);
    if (wide_radix(R)) {
        if (!diag) return static_cast<int>(hipErrorInvalidValue);
        const dim3 wgrid(static_cast<unsigned>(blocks)), wblock(1024);
        if (R == 64)
            hipLaunchKernelGGL((gram_finish_wide_kernel<64>), wgrid, wblock, 0, st, partials, gt.layer_begin, ngt, n_layers,
                               gram, weights, order, K_leaves, depth);
        else if (R == 32)
            hipLaunchKernelGGL((gram_finish_wide_kernel<32>), wgrid, wblock, 0, st, partials, gt.layer_begin, ngt, n_layers,
                               gram, weights, order, K_leaves, depth);
        else return static_cast<int>(hipErrorInvalidValue);
        return check_launch();
    }
    const dim3 grid(static_cast<unsigned>(blocks)), block(finish_threads(R));
#define ADASUM_FINISH(RR, DD)                                                                      \
    hipLaunchKernelGGL((gram_finish_kernel<RR, DD>), grid, block, 0, st, partials, normparts,      \
                       gt.layer_begin, ngt, n_layers, gram, weights, order, K_leaves, depth)
    switch (R) {
        case 2: if (diag) ADASUM_FINISH(2, true); else ADASUM_FINISH(2, false); break;
        case 4: if (diag) ADASUM_FINISH(4, true); else ADASUM_FINISH(4, false); break;
        case 8: if (diag) ADASUM_FINISH(8, true); else ADASUM_FINISH(8, false); break;
        case 16: if (diag) ADASUM_FINISH(16, true); else ADASUM_FINISH(16, false); break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
#undef ADASUM_FINISH
    return check_launch();
}

int launch_weights(const double* gram, int R, int64_t n_items, int order, int n_layers, int K_leaves, int depth,
                   double* weights, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_items == 0) return 0;
    const long long blocks = n_items;
    if (!grid_fits(blocks)) return static_cast<int>(hipErrorInvalidConfiguration);
    const dim3 grid(static_cast<unsigned>(blocks)), block(64);
    const long long n = n_items;
    const int nl = n_layers > 0 ? n_layers : 1;
    switch (R) {
        case 2: hipLaunchKernelGGL((weights_kernel<2>), grid, block, 0, st, gram, n, order, nl, K_leaves, depth, weights); break;
        case 4: hipLaunchKernelGGL((weights_kernel<4>), grid, block, 0, st, gram, n, order, nl, K_leaves, depth, weights); break;
        case 8: hipLaunchKernelGGL((weights_kernel<8>), grid, block, 0, st, gram, n, order, nl, K_leaves, depth, weights); break;
        case 16: hipLaunchKernelGGL((weights_kernel<16>), grid, block, 0, st, gram, n, order, nl, K_leaves, depth, weights); break;
        case 32: hipLaunchKernelGGL((weights_kernel<32>), grid, block, 0, st, gram, n, order, nl, K_leaves, depth, weights); break;
        case 64: hipLaunchKernelGGL((weights_kernel<64>), grid, block, 0, st, gram, n, order, nl, K_leaves, depth, weights); break;
        default: return static_cast<int>(hipErrorInvalidValue);
    }
    return check_launch();
}

int launch_combine(int dtype, int out_dtype, const Operands& ops, const Outputs& out, const TileSet& ct,
                   int n_layers, int n_groups, int R, const double* weights, double* normparts,
                   const void* sub_in, const void* add_out, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ct.n_tiles == 0 || n_groups == 0) return 0;
    if (wide_radix(R)) {
        // 16-bit leaves into fp32 or their own type; no delta form
        if (sub_in != nullptr || add_out != nullptr) return static_cast<int>(hipErrorInvalidValue);
        if (dtype == ADASUM_BF16 && out_dtype == ADASUM_BF16)
            return launch_combine_wide_t<bf16_t, bf16_t>(ops, out, ct, n_layers, n_groups, R, weights, normparts, st);
        if (dtype == ADASUM_BF16 && out_dtype == ADASUM_F32)
            return launch_combine_wide_t<bf16_t, float>(ops, out, ct, n_layers, n_groups, R, weights, normparts, st);
        if (dtype == ADASUM_F16 && out_dtype == ADASUM_F16)
            return launch_combine_wide_t<f16_t, f16_t>(ops, out, ct, n_layers, n_groups, R, weights, normparts, st);
        if (dtype == ADASUM_F16 && out_dtype == ADASUM_F32)
            return launch_combine_wide_t<f16_t, float>(ops, out, ct, n_layers, n_groups, R, weights, normparts, st);
        return static_cast<int>(hipErrorInvalidValue);
    }
    // (a kernel of another tile capacity would skip part of every tile)
    if (ct.capacity != combine_tile_capacity(dtype, R)) return static_cast<int>(hipErrorInvalidValue);
    // supported pairs: T -> fp32, fp32 -> T, T -> T; fp64 only with itself
    if (dtype == ADASUM_F64 || out_dtype == ADASUM_F64) {
        if (dtype != out_dtype) return static_cast<int>(hipErrorInvalidValue);
        return launch_combine_r<double, double>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
    }
    if (dtype == ADASUM_BF16) {
        if (out_dtype == ADASUM_BF16)
            return launch_combine_r<bf16_t, bf16_t>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
        if (out_dtype == ADASUM_F32)
            return launch_combine_r<bf16_t, float>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
        return static_cast<int>(hipErrorInvalidValue);
    }
    if (dtype == ADASUM_F16) {
        if (out_dtype == ADASUM_F16)
            return launch_combine_r<f16_t, f16_t>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
        if (out_dtype == ADASUM_F32)
            return launch_combine_r<f16_t, float>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
        return static_cast<int>(hipErrorInvalidValue);
    }
    if (out_dtype == ADASUM_BF16)
        return launch_combine_r<float, bf16_t>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
    if (out_dtype == ADASUM_F16)
        return launch_combine_r<float, f16_t>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
    return launch_combine_r<float, float>(ops, out, ct, n_layers, n_groups, R, weights, normparts, sub_in, add_out, st);
}

int launch_layer_sums(const double* parts, int n_rows, const TileSet& t, int n_layers, double* layer_sum,
                      int out_stride, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_layers == 0) return 0;
    hipLaunchKernelGGL(layer_sums_kernel, dim3(n_layers), dim3(kThreads), 0, st, parts, n_rows,
                       t.layer_begin, static_cast<int>(t.n_tiles), layer_sum, out_stride);
    return check_launch();
}

int launch_trace_sums(const double* gram, int R, int n_groups, int n_layers, int K_leaves, int depth,
                      int first_entry, bool accumulate, double* out, int out_stride, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_layers == 0) return 0;
    hipLaunchKernelGGL(trace_sums_kernel, dim3((n_layers + 63) / 64), dim3(64), 0, st, gram, R, n_groups,
                       n_layers, K_leaves, depth, first_entry, accumulate ? 1 : 0, out, out_stride);
    return check_launch();
}

int launch_small_gather(int dtype, const Operands& ops, int n_leaves, int leaf0, const SmallLayer* small,
                        int n_small, int64_t small_elems, const void* delta_start, bool stash_start,
                        int start_row, double* compact, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_small == 0 || n_leaves == 0) return 0;
    if (n_leaves > kMaxPack || (stash_start && delta_start == nullptr)) return static_cast<int>(hipErrorInvalidValue);
    const dim3 grid(static_cast<unsigned>(n_small)), block(kThreads);
    const long long se = small_elems;
    const int stash = stash_start ? 1 : 0;
#define ADASUM_GATHER(T)                                                                              \
    hipLaunchKernelGGL((small_gather_kernel<T>), grid, block, 0, st, ops, n_leaves, leaf0, small, se, \
                       static_cast<const T*>(delta_start), stash, start_row, compact)
    if (dtype == ADASUM_BF16) ADASUM_GATHER(bf16_t);
    else if (dtype == ADASUM_F16) ADASUM_GATHER(f16_t);
    else if (dtype == ADASUM_F64) ADASUM_GATHER(double);
    else ADASUM_GATHER(float);
#undef ADASUM_GATHER
    return check_launch();
}

int launch_small_reduce(int out_dtype, const double* compact, int K, const SmallLayer* small, int n_small,
                        int64_t small_elems, int order, bool add_start, int start_row, void* out, double* stats,
                        void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_small == 0) return 0;
    const dim3 grid(static_cast<unsigned>(n_small)), block(64);
    const long long se = small_elems;
    const int add = add_start ? 1 : 0;
#define ADASUM_SMALL(T)                                                                                 \
    hipLaunchKernelGGL((small_reduce_kernel<T>), grid, block, 0, st, compact, K, small, se, order, add, \
                       start_row, static_cast<T*>(out), stats)
    if (out_dtype == ADASUM_BF16) ADASUM_SMALL(bf16_t);
    else if (out_dtype == ADASUM_F16) ADASUM_SMALL(f16_t);
    else if (out_dtype == ADASUM_F64) ADASUM_SMALL(double);
    else ADASUM_SMALL(float);
#undef ADASUM_SMALL
    return check_launch();
}

int static_scratch(char** base, size_t* bytes) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static char* ptrs[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<int>(e);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mu);
    if (ptrs[dev] == nullptr) {
        // every GPU holds its own copy of the array at its own address
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return static_cast<int>(e);
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return static_cast<int>(hipErrorInvalidSymbol);
        ptrs[dev] = static_cast<char*>(p);
    }
    *base = ptrs[dev];
    *bytes = sizeof(scratch);
    return 0;
}

int launch_put_words(const int64_t* words, size_t n_words, int64_t* d_words, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n = static_cast<int64_t>(n_words);
    for (int64_t i0 = 0; i0 < n; i0 += kOffsetsPerLaunch) {
        const int m = static_cast<int>(std::min<int64_t>(kOffsetsPerLaunch, n - i0));
        OffsetChunk c;
        for (int i = 0; i < kOffsetsPerLaunch; ++i) c.v[i] = i < m ? words[i0 + i] : 0;
        hipLaunchKernelGGL(put_offsets_kernel, dim3(1), dim3(kOffsetsPerLaunch), 0, st, c, m,
                           reinterpret_cast<long long*>(d_words) + i0);
        const int rc = check_launch();
        if (rc != 0) return rc;
    }
    return 0;
}

int launch_put_offsets(const int64_t* layer_offsets, int n_layers, int64_t* d_offsets, void* stream) {
    return launch_put_words(layer_offsets, static_cast<size_t>(n_layers) + 1, d_offsets, stream);
}

int launch_build_tiles(const int64_t* d_offsets, int n_layers, int64_t capacity, int64_t n_tiles,
                       adasum_tile* d_tiles, int32_t* d_layer_begin, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_layers < 1 || capacity < 1 || n_tiles < 0 || n_tiles > 0x7fffffffLL)
        return static_cast<int>(hipErrorInvalidValue);
    const long long* offs = reinterpret_cast<const long long*>(d_offsets);
    hipLaunchKernelGGL(tile_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, offs, n_layers,
                       static_cast<long long>(capacity), d_layer_begin);
    int rc = check_launch();
    if (rc != 0 || n_tiles == 0) return rc;
    const unsigned blocks = static_cast<unsigned>((n_tiles + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(tile_fill_kernel, dim3(blocks), dim3(kThreads), 0, st, offs, n_layers,
                       static_cast<long long>(capacity), d_layer_begin, static_cast<int>(n_tiles), d_tiles);
    return check_launch();
}

int launch_index_tiles(const int64_t* d_offsets, const adasum_tile* d_gram_tiles, int64_t n_gram, int64_t ccap,
                       const int32_t* d_comb_layer_begin, int64_t n_comb, int32_t* d_first_in_gram, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_gram < 0 || n_gram >= 0x7fffffffLL || n_comb < 0 || n_comb > 0x7fffffffLL || ccap < 1)
        return static_cast<int>(hipErrorInvalidValue);
    const unsigned blocks = static_cast<unsigned>((n_gram + 1 + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(tile_index_kernel, dim3(blocks), dim3(kThreads), 0, st,
                       reinterpret_cast<const long long*>(d_offsets), d_gram_tiles, static_cast<int>(n_gram),
                       static_cast<long long>(ccap), d_comb_layer_begin, static_cast<int>(n_comb), d_first_in_gram);
    return check_launch();
}

int launch_build_small(const int64_t* d_offsets, int n_layers, int n_small, SmallLayer* d_small, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_small == 0) return 0;
    if (n_layers < 1) return static_cast<int>(hipErrorInvalidValue);
    hipLaunchKernelGGL(small_table_kernel, dim3(1), dim3(kScanThreads), 0, st,
                       reinterpret_cast<const long long*>(d_offsets), n_layers, d_small);
    return check_launch();
}

const char* kernel_name(const char* kind, int dtype, int out_dtype, int R, bool diag, char* buf, size_t n) {
    auto name = [](int d) {
        return d == ADASUM_BF16 ? "bf16" : d == ADASUM_F16 ? "f16" : d == ADASUM_F64 ? "f64" : "f32";
    };
    const char* in = name(dtype);
    const char* out = name(out_dtype);
    if (std::strcmp(kind, "gram") == 0) {
        std::snprintf(buf, n, "gram<%s,R=%d,%s>", in, R, diag ? "diag" : "offdiag");
    } else if (std::strcmp(kind, "combine") == 0) {
        std::snprintf(buf, n, "combine<%s,%s,R=%d>", in, out, R);
    } else {
        std::snprintf(buf, n, "%s<R=%d>", kind, R);
    }
    return buf;
}

}  // namespace adasum
