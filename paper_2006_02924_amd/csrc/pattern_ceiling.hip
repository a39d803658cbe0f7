// What the memory system gives the combine pass's access pattern, with everything else taken
// away: R streams of bf16 read with one 16-byte non-temporal load per lane and stream, an
// optional fp32 stream written (two 16-byte stores per lane), workgroups that do one such step
// and end, direct indexing (no tile table, no weights table, constant weights), buffers of the
// headline workload's size.  A third variant writes a narrow stream instead (16 bytes per lane,
// as a bf16 result would be): it shows that what a written stream costs does not depend on how
// much is written.  A fourth takes two streams per load instruction (lanes 0-31 one stream, lanes
// 32-63 the next: 512 bytes of each), lets the halves exchange their sums and writes the fp32
// stream with one 16-byte store per lane: the pattern of the library's 16-operand combine of
// 16-bit inputs.  A measuring tool for the roofline discussion: not part of libadasum, shares no
// code with it.
//
//   pattern_ceiling [elements per stream, default 335141888] [repetitions, default 5]
//
// Prints one line per variant: streams, lanes per workgroup, what is written, ms, GB/s moved.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                          \
        }                                                                          \
    } while (0)

typedef unsigned int u4 __attribute__((ext_vector_type(4)));
constexpr int kMaxStreams = 16;
struct Streams {
    const u4* p[kMaxStreams];
};

template <int R, int LANES, int WRITE>   // 0: read only, 1: fp32 stream written, 2: 16-bit stream written
__global__ void __launch_bounds__(LANES) step_kernel(const Streams in, u4* __restrict__ out, float* __restrict__ sink,
                                                     size_t granules) {
    const size_t i = static_cast<size_t>(blockIdx.x) * LANES + threadIdx.x;
    if (i >= granules) return;
    u4 v[R];
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = __builtin_nontemporal_load(in.p[r] + i);
    float z[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) z[k] = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const unsigned w[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
        const float c = 0.25f + 0.01f * r;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            z[2 * k] = __builtin_fmaf(c, __uint_as_float(w[k] << 16), z[2 * k]);
            z[2 * k + 1] = __builtin_fmaf(c, __uint_as_float(w[k] & 0xffff0000u), z[2 * k + 1]);
        }
    }
    if (WRITE == 2) {
        u4 a;
        a.x = __float_as_uint(z[0]) ^ __float_as_uint(z[4]);
        a.y = __float_as_uint(z[1]) ^ __float_as_uint(z[5]);
        a.z = __float_as_uint(z[2]) ^ __float_as_uint(z[6]);
        a.w = __float_as_uint(z[3]) ^ __float_as_uint(z[7]);
        __builtin_nontemporal_store(a, out + i);
    } else if (WRITE == 1) {
        u4 a, b;
        a.x = __float_as_uint(z[0]); a.y = __float_as_uint(z[1]); a.z = __float_as_uint(z[2]); a.w = __float_as_uint(z[3]);
        b.x = __float_as_uint(z[4]); b.y = __float_as_uint(z[5]); b.z = __float_as_uint(z[6]); b.w = __float_as_uint(z[7]);
        __builtin_nontemporal_store(a, out + 2 * i);
        __builtin_nontemporal_store(b, out + 2 * i + 1);
    } else {
        // keep the loads alive without writing anything that matters
        const float acc = z[0] + z[1] + z[2] + z[3] + z[4] + z[5] + z[6] + z[7];
        if (acc == 12345.678f) sink[blockIdx.x] = acc;
    }
}

// Two streams per load instruction: a one-wave workgroup covers 32 granules of R streams with R / 2 loads per lane.
template <int R>
__global__ void __launch_bounds__(64) pair_kernel(const Streams in, u4* __restrict__ out, size_t granules) {
    const int lane = threadIdx.x, half = lane >> 5, c = lane & 31;
    const size_t i = static_cast<size_t>(blockIdx.x) * 32 + c;
    const bool active = i < granules;
    float z[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) z[k] = 0.f;
    if (active) {
        u4 v[R / 2];
#pragma unroll
        for (int j = 0; j < R / 2; ++j) v[j] = __builtin_nontemporal_load((half ? in.p[2 * j + 1] : in.p[2 * j]) + i);
#pragma unroll
        for (int j = 0; j < R / 2; ++j) {
            const unsigned w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            const float cf = 0.25f + 0.01f * (2 * j + half);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                z[2 * k] = __builtin_fmaf(cf, __uint_as_float(w[k] << 16), z[2 * k]);
                z[2 * k + 1] = __builtin_fmaf(cf, __uint_as_float(w[k] & 0xffff0000u), z[2 * k + 1]);
            }
        }
    }
    // half h keeps columns 4 h .. 4 h + 3 of its granule and gets the other half's sums for them
    u4 a;
    unsigned m[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float send = half ? z[k] : z[4 + k];
        const float keep = half ? z[4 + k] : z[k];
        m[k] = __float_as_uint(keep + __shfl_xor(send, 32, 64));
    }
    a.x = m[0]; a.y = m[1]; a.z = m[2]; a.w = m[3];
    if (active) __builtin_nontemporal_store(a, out + 2 * i + half);
}

template <int R>
void run_pairs(const Streams& in, u4* out, size_t granules, int reps) {
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    const unsigned blocks = static_cast<unsigned>((granules + 31) / 32);
    for (int w = 0; w < 2; ++w) hipLaunchKernelGGL((pair_kernel<R>), dim3(blocks), dim3(64), 0, 0, in, out, granules);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int w = 0; w < reps; ++w) hipLaunchKernelGGL((pair_kernel<R>), dim3(blocks), dim3(64), 0, 0, in, out, granules);
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
    CK(hipGetLastError());
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, a, b));
    ms /= reps;
    const double bytes = static_cast<double>(granules) * 16 * R + static_cast<double>(granules) * 32;
    std::printf("streams %2d  lanes %3d  %-18s %8.3f ms  %6.0f GB/s  %5.1f %% of 8 TB/s\n", R, 64, "pairs + fp32 written", ms,
                bytes / ms / 1e6, bytes / ms / 1e6 / 80.0);
    std::fflush(stdout);
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
}

template <int R, int LANES, int WRITE>
void run(const Streams& in, u4* out, float* sink, size_t granules, int reps) {
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    const unsigned blocks = static_cast<unsigned>((granules + LANES - 1) / LANES);
    for (int w = 0; w < 2; ++w)
        hipLaunchKernelGGL((step_kernel<R, LANES, WRITE>), dim3(blocks), dim3(LANES), 0, 0, in, out, sink, granules);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int w = 0; w < reps; ++w)
        hipLaunchKernelGGL((step_kernel<R, LANES, WRITE>), dim3(blocks), dim3(LANES), 0, 0, in, out, sink, granules);
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
    CK(hipGetLastError());
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, a, b));
    ms /= reps;
    const double bytes = static_cast<double>(granules) * 16 * R + static_cast<double>(granules) * (WRITE == 1 ? 32 : WRITE == 2 ? 16 : 0);
    std::printf("streams %2d  lanes %3d  %-18s %8.3f ms  %6.0f GB/s  %5.1f %% of 8 TB/s\n", R, LANES,
                WRITE == 1 ? "read + fp32 written" : WRITE == 2 ? "read + bf16 written" : "read only", ms,
                bytes / ms / 1e6, bytes / ms / 1e6 / 80.0);
    std::fflush(stdout);
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
}

template <int R>
void run_all(const Streams& in, u4* out, float* sink, size_t granules, int reps) {
    run<R, 64, 0>(in, out, sink, granules, reps);
    run<R, 256, 0>(in, out, sink, granules, reps);
    run<R, 64, 1>(in, out, sink, granules, reps);
    run<R, 256, 1>(in, out, sink, granules, reps);
    run<R, 64, 2>(in, out, sink, granules, reps);
    run_pairs<R>(in, out, granules, reps);
}

int main(int argc, char** argv) {
    const size_t n = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 335141888ull;   // bf16 elements per stream
    const int reps = argc > 2 ? std::atoi(argv[2]) : 5;
    if (n < 8 || n > (1ull << 33) || reps < 1 || reps > 1000) {
        std::printf("usage: pattern_ceiling [elements per stream: 8 .. 2^33] [repetitions: 1 .. 1000]\n");
        return 2;
    }
    const size_t granules = n / 8;   // 16-byte pieces per stream
    Streams in;
    for (int r = 0; r < kMaxStreams; ++r) {
        void* p = nullptr;
        CK(hipMalloc(&p, granules * 16));
        // distinct non-trivial bit patterns per stream (bf16 values around 1)
        CK(hipMemset(p, 0x3c + r, granules * 16));
        in.p[r] = static_cast<const u4*>(p);
    }
    u4* out = nullptr;
    CK(hipMalloc(reinterpret_cast<void**>(&out), granules * 32));
    float* sink = nullptr;
    CK(hipMalloc(reinterpret_cast<void**>(&sink), (granules / 64 + 1) * sizeof(float)));
    CK(hipDeviceSynchronize());
    std::printf("%zu bf16 elements per stream (%.2f GB), %d repetitions per line\n", n, granules * 16 / 1e9, reps);
    run_all<2>(in, out, sink, granules, reps);
    run_all<4>(in, out, sink, granules, reps);
    run_all<8>(in, out, sink, granules, reps);
    run_all<16>(in, out, sink, granules, reps);
    for (int r = 0; r < kMaxStreams; ++r) CK(hipFree(const_cast<u4*>(in.p[r])));
    CK(hipFree(out));
    CK(hipFree(sink));
    return 0;
}
