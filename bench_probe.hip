// Measurement aid for bench.py, not part of the backpropagation library: plain streaming kernels, the access patterns of the
// single-sample backward pass as plain kernels, and a loop of matrix instructions that
// never leaves the registers, on every compute unit, to show what the matrix cores sustain on this machine
// at the clock they hold under that load (the published peaks are quoted at the maximum clock).
#include <hip/hip_runtime.h>

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;            // 4 waves, one per SIMD
constexpr int kChains = 4;               // independent accumulators per wave

// Each wave keeps kChains independent chains of 32 x 32 x 16 bfloat16 products going.
__global__ __launch_bounds__(kThreads) void k_mfma_loop_bf16(int iters, float* sink) {
    v16f acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.0f;
    v8bf a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(0.001f * (float)((threadIdx.x + e) & 7));
        b[e] = (__bf16)(0.002f * (float)((threadIdx.x + 3 * e) & 7));
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[c][e];
    if (s == 12345.678f) sink[0] = s;     // keeps the loop alive; never true
}

// The same with 32 x 32 x 2 fp32 products.
__global__ __launch_bounds__(kThreads) void k_mfma_loop_f32(int iters, float* sink) {
    v16f acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.0f;
    const float a = 0.001f * (float)(threadIdx.x & 7), b = 0.002f * (float)(threadIdx.x & 5);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[c][e];
    if (s == 12345.678f) sink[0] = s;
}

typedef float v4f __attribute__((ext_vector_type(4)));

// Plain streaming kernels over n float4 vectors, grid-stride, 128-bit accesses: what HBM delivers to kernels
// that only read, only write (non-temporal stores), or do both at once (even workgroups read the first
// buffer, odd workgroups write the second).
__global__ __launch_bounds__(kThreads) void k_stream_read(const v4f* __restrict__ src, size_t n, float* sink) {
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    const size_t stride = (size_t)gridDim.x * kThreads;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {       // four loads in flight per thread
        const v4f a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc += (a + b) + (c + d);
    }
    for (; i < n; i += stride) acc += src[i];
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;   // never true for the zero-filled buffer
}

__global__ __launch_bounds__(kThreads) void k_stream_write(v4f* __restrict__ dst, size_t n) {
    const v4f v = {1.0f, 2.0f, 3.0f, 4.0f};
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
        __builtin_nontemporal_store(v, dst + i);
}

__global__ __launch_bounds__(kThreads) void k_stream_read_write(const v4f* __restrict__ src, v4f* __restrict__ dst,
                                                               size_t n, float* sink) {
    const size_t stride = (size_t)(gridDim.x / 2) * kThreads;
    size_t i = (size_t)(blockIdx.x / 2) * kThreads + threadIdx.x;
    if (blockIdx.x & 1) {
        const v4f v = {1.0f, 2.0f, 3.0f, 4.0f};
        for (; i < n; i += stride) __builtin_nontemporal_store(v, dst + i);
    } else {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        for (; i + 3 * stride < n; i += 4 * stride) {
            const v4f a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
            acc += (a + b) + (c + d);
        }
        for (; i < n; i += stride) acc += src[i];
        if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;
    }
}

// The access patterns of the single-sample backward pass at N = 4096, without its arithmetic and exchanges: 256
// workgroups that read the matrices as column strips of 256 bytes in four row blocks (sixteen 128-bit loads in
// flight per thread), and 256 workgroups that write matrices row by row with non-temporal 128-bit stores.
constexpr int kPatternN = 4096;
__global__ __launch_bounds__(kThreads) void k_strip_read(const float* base, int matrices, int passes, float* sink) {
    constexpr int N = kPatternN, TPS = 16, RPP = kThreads / TPS, STRIPS = N * 4 / 256;
    const int RB = gridDim.x / STRIPS, NR = N / RB;        // (not constants: the loop below is then left rolled, the
    const int strip = blockIdx.x % STRIPS, rb = blockIdx.x / STRIPS;        // faster form by a quarter)
    const int t = threadIdx.x, c = t % TPS, rs = t / TPS;
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    for (int m = 0; m < passes; ++m) {
        const float* W = base + (size_t)(m % matrices) * N * N + (size_t)(rb * NR + rs) * N + strip * 64 + 4 * c;
        for (int r = 0; r < NR; r += RPP * 16) {
            v4f v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load((const v4f*)(W + (size_t)(r + u * RPP) * N));
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += v[u];
        }
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;
}
__global__ __launch_bounds__(kThreads) void k_row_write(float* base, int matrices, int passes) {
    constexpr int N = kPatternN;
    const int t = threadIdx.x, rows = N / gridDim.x;
    for (int m = 0; m < passes; ++m) {
        float* G = base + (size_t)(m % matrices) * N * N;
        for (int row = blockIdx.x * rows; row < (blockIdx.x + 1) * rows; ++row)
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const v4f o = {(float)row, (float)p, 1.f, 2.f};
                __builtin_nontemporal_store(o, (v4f*)(G + (size_t)row * N + 4 * (t + kThreads * p)));
            }
    }
}

}  // namespace

extern "C" {

// The two pattern kernels above, each on a stream of its own: `passes` matrices of 4096 x 4096 floats read from
// src (mode 0), written to dst (mode 1), or both side by side (mode 2); each buffer holds `matrices` of them, used
// in turn.  Synchronous.  Returns the milliseconds from the start of the first to the end of the last kernel, a
// negative number on a bad argument or a HIP error.
double probe_strips_beside_rows(int mode, const float* src, float* dst, int matrices, int passes, float* sink) {
    if (mode < 0 || mode > 2 || matrices < 1 || passes < 1 || !sink || (mode != 1 && !src) || (mode != 0 && !dst)) return -1.0;
    hipStream_t s1 = nullptr, s2 = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr, e2 = nullptr;
    double ms = -1.0;
    if (hipStreamCreate(&s1) == hipSuccess && hipStreamCreate(&s2) == hipSuccess && hipEventCreate(&e0) == hipSuccess &&
        hipEventCreate(&e1) == hipSuccess && hipEventCreate(&e2) == hipSuccess && hipDeviceSynchronize() == hipSuccess) {
        (void)hipEventRecord(e0, s1);
        (void)hipStreamWaitEvent(s2, e0, 0);
        if (mode != 1) k_strip_read<<<256, kThreads, 0, s1>>>(src, matrices, passes, sink);
        if (mode != 0) k_row_write<<<256, kThreads, 0, s2>>>(dst, matrices, passes);
        (void)hipEventRecord(e2, s2);
        (void)hipStreamWaitEvent(s1, e2, 0);
        (void)hipEventRecord(e1, s1);
        float f = 0.0f;
        if (hipEventSynchronize(e1) == hipSuccess && hipGetLastError() == hipSuccess &&
            hipEventElapsedTime(&f, e0, e1) == hipSuccess)
            ms = f;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e2) (void)hipEventDestroy(e2);
    if (s1) (void)hipStreamDestroy(s1);
    if (s2) (void)hipStreamDestroy(s2);
    return ms;
}

// Enqueue one streaming kernel over `bytes` bytes (a multiple of 16) of each buffer it uses.  mode 0: read src;
// 1: write dst; 2: read src and write dst at once.  groups: workgroups of 256 threads (even for mode 2).
// Returns the bytes the launch moves, 0 on a bad argument or a failed launch.
double probe_stream(int mode, int groups, const void* src, void* dst, size_t bytes, float* sink, void* hip_stream) {
    if (groups < 2 || groups > (1 << 20) || bytes < 16 || bytes % 16 != 0 || !sink) return 0.0;
    if ((mode == 0 || mode == 2) && !src) return 0.0;
    if ((mode == 1 || mode == 2) && !dst) return 0.0;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const size_t n = bytes / 16;
    if (mode == 0) k_stream_read<<<groups, kThreads, 0, s>>>(static_cast<const v4f*>(src), n, sink);
    else if (mode == 1) k_stream_write<<<groups, kThreads, 0, s>>>(static_cast<v4f*>(dst), n);
    else if (mode == 2) k_stream_read_write<<<groups & ~1, kThreads, 0, s>>>(static_cast<const v4f*>(src),
                                                                             static_cast<v4f*>(dst), n, sink);
    else return 0.0;
    if (hipGetLastError() != hipSuccess) return 0.0;
    return mode == 2 ? 2.0 * (double)bytes : (double)bytes;
}

// Enqueue the loop on `hip_stream`: `groups` workgroups of four waves, each wave issuing 4 * iters matrix
// instructions.  bf16 != 0: 32 x 32 x 16 bfloat16 (32768 flops each), else 32 x 32 x 2 fp32 (4096 flops each).
// sink: one float of device memory (never written).  Returns the flops the launch performs, 0 on a bad
// argument or a failed launch.
double probe_mfma_loop(int bf16, int groups, int iters, float* sink, void* hip_stream) {
    if (groups < 1 || groups > 65536 || iters < 1 || !sink) return 0.0;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (bf16) k_mfma_loop_bf16<<<groups, kThreads, 0, s>>>(iters, sink);
    else k_mfma_loop_f32<<<groups, kThreads, 0, s>>>(iters, sink);
    if (hipGetLastError() != hipSuccess) return 0.0;
    const double per = bf16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    return per * kChains * (double)iters * 4.0 * (double)groups;
}

}  // extern "C"
