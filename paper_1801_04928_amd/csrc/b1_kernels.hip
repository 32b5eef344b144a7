// Single-sample (B = 1) fp32 kernels: every step is bound by HBM traffic on the N x N matrix
// (one read of w^l forward, one read of w^{l+1} on the delta chain, one write of nabla_w^l), so the
// kernels are organised around coalesced 128-bit accesses, many loads in flight per wave, and
// reduction trees that depend on N alone (results are bit-identical for every launch shape and k).
#include "lf_internal.h"

namespace lf {

namespace {

constexpr int kThreads = 256;            // 4 waves per workgroup
constexpr int kWavesPerWg = kThreads / kWave;

__host__ __device__ constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------------------------------------
// eqs. (z),(a):  a_out[j] = sigma( sum_k W[j][k] a_in[k] + b[j] ),  W is rows x cols
// One wave owns R consecutive rows.  a_in is staged once per workgroup in LDS; a lane walks the row
// in float4 steps of stride 64 lanes, keeps one accumulator per row, and the 64 lane sums are
// combined in a fixed order (row rotations, then the four rows of 16 lanes).
template <int R>
__global__ __launch_bounds__(kThreads) void k_fwd_gemv(const float* __restrict__ W,
                                                       const float* __restrict__ bias,
                                                       const float* __restrict__ a_in,
                                                       float* __restrict__ a_out, int rows, int cols) {
    extern __shared__ v4f s_a[];   // cols/4 float4
    const int nvec = cols >> 2;
    for (int v = threadIdx.x; v < nvec; v += kThreads) s_a[v] = reinterpret_cast<const v4f*>(a_in)[v];
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.x * kWavesPerWg + wave) * R;
    if (row0 >= rows) return;

    const v4f* wrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = min(row0 + r, rows - 1);   // rows past the end repeat the last one; not stored
        wrow[r] = reinterpret_cast<const v4f*>(W + (size_t)row * cols);
    }
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.0f;

    constexpr int U = (R >= 4) ? 2 : (R == 2 ? 4 : 8);   // float4 loads in flight per lane = R*U
    int v = lane;
    for (; v + (U - 1) * kWave < nvec; v += U * kWave) {
        v4f w[U][R];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r) w[u][r] = wrow[r][v + u * kWave];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const v4f a = s_a[v + u * kWave];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                acc[r] = fmaf(w[u][r].x, a.x, acc[r]);
                acc[r] = fmaf(w[u][r].y, a.y, acc[r]);
                acc[r] = fmaf(w[u][r].z, a.z, acc[r]);
                acc[r] = fmaf(w[u][r].w, a.w, acc[r]);
            }
        }
    }
    for (; v < nvec; v += kWave) {
        const v4f a = s_a[v];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const v4f w = wrow[r][v];
            acc[r] = fmaf(w.x, a.x, acc[r]);
            acc[r] = fmaf(w.y, a.y, acc[r]);
            acc[r] = fmaf(w.z, a.z, acc[r]);
            acc[r] = fmaf(w.w, a.w, acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float z = wave_sum(acc[r]);
        if (lane == 0 && row0 + r < rows) a_out[row0 + r] = sigmoidf(z + bias[row0 + r]);
    }
}

// ------------------------------------------------------------------------------------------------
// eq. (bp2), stage 1: partial[p][k] = sum over the rows j of block p of W[j][k] * delta[j]; W is rows x cols.
// A workgroup covers one strip of 256 columns (a lane owns 4 consecutive columns, so each row is read
// as one contiguous 1 KiB segment) and RPW rows per wave; the four waves' sums are added in wave
// order through LDS.
template <int RPW>
__global__ __launch_bounds__(kThreads) void k_chain_partial(const float* __restrict__ W,
                                                            const float* __restrict__ delta,
                                                            float* __restrict__ partial, int rows,
                                                            int cols) {
    __shared__ v4f s_acc[kWavesPerWg][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int col = blockIdx.x * (kWave * 4) + lane * 4;
    const int row_begin = (blockIdx.y * kWavesPerWg + wave) * RPW;
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    if (col < cols) {
        const float* wp = W + (size_t)row_begin * cols + col;
        if (row_begin + RPW <= rows) {
            v4f w[RPW];
#pragma unroll
            for (int r = 0; r < RPW; ++r) w[r] = *reinterpret_cast<const v4f*>(wp + (size_t)r * cols);
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const float d = delta[row_begin + r];
                acc.x = fmaf(w[r].x, d, acc.x);
                acc.y = fmaf(w[r].y, d, acc.y);
                acc.z = fmaf(w[r].z, d, acc.z);
                acc.w = fmaf(w[r].w, d, acc.w);
            }
        } else {
            for (int r = 0; r < RPW && row_begin + r < rows; ++r) {
                const v4f w = *reinterpret_cast<const v4f*>(wp + (size_t)r * cols);
                const float d = delta[row_begin + r];
                acc.x = fmaf(w.x, d, acc.x);
                acc.y = fmaf(w.y, d, acc.y);
                acc.z = fmaf(w.z, d, acc.z);
                acc.w = fmaf(w.w, d, acc.w);
            }
        }
    }
    s_acc[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && col < cols) {
        v4f t = s_acc[0][lane];
#pragma unroll
        for (int q = 1; q < kWavesPerWg; ++q) t += s_acc[q][lane];
        *reinterpret_cast<v4f*>(partial + (size_t)blockIdx.y * cols + col) = t;
    }
}

// eq. (bp2), stage 2: delta_l[k] = (sum_p partial[p][k]) * a_l[k] * (1 - a_l[k]), p in ascending order.
__global__ __launch_bounds__(kThreads) void k_chain_finish(const float* __restrict__ partial,
                                                           const float* __restrict__ a_l,
                                                           float* __restrict__ delta_l, int N, int P) {
    const int k = blockIdx.x * kThreads + threadIdx.x;
    if (k >= N) return;
    float u = 0.0f;
    for (int p = 0; p < P; ++p) u += partial[(size_t)p * N + k];
    const float a = a_l[k];
    delta_l[k] = u * (a * (1.0f - a));
}

// ------------------------------------------------------------------------------------------------
// eqs. (bp3),(bp4):  nabla_b[j] = delta[j];  nabla_w[j][k] = delta[j] * a_prev[k]  (rows x cols).
// Pure store stream.  A wave owns a strip of 256 columns (its a_prev values stay in registers) and
// RW rows, and writes each row segment with one non-temporal 128-bit store per lane.
// SGD: the gradient-descent step fused into the worker -- `nabla_w` and `nabla_b` are then w^l and b^l
// themselves and receive w - eta * nabla_w, b - eta * nabla_b (the gradient entry is rounded to fp32 exactly as
// it would have been stored, then one fused multiply-add); the gradients are not stored.
template <int RW, bool SGD>
__global__ __launch_bounds__(kThreads) void k_grad_outer(const float* __restrict__ delta,
                                                         const float* __restrict__ a_prev,
                                                         float* nabla_w, float* nabla_b, int rows,
                                                         int cols, int nstrips, float eta) {
    const int lane = threadIdx.x & (kWave - 1);
    const int gw = blockIdx.x * kWavesPerWg + (threadIdx.x >> 6);   // global wave index
    const int strip = gw % nstrips;
    const int row0 = (gw / nstrips) * RW;
    if (row0 >= rows) return;
    const int col = strip * (kWave * 4) + lane * 4;
    if (strip == 0) {
        for (int r = lane; r < RW && row0 + r < rows; r += kWave) {
            if constexpr (SGD) nabla_b[row0 + r] = fmaf(-eta, delta[row0 + r], nabla_b[row0 + r]);
            else nabla_b[row0 + r] = delta[row0 + r];
        }
    }
    if (col >= cols) return;
    const v4f a = *reinterpret_cast<const v4f*>(a_prev + col);
    float* out = nabla_w + (size_t)row0 * cols + col;
    if constexpr (SGD) {
        constexpr int U = 8;                          // rows read ahead
#pragma unroll 1
        for (int r0 = 0; r0 < RW; r0 += U) {
            v4f w[U];
#pragma unroll
            for (int u = 0; u < U; ++u)   // rows past the end re-read the last one; not stored
                w[u] = *reinterpret_cast<const v4f*>(out + (size_t)(min(row0 + r0 + u, rows - 1) - row0) * cols);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (row0 + r0 + u >= rows) break;
                const float d = delta[row0 + r0 + u];
                const v4f g = {d * a.x, d * a.y, d * a.z, d * a.w};
                const v4f o = {fmaf(-eta, g.x, w[u].x), fmaf(-eta, g.y, w[u].y), fmaf(-eta, g.z, w[u].z),
                               fmaf(-eta, g.w, w[u].w)};
                *reinterpret_cast<v4f*>(out + (size_t)(r0 + u) * cols) = o;
            }
        }
    } else {
#pragma unroll 4
        for (int r = 0; r < RW; ++r) {
            if (row0 + r >= rows) break;
            const float d = delta[row0 + r];
            const v4f g = {d * a.x, d * a.y, d * a.z, d * a.w};
            __builtin_nontemporal_store(g, reinterpret_cast<v4f*>(out + (size_t)r * cols));
        }
    }
}

// ------------------------------------------------------------------------------------------------
// eq. (bp1): delta_L = (a_L - y) * a_L * (1 - a_L), elementwise, fp32 or bfloat16 storage.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_output_error(const T* __restrict__ a_L,
                                                           const T* __restrict__ y,
                                                           float* __restrict__ delta_L,
                                                           __bf16* __restrict__ delta_bf, size_t count,
                                                           float scale) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= count) return;
    const float a = (float)a_L[i];
    const float d = scale * ((a - (float)y[i]) * (a * (1.0f - a)));
    delta_L[i] = d;
    if (delta_bf) delta_bf[i] = (__bf16)d;
}

int chain_rows_per_wave(int rows) { return rows >= 4096 ? 16 : (rows >= 2048 ? 8 : 4); }

}  // namespace

int chain_partial_blocks(int rows) { return ceil_div(rows, kWavesPerWg * chain_rows_per_wave(rows)); }

hipError_t launch_fwd_gemv_f32(const float* W, const float* b, const float* a_in, float* a_out,
                               int rows, int cols, hipStream_t s) {
    const size_t lds = (size_t)cols * sizeof(float);
    const size_t elems = (size_t)rows * cols;
    if (elems >= (size_t)4096 * 4096) {
        k_fwd_gemv<4><<<ceil_div(rows, kWavesPerWg * 4), kThreads, lds, s>>>(W, b, a_in, a_out, rows, cols);
    } else if (elems >= (size_t)2048 * 2048) {
        k_fwd_gemv<2><<<ceil_div(rows, kWavesPerWg * 2), kThreads, lds, s>>>(W, b, a_in, a_out, rows, cols);
    } else {
        k_fwd_gemv<1><<<ceil_div(rows, kWavesPerWg), kThreads, lds, s>>>(W, b, a_in, a_out, rows, cols);
    }
    return hipGetLastError();
}

hipError_t launch_chain_gemvT_f32(const float* W_next, const float* delta_next, const float* a_l,
                                  float* delta_l, float* partial, int rows, int cols, hipStream_t s) {
    const int rpw = chain_rows_per_wave(rows);
    const int P = chain_partial_blocks(rows);
    const dim3 grid(ceil_div(cols, kWave * 4), P);
    if (rpw == 16) k_chain_partial<16><<<grid, kThreads, 0, s>>>(W_next, delta_next, partial, rows, cols);
    else if (rpw == 8) k_chain_partial<8><<<grid, kThreads, 0, s>>>(W_next, delta_next, partial, rows, cols);
    else k_chain_partial<4><<<grid, kThreads, 0, s>>>(W_next, delta_next, partial, rows, cols);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_chain_finish<<<ceil_div(cols, kThreads), kThreads, 0, s>>>(partial, a_l, delta_l, cols, P);
    return hipGetLastError();
}

hipError_t launch_grad_outer_f32(const float* delta, const float* a_prev, float* nabla_w,
                                 float* nabla_b, int rows, int cols, float sgd_eta, hipStream_t s) {
    const int nstrips = ceil_div(cols, kWave * 4);
    constexpr int RW = 16;
    const int waves = nstrips * ceil_div(rows, RW);
    const int grid = ceil_div(waves, kWavesPerWg);
    if (sgd_eta != 0.0f)
        k_grad_outer<RW, true><<<grid, kThreads, 0, s>>>(delta, a_prev, nabla_w, nabla_b, rows, cols, nstrips,
                                                         sgd_eta);
    else
        k_grad_outer<RW, false><<<grid, kThreads, 0, s>>>(delta, a_prev, nabla_w, nabla_b, rows, cols, nstrips,
                                                          0.0f);
    return hipGetLastError();
}

hipError_t launch_output_error(const void* a_L, const void* y, float* delta_L, void* delta_bf,
                               size_t count, bool bf16, float scale, hipStream_t s) {
    const unsigned grid = (unsigned)((count + kThreads - 1) / kThreads);
    if (bf16)
        k_output_error<__bf16><<<grid, kThreads, 0, s>>>((const __bf16*)a_L, (const __bf16*)y, delta_L,
                                                         (__bf16*)delta_bf, count, scale);
    else
        k_output_error<float><<<grid, kThreads, 0, s>>>((const float*)a_L, (const float*)y, delta_L,
                                                        (__bf16*)delta_bf, count, scale);
    return hipGetLastError();
}

}  // namespace lf
