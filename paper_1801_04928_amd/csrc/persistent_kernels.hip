// Persistent-kernel realisation of the single-sample (B = 1, fp32) pass.
//
// At B = 1 a layer step moves one N x N matrix and the chain has 2(L-1) dependent steps, so for
// N ~ 1K the pass is bound by the latency of whatever separates two steps.  Here one kernel per
// direction stays resident (one workgroup per compute unit, G <= 256 workgroups) and walks all layers;
// consecutive layers are separated by a single exchange through memory, not by a kernel boundary.
//
// Exchange format ("tagged words"): a 64-bit word = (fp32 value, 32-bit tag), written and read with
// relaxed agent-scope 64-bit atomics.  Value and tag arrive together, so a reader that sees the tag it
// expects has the value: no fence, no separate flag.  Tags change with every pass (epoch) and layer,
// so buffers are never cleared between passes.  These words are the per-layer ready flags that feed
// the k workers of section 3.
//
// Ownership: workgroup g owns the index block J_g = [g*RPG, (g+1)*RPG) of every layer.
//   forward  (z),(a): g computes a^l[J_g] from rows J_g of w^l (needs all of a^{l-1}: gathered from the
//                     tagged words the owners published), publishes a^l[J_g].
//   backward (bp2):   g holds delta^{l+1}[J_g], forms the partial column sums of rows J_g of w^{l+1}
//                     (all N columns), publishes them; then gathers, for its columns J_g, the partials
//                     of every workgroup, adds them in workgroup order and applies sigma'.  One
//                     exchange per layer; the sum order depends on (N, G) only.
//   (bp3),(bp4):      layer l belongs to worker (L-l) mod k = the workgroups with g mod k equal to it.
//                     They split its rows, wait for delta^l through its tagged words and stream
//                     nabla_w^l out with non-temporal stores in the gaps of the chain (k >= 2), or in
//                     line before the next chain step (k = 1, the sequential pass).
//
// Every wait is bounded: a poll that exceeds its spin limit raises an abort flag that all loops
// observe, the kernel drains, and the host reports LF_EHIP.
#include "lf_internal.h"
#include "persistent.h"

namespace lf {
namespace {

typedef unsigned long long u64;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr unsigned kSpinLimit = 4u << 20;   // polls before a wait gives up (seconds, not microseconds)

__device__ __forceinline__ u64 ll_pack(float v, unsigned tag) {
    return ((u64)tag << 32) | (u64)__float_as_uint(v);
}
__device__ __forceinline__ void ll_store(u64* p, float v, unsigned tag) {
    __hip_atomic_store(p, ll_pack(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 ll_load(const u64* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ll_tag(u64 w) { return (unsigned)(w >> 32); }
__device__ __forceinline__ float ll_val(u64 w) { return __uint_as_float((unsigned)w); }

// Where a wait gave up: site (1 forward gather, 2 chain gather, 3 gradient wait), layer, workgroup.
__device__ __forceinline__ int abort_code(int site, int l, int g) { return (site << 24) | (l << 10) | g; }

struct Abort {
    int* dev;       // device word, agent scope
    int* host;      // mapped pinned host word (may be null)
    bool dead;
    __device__ void raise(int code) {
        dead = true;
        __hip_atomic_store(dev, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (host) __hip_atomic_store(host, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    __device__ bool seen() {
        if (!dead && __hip_atomic_load(dev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) dead = true;
        return dead;
    }
};

// Poll up to four consecutive tagged words until all carry `tag`.  n in 1..4 words are valid.
__device__ __forceinline__ void ll_wait4(const u64* p, int n, unsigned tag, float out[4], Abort& ab,
                                         int code) {
    out[0] = out[1] = out[2] = out[3] = 0.0f;
    if (n <= 0) return;
    unsigned spin = 0;
    while (!ab.dead) {
        u64 w[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) w[c] = (c < n) ? ll_load(p + c) : 0;
        bool ok = true;
#pragma unroll
        for (int c = 0; c < 4; ++c) ok = ok && (c >= n || ll_tag(w[c]) == tag);
        if (ok) {
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c] = (c < n) ? ll_val(w[c]) : 0.0f;
            return;
        }
        ++spin;
        if (spin > kSpinLimit) { ab.raise(code); return; }
        if ((spin & 255u) == 0u) ab.seen();
    }
}

__device__ __forceinline__ const float* act_ptr(const PersistArgs& A, int l) {
    return l == 1 ? A.a1 : A.a_base + (size_t)(l - 2) * A.a_stride;
}

// ================================================================================================
// forward
// ================================================================================================
// Q = float4 column groups per lane and row (Q*256 >= N); CH = groups fetched per chunk.
template <int Q>
__global__ __launch_bounds__(kThreads) void k_fwd_persistent(const PersistArgs A) {
    constexpr int CH = Q < 16 ? Q : 16;
    constexpr int CPR = Q / CH;   // chunks per row
    __shared__ v4f s_a[Q * 64];
    __shared__ float s_bias[kMaxRowsPerGroup];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, g = blockIdx.x;
    const int N = A.N, L = A.L, RPG = A.RPG, nvec = N >> 2;
    const int RW = (RPG + kWaves - 1) / kWaves;             // rows per wave
    const int wrow0 = g * RPG + wave * RW;                  // first row of this wave
    const int wrow_end = min(min(N, (g + 1) * RPG), wrow0 + RW);
    const int nchunks = RW * CPR;
    Abort ab{A.abort_dev, A.abort_host, false};

    auto load_chunk = [&](v4f (&buf)[CH], const float* W, int ci) {
        const int r = ci / CPR, h = ci % CPR;
        const int row = wrow0 + r;
        const v4f* wp = reinterpret_cast<const v4f*>(W + (size_t)row * N);
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int v = lane + 64 * (h * CH + u);
            buf[u] = (row < wrow_end && v < nvec) ? wp[v] : v4f{0.f, 0.f, 0.f, 0.f};
        }
    };

    v4f cur[CH], nxt[CH];
    load_chunk(cur, A.w[0], 0);
    for (int l = 2; l <= L; ++l) {
        if (t < RPG && g * RPG + t < N) s_bias[t] = A.b[l - 2][g * RPG + t];   // off the critical path
        // gather a^{l-1} into LDS
        if (l == 2) {
            for (int v = t; v < nvec; v += kThreads) s_a[v] = reinterpret_cast<const v4f*>(A.a1)[v];
        } else {
            const u64* src = A.ALL + (size_t)(l - 3) * N;    // words of a^{l-1}
            for (int v = t; v < nvec; v += kThreads) {
                float o[4];
                ll_wait4(src + 4 * v, 4, A.epoch, o, ab, abort_code(1, l, g));
                s_a[v] = v4f{o[0], o[1], o[2], o[3]};
            }
        }
        __syncthreads();
        const float* W = A.w[l - 2];
        const float* Wn = l < L ? A.w[l - 1] : nullptr;
        float* a_out = A.a_base + (size_t)(l - 2) * A.a_stride;
        u64* pub = A.ALL + (size_t)(l - 2) * N;
        float acc = 0.0f;
        for (int ci = 0; ci < nchunks; ++ci) {
            if (ci + 1 < nchunks) load_chunk(nxt, W, ci + 1);
            else if (Wn) load_chunk(nxt, Wn, 0);             // next layer's first chunk, across the exchange
            const int r = ci / CPR, h = ci % CPR;
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int v = lane + 64 * (h * CH + u);
                const v4f a = v < nvec ? s_a[v] : v4f{0.f, 0.f, 0.f, 0.f};
                acc = fmaf(cur[u].x, a.x, acc);
                acc = fmaf(cur[u].y, a.y, acc);
                acc = fmaf(cur[u].z, a.z, acc);
                acc = fmaf(cur[u].w, a.w, acc);
            }
            if (h == CPR - 1) {
                const int row = wrow0 + r;
                const float z = wave_sum(acc);
                if (lane == 0 && row < wrow_end) {
                    const float a = sigmoidf(z + s_bias[row - g * RPG]);
                    a_out[row] = a;
                    if (l < L) ll_store(pub + row, a, A.epoch);
                }
                acc = 0.0f;
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) cur[u] = nxt[u];
        }
        __syncthreads();   // s_a is rewritten by the next layer's gather
    }
}

// ================================================================================================
// backward
// ================================================================================================
// P = float4 column groups per thread (P*1024 >= N).
template <int P>
__global__ __launch_bounds__(kThreads) void k_bwd_persistent(const PersistArgs A) {
    constexpr int RC = P <= 4 ? 4 : 2;     // rows per fetched chunk (RC*P float4 in flight per thread)
    __shared__ float s_delta[kMaxRowsPerGroup];
    __shared__ float s_red[kWaves][kMaxRowsPerGroup];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, g = blockIdx.x;
    const int N = A.N, L = A.L, G = A.G, RPG = A.RPG, k = A.k, nvec = N >> 2;
    const int row0 = g * RPG;
    const int nrows = max(0, min(RPG, N - row0));
    const int nchunks = (RPG + RC - 1) / RC;
    Abort ab{A.abort_dev, A.abort_host, false};

    // ---- gradient jobs of this workgroup: layers l = L - part - m k, rows [jrow_begin, jrow_end)
    const int part = g % k, member = g / k, members = (G - part + k - 1) / k;
    const int RM = (N + members - 1) / members;
    const int jrow_begin = min(N, member * RM), jrow_end = min(N, jrow_begin + RM);
    int job_layer = L - part, job_row = jrow_begin;
    bool ja_loaded = false;
    v4f ja[P];

    // Store up to max_rows rows of pending gradient work whose delta is published.  With `wait`
    // the call blocks (bounded) until the rows are there; otherwise it returns at the first row that
    // is not ready.  Layers above `lowest_ready` have their delta computed by the whole grid.
    auto grad_rows = [&](int max_rows, int lowest_ready, bool wait) {
        while (max_rows > 0 && job_layer >= 2 && job_layer >= lowest_ready && !ab.dead) {
            if (job_row >= jrow_end) {
                job_layer -= k;
                job_row = jrow_begin;
                ja_loaded = false;
                continue;
            }
            if (!ja_loaded) {
                const v4f* ap = reinterpret_cast<const v4f*>(act_ptr(A, job_layer - 1));
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int v = t + kThreads * p;
                    ja[p] = v < nvec ? ap[v] : v4f{0.f, 0.f, 0.f, 0.f};
                }
                ja_loaded = true;
            }
            const int n = min(min(4, max_rows), jrow_end - job_row);
            const u64* dl = A.DLL + (size_t)(job_layer - 2) * N + job_row;
            float d[4];
            if (wait) {
                ll_wait4(dl, n, A.epoch, d, ab, abort_code(3, job_layer, g));
                if (ab.dead) return;
            } else {
                u64 w[4];
                bool ok = true;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    w[c] = c < n ? ll_load(dl + c) : 0;
                    ok = ok && (c >= n || ll_tag(w[c]) == A.epoch);
                    d[c] = ll_val(w[c]);
                }
                if (!ok) return;
            }
            float* gw = A.gw[job_layer - 2] + (size_t)job_row * N;
            float* gb = A.gb[job_layer - 2] + job_row;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (c < n) {
#pragma unroll
                    for (int p = 0; p < P; ++p) {
                        const int v = t + kThreads * p;
                        if (v < nvec) {
                            const v4f o = {d[c] * ja[p].x, d[c] * ja[p].y, d[c] * ja[p].z, d[c] * ja[p].w};
                            __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(gw + (size_t)c * N) + v);
                        }
                    }
                    if (t == 0) gb[c] = d[c];
                }
            }
            job_row += n;
            max_rows -= n;
        }
    };

    auto load_chunk = [&](v4f (&buf)[RC][P], const float* W, int ci) {
#pragma unroll
        for (int rr = 0; rr < RC; ++rr) {
            const int r = ci * RC + rr;
            const v4f* wp = reinterpret_cast<const v4f*>(W + (size_t)(row0 + r) * N);
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int v = t + kThreads * p;
                buf[rr][p] = (r < nrows && v < nvec) ? wp[v] : v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
    };

    v4f cur[RC][P], nxt[RC][P];
    if (L > 2) load_chunk(cur, A.w[L - 2], 0);      // rows J_g of w^L, needed by the first chain step

    // (bp1): delta^L on the owned block
    if (t < nrows) {
        const int j = row0 + t;
        const float a = act_ptr(A, L)[j];
        const float d = (a - A.y[j]) * (a * (1.0f - a));
        s_delta[t] = d;
        A.d_base[(size_t)(L - 2) * A.d_stride + j] = d;
        ll_store(A.DLL + (size_t)(L - 2) * N + j, d, A.epoch);
    }
    __syncthreads();

    for (int l = L - 1; l >= 2; --l) {
        // k = 1: the gradients of layer l+1 sit on the chain, before the step to layer l
        if (k == 1) grad_rows(RPG, l + 1, true);

        const float a_l = t < nrows ? act_ptr(A, l)[row0 + t] : 0.0f;   // for sigma', off the critical path

        // partial column sums over the owned rows of w^{l+1}
        const float* W = A.w[l - 1];
        const float* Wn = l > 2 ? A.w[l - 2] : nullptr;
        v4f acc[P];
#pragma unroll
        for (int p = 0; p < P; ++p) acc[p] = v4f{0.f, 0.f, 0.f, 0.f};
        for (int ci = 0; ci < nchunks; ++ci) {
            if (ci + 1 < nchunks) load_chunk(nxt, W, ci + 1);
            else if (Wn) load_chunk(nxt, Wn, 0);        // next step's first chunk, across the exchange
#pragma unroll
            for (int rr = 0; rr < RC; ++rr) {
                const int r = ci * RC + rr;
                const float d = r < nrows ? s_delta[r] : 0.0f;
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    acc[p].x = fmaf(cur[rr][p].x, d, acc[p].x);
                    acc[p].y = fmaf(cur[rr][p].y, d, acc[p].y);
                    acc[p].z = fmaf(cur[rr][p].z, d, acc[p].z);
                    acc[p].w = fmaf(cur[rr][p].w, d, acc[p].w);
                }
            }
#pragma unroll
            for (int rr = 0; rr < RC; ++rr)
#pragma unroll
                for (int p = 0; p < P; ++p) cur[rr][p] = nxt[rr][p];
        }
        // publish: X[parity][g][column]
        const unsigned tagx = (A.epoch << 13) | (unsigned)l;
        u64* xw = A.X + ((size_t)(l & 1) * G + g) * N;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int v = t + kThreads * p;
            if (v < nvec) {
                ll_store(xw + 4 * v + 0, acc[p].x, tagx);
                ll_store(xw + 4 * v + 1, acc[p].y, tagx);
                ll_store(xw + 4 * v + 2, acc[p].z, tagx);
                ll_store(xw + 4 * v + 3, acc[p].w, tagx);
            }
        }
        // k >= 2: gradient work fills the wait for the other workgroups' partials
        if (k > 1) grad_rows(2 * RPG, l + 1, false);

        // gather the partials of my columns from every workgroup (thread t <-> workgroup t), add them
        const u64* xr = A.X + ((size_t)(l & 1) * G + t) * N + row0;
        for (int i0 = 0; i0 < RPG; i0 += 4) {
            float v[4];
            ll_wait4(xr + i0, t < G ? min(4, nrows - i0) : 0, tagx, v, ab, abort_code(2, l, g));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float s = wave_sum(v[c]);
                if (lane == 0) s_red[wave][i0 + c] = s;
            }
        }
        __syncthreads();
        if (t < nrows) {
            const int j = row0 + t;
            const float u = ((s_red[0][t] + s_red[1][t]) + s_red[2][t]) + s_red[3][t];
            const float d = u * (a_l * (1.0f - a_l));
            s_delta[t] = d;
            A.d_base[(size_t)(l - 2) * A.d_stride + j] = d;
            ll_store(A.DLL + (size_t)(l - 2) * N + j, d, A.epoch);
        }
        __syncthreads();
    }
    // drain: whatever gradient work is left (all of it has its delta on the way)
    grad_rows(0x7fffffff, 2, true);
}

__global__ __launch_bounds__(kThreads) void k_fill_u64(u64* p, size_t n, u64 v) {
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads)
        p[i] = v;
}

}  // namespace

// Every workgroup must own at least one row: a workgroup is throttled by the gather of its own
// columns, and one with nothing to gather would run ahead and overwrite exchange words (two buffers,
// reused every other layer) that slower workgroups have not read yet.
int persistent_groups(int N, int num_cus) {
    int G = (N + 3) / 4;
    if (G > kMaxGroups) G = kMaxGroups;
    if (num_cus > 0 && G > num_cus) G = num_cus;
    if (G < 1) G = 1;
    const int rpg = (N + G - 1) / G;
    return (N + rpg - 1) / rpg;
}

bool persistent_supported(int N) { return N % 4 == 0 && N >= 4 && N <= kMaxPersistentN; }

int persistent_rows_per_group(int N, int G) { return (N + G - 1) / G; }

hipError_t launch_fill_u64(void* p, size_t n_words, unsigned long long v, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    k_fill_u64<<<1024, kThreads, 0, s>>>(static_cast<u64*>(p), n_words, v);
    return hipGetLastError();
}

hipError_t launch_fwd_persistent(const PersistArgs& A, hipStream_t s) {
    const int q = (A.N / 4 + 63) / 64;
    if (q <= 4) k_fwd_persistent<4><<<A.G, kThreads, 0, s>>>(A);
    else if (q <= 8) k_fwd_persistent<8><<<A.G, kThreads, 0, s>>>(A);
    else if (q <= 16) k_fwd_persistent<16><<<A.G, kThreads, 0, s>>>(A);
    else k_fwd_persistent<32><<<A.G, kThreads, 0, s>>>(A);
    return hipGetLastError();
}

hipError_t launch_bwd_persistent(const PersistArgs& A, hipStream_t s) {
    const int p = (A.N / 4 + kThreads - 1) / kThreads;
    if (p <= 1) k_bwd_persistent<1><<<A.G, kThreads, 0, s>>>(A);
    else if (p <= 2) k_bwd_persistent<2><<<A.G, kThreads, 0, s>>>(A);
    else if (p <= 4) k_bwd_persistent<4><<<A.G, kThreads, 0, s>>>(A);
    else k_bwd_persistent<8><<<A.G, kThreads, 0, s>>>(A);
    return hipGetLastError();
}

}  // namespace lf
