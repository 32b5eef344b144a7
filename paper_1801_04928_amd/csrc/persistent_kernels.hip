// Persistent-kernel realisation of the single-sample (B = 1, fp32) pass.
//
// At B = 1 a layer step moves one N x N matrix and the chain has 2(L-1) dependent steps, so for
// N ~ 1K the pass is bound by the latency of whatever separates two steps.  Here one kernel per
// direction stays resident and walks all layers; consecutive layers are separated by one exchange
// through memory (an all-gather of N values), not by a kernel boundary.
//
// Exchange format ("tagged words"): a 64-bit word = (fp32 value, 32-bit tag), written and read with
// relaxed agent-scope 64-bit atomics.  Value and tag arrive together, so a reader that sees the tag it
// expects has the value: no fence, no separate flag.  The tag is the launch's epoch (a per-workgroup launch
// count kept in device memory), so buffers are never cleared between passes.  The words of delta^l are also the per-layer ready flags that feed the k
// workers of section 3.
//
//   forward  (z),(a): workgroup g owns a block of rows of w^l, hence of a^l.  It gathers all of a^{l-1}
//                     (tagged words published by the owners), forms its a^l entries, publishes them.
//   backward (bp2):   workgroup g owns a block of COLUMNS of w^{l+1}, hence of delta^l: it reads its
//                     strip (16 to 128 bytes wide) of every row, so each column sum is formed inside one
//                     workgroup (fixed order) and the exchange is again an all-gather, of delta^l.
//                     Strips of workgroups that share an L2 (equal g mod 8) are adjacent in memory.
//                     Wide layers: 256-byte strips shared by four workgroups, each taking a block of
//                     rows; their partial sums are exchanged first, then delta^l.
//   (bp3),(bp4):      layer l belongs to worker (L-l) mod k.  With k >= 2 the workers are separate
//                     workgroups of the same kernel (k partitions of them, see gradient_worker); they
//                     split the rows of nabla_w^l, wait for delta^l through its tagged words and stream
//                     the gradient out with non-temporal stores while the chain moves on; the chain
//                     never waits for them.  With k = 1 (the sequential pass) the chain workgroups
//                     form the gradients in line, before stepping to the next layer.
//   descent step:     when it is fused in, the workers (present for every k then) read, step and rewrite
//                     w^l and b^l instead of storing the gradients, once every chain workgroup has
//                     reported the end of its reads of w^l.
//
// Every wait is bounded: a poll that exceeds its spin limit raises an abort word that all loops
// observe, the kernel drains, and the host reports LF_EHIP with the place of the failed wait.
#include "lf_internal.h"
#include "persistent.h"
#include "persistent_epoch.h"
#include "persistent_partition.h"

namespace lf {
namespace {

typedef unsigned long long u64;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kTableLds = kMaxPersistentDepth - 1;   // per-layer pointers, all kept in LDS

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
    unsigned limit; // polls before a wait gives up
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

// Poll up to four consecutive tagged words until all carry `tag`; n in 1..4 of them are valid.
// The four loads of a round are always issued together (slots past n re-read word n-1), so a round
// costs one memory round trip, not four.
// Returns whether the first poll missed.
__device__ __forceinline__ bool ll_wait4(const u64* p, int n, unsigned tag, float out[4], Abort& ab,
                                         int code) {
    out[0] = out[1] = out[2] = out[3] = 0.0f;
    if (n <= 0) return false;
    const u64* q[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) q[c] = p + min(c, n - 1);
    unsigned spin = 0;
    while (!ab.dead) {
        u64 w[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) w[c] = ll_load(q[c]);
        const bool ok = ll_tag(w[0]) == tag && ll_tag(w[1]) == tag && ll_tag(w[2]) == tag && ll_tag(w[3]) == tag;
        if (ok) {
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c] = (c < n) ? ll_val(w[c]) : 0.0f;
            return spin != 0;
        }
        ++spin;
        __builtin_amdgcn_s_sleep(2);   // a short back-off keeps the pollers from crowding the fabric
        if (spin > ab.limit) { ab.raise(code); return true; }
        if ((spin & 255u) == 0u) ab.seen();
    }
    return true;
}

// Gather up to four groups of four consecutive tagged words (group i at p[i], valid if n[i] > 0) with all
// sixteen loads in flight at once; groups that do not carry the tag yet are then polled one by one.
// Returns whether any group missed at the first look.
__device__ __forceinline__ bool ll_gather4x4(const u64* const p[4], const int n[4], unsigned tag,
                                             float out[4][4], Abort& ab, int code) {
    bool missed = false;
    u64 w[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) w[i][c] = ll_load(p[i] + min(c, max(n[i], 1) - 1));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool ok = ll_tag(w[i][0]) == tag && ll_tag(w[i][1]) == tag && ll_tag(w[i][2]) == tag &&
                        ll_tag(w[i][3]) == tag;
#pragma unroll
        for (int c = 0; c < 4; ++c) out[i][c] = c < n[i] ? ll_val(w[i][c]) : 0.0f;
        if (!ok && n[i] > 0) {
            missed = true;
            ll_wait4(p[i], n[i], tag, out[i], ab, code);
        }
    }
    return missed;
}

// Pause before the first poll of an exchange.  The peers need about a step's time to publish; polls sent
// earlier find nothing and only queue up, in front of the peers' stores, at the few memory channels that
// hold the exchanged words.
__device__ __forceinline__ void nap(int units) {
    for (int i = 0; i < units; ++i) __builtin_amdgcn_s_sleep(4);
}
// The tag of a launch's words lives in device memory, not in the kernel's arguments: a launch recorded in a
// HIP graph is replayed with the same arguments, and a replay whose words carried the tags of the launch
// before it would take that launch's leftovers for fresh data.  Every workgroup keeps a launch count of
// its own (so nothing is shared between workgroups and nobody waits).  All workgroups of a grid are launched
// equally often, so their counts agree; the end of the kernel orders the store before the next launch.
// One thread alone reads the count, stores the next one and hands the value to the rest of the workgroup
// through LDS behind the kernel's first barrier (which waits for the per-layer pointer tables anyway): no
// other thread ever reads the word in memory, so no wave can see the count of the next launch.
__device__ __forceinline__ void take_launch_count(unsigned* counts, unsigned* s_count) {
    if (threadIdx.x == 0) {
        unsigned* mine = counts + blockIdx.x;
        const unsigned c = __hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine, next_launch_count(c), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_count = c;
    }
}

// Word that holds element i of an exchanged vector.  Groups of eight words (64 bytes) are spread
// 8 << ll_shift bytes apart, so that the polls for one vector go to many memory channels instead of the
// one or two a packed vector would occupy.  Four consecutive elements starting at a multiple of four
// are always four consecutive words.
__device__ __forceinline__ size_t ll_index(const PersistArgs& A, int i) {
    return ((size_t)(i >> 3) << A.ll_shift) + (size_t)(i & 7);
}

__device__ __forceinline__ const float* act_ptr(const PersistArgs& A, int l) {
    return l == 1 ? A.a1 : A.a_base + (size_t)(l - 2) * A.a_stride;
}

// w^l has rows_of(l) rows of cols_of(l) entries: the neurons of layer l and of layer l-1.  Only the first and
// the last layer may be narrower than N.
// (The fields are copied to values first: a choice between two members of the argument block would keep the
// block in memory.)
__device__ __forceinline__ int cols_of(const PersistArgs& A, int l) {
    const int n = A.N, first = A.n_in;
    return l == 2 ? first : n;
}
__device__ __forceinline__ int rows_of(const PersistArgs& A, int l) {
    const int n = A.N, last = A.n_out, top = A.L;
    return l == top ? last : n;
}

// ================================================================================================
// forward
// ================================================================================================
// Q = float4 column groups per lane and row (Q*256 >= N); RF = rows per fetched chunk.  A wave owns RW
// consecutive rows and fetches them RF at a time; the chunk after the one being used is always in
// flight, also across the exchange between two layers.
// SINGLE: the wave's rows of a layer are one chunk (the latency-bound small nets); otherwise an even
// number of chunks per layer.
// NT: the weights are read with non-temporal loads (nets whose weights cannot stay in the caches between passes:
// every entry is read once per pass, by one workgroup; measured at L = 64, N = 4096: forward 850 -> 790 us, backward
// 1.67 -> 1.64 ms -- and 108 -> 169 us backward at L = 32, N = 1024, whose 130 MB of weights do stay).
template <int Q, int RF, bool SINGLE, bool NT>
__device__ __forceinline__ void forward_pass(const PersistArgs& args) {
    __shared__ unsigned s_count;
    __shared__ v4f s_a[Q * 64];
    __shared__ float s_bias[kMaxRowsPerGroup];
    __shared__ float s_z[kMaxRowsPerGroup];      // w^l a^{l-1} of my rows, until the layer's end
    __shared__ const float* s_w[kTableLds];      // w^l and b^l pointers: a table entry fetched from
    __shared__ const float* s_b[kTableLds];      // memory on the chain would cost a round trip per layer,
                                                 // and a generic load of it would be waited for together
                                                 // with every weight load in flight
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    PersistArgs A = args;
    int g = blockIdx.x;
    // Nets read from memory (fwd_band): the row blocks are numbered XCD by XCD, so that an XCD (workgroups are dealt
    // to the 8 XCDs round-robin) owns a contiguous eighth of the rows of w^l instead of every eighth block
    // (L = 64, N = 4096: 786 -> 757 us; runs of 4, 8 or 16 blocks per XCD: 768-772 us, of 2: 829 us).  Nets in the
    // cache are slower that way (L = 32, N = 1024: 66 -> 70 us).  g is the row block from here on.
    if (A.fwd_band && A.G % 8 == 0) g = (g % 8) * (A.G / 8) + g / 8;
    const int N = A.N, L = A.L, RPG = A.RPG, nvec = N >> 2;
    take_launch_count(A.counts_fwd, &s_count);
    for (int i = t; i < L - 1; i += kThreads) { s_w[i] = A.w[i]; s_b[i] = A.b[i]; }
    __syncthreads();
    A.epoch = forward_epoch(s_count);
    auto wptr = [&](int i) { return s_w[i]; };
    auto bptr = [&](int i) { return s_b[i]; };
    const int RW = (RPG + kWaves - 1) / kWaves;             // rows per wave
    const int wrow0 = g * RPG + wave * RW;                  // first row of this wave
    const int wrow_end = min(min(N, (g + 1) * RPG), wrow0 + RW);
    const int nchunks = SINGLE ? 1 : (((RW + RF - 1) / RF + 1) & ~1);   // even: see `layer` below
    Abort ab{A.abort_dev, A.abort_host, false, A.spin_limit};

    auto load_chunk = [&](v4f (&buf)[RF][Q], const float* W, int ci, int l) {        // W = w^l
        const int cols = cols_of(A, l), last_row = rows_of(A, l) - 1;
#pragma unroll
        for (int rr = 0; rr < RF; ++rr) {
            // one buffer per row: column groups past its end load zeros; rows past the end of the
            // matrix re-read the last row (their results are never used)
            const int row = min(wrow0 + ci * RF + rr, last_row);
            const __amdgpu_buffer_rsrc_t r = make_buffer(W + (size_t)row * cols, (unsigned)cols * 4u);
#pragma unroll
            for (int u = 0; u < Q; ++u) buf[rr][u] = buffer_load_v4f_as<NT>(r, (unsigned)(lane + 64 * u) * 16u);
        }
    };

    // A wait for one load also waits for every older load and store of the wave, and for nothing newer:
    // next layer's bias is requested ahead of next layer's weights.
    const bool own = t < RPG && g * RPG + t < N;
    auto own_row_of = [&](int l) { return own && g * RPG + t < rows_of(A, l); };      // my row exists in layer l
    float bias_next = own_row_of(2) ? load_global_f32_here(bptr(0) + g * RPG + t) : 0.0f;

    // a^{l-1}, from the tagged words its owners published, into LDS
    auto gather_activation = [&](int l) -> bool {
        bool missed = false;
        if (l == 2) {
            for (int v = t; v < (A.n_in >> 2); v += kThreads) s_a[v] = reinterpret_cast<const v4f*>(A.a1)[v];
            return false;
        }
        const u64* src = A.ALL + (size_t)(l - 3) * A.ll_layer;
        if (nvec <= kThreads) {
            if (t < nvec) {
                float o[4];
                missed = ll_wait4(src + ll_index(A, 4 * t), 4, A.epoch, o, ab, abort_code(1, l, (int)blockIdx.x));
                s_a[t] = v4f{o[0], o[1], o[2], o[3]};
            }
            return missed;
        }
        for (int v0 = t; v0 < nvec; v0 += 4 * kThreads) {
            const u64* gp[4];
            int gn[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int v = v0 + i * kThreads;
                gn[i] = v < nvec ? 4 : 0;
                gp[i] = src + ll_index(A, 4 * min(v, nvec - 1));
            }
            float o[4][4];
            missed |= ll_gather4x4(gp, gn, A.epoch, o, ab, abort_code(1, l, (int)blockIdx.x));
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (gn[i]) s_a[v0 + i * kThreads] = v4f{o[i][0], o[i][1], o[i][2], o[i][3]};
        }
        return missed;
    };
    // rows ci*RF .. of this wave: dot products with a^{l-1}, then bias, sigma, publish.  With several chunks per
    // layer the sums are left in LDS and the rest follows at the layer's end, for all rows at once: a store between
    // two chunks' loads would stand in front of the later loads in the wave's one queue, and the wait for those
    // loads would also wait for the store to be acknowledged by memory (N = 4096: 875 -> 853 us per pass).
    auto finish_chunk = [&](const v4f (&buf)[RF][Q], int ci, int l) {
        float acc[RF];
        const int nv = cols_of(A, l) >> 2, row_end = min(wrow_end, rows_of(A, l));
#pragma unroll
        for (int rr = 0; rr < RF; ++rr) acc[rr] = 0.0f;
#pragma unroll
        for (int u = 0; u < Q; ++u) {
            const int v = lane + 64 * u;
            const v4f av = s_a[min(v, Q * 64 - 1)];
            const v4f a = v < nv ? av : v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int rr = 0; rr < RF; ++rr) {
                acc[rr] = fmaf(buf[rr][u].x, a.x, acc[rr]);
                acc[rr] = fmaf(buf[rr][u].y, a.y, acc[rr]);
                acc[rr] = fmaf(buf[rr][u].z, a.z, acc[rr]);
                acc[rr] = fmaf(buf[rr][u].w, a.w, acc[rr]);
            }
        }
#pragma unroll
        for (int rr = 0; rr < RF; ++rr) {
            const int row = wrow0 + ci * RF + rr;
            const float z = wave_sum(acc[rr]);
            if constexpr (SINGLE) {
                if (lane == 0 && row < row_end) {
                    const float a = sigmoidf(z + s_bias[row - g * RPG]);
                    if (l < L) ll_store(A.ALL + (size_t)(l - 2) * A.ll_layer + ll_index(A, row), a, A.epoch);
                    A.a_base[(size_t)(l - 2) * A.a_stride + row] = a;
                }
            } else {
                if (lane == 0 && row < row_end) s_z[row - g * RPG] = z;
            }
        }
    };
    // One layer.  On entry bufA holds (possibly still in flight) this wave's first chunk of w^l.  The
    // two buffers alternate so that the chunk after the one in use is always in flight -- also across
    // the exchange -- without any register copy.  With one chunk per layer the next layer's chunk ends
    // up in bufB; with an even number of chunks it ends up in bufA again.
    auto layer = [&](v4f (&bufA)[RF][Q], v4f (&bufB)[RF][Q], int l) {
        if (own) s_bias[t] = bias_next;
        if (l > 2) nap(A.nap);
        gather_activation(l);
        __syncthreads();
        const float* W = wptr(l - 2);
        const float* Wn = l < L ? wptr(l - 1) : nullptr;
        // requested before any of the next layer's weights: the wait for it then leaves those in flight
        if (l < L) bias_next = own_row_of(l + 1) ? load_global_f32_here(bptr(l - 1) + g * RPG + t) : 0.0f;
        if constexpr (SINGLE) {
            if (Wn) load_chunk(bufB, Wn, 0, l + 1);
            finish_chunk(bufA, 0, l);
        } else {
            // both buffers enter the layer loaded (chunks 0 and 1 were requested before the exchange, so
            // that twice as much is in flight while the workgroups wait for each other)
            for (int ci = 0; ci < nchunks; ci += 2) {
                if (ci > 0) load_chunk(bufB, W, ci + 1, l);
                finish_chunk(bufA, ci, l);
                if (ci + 2 < nchunks) load_chunk(bufA, W, ci + 2, l);
                else if (Wn) load_chunk(bufA, Wn, 0, l + 1);
                finish_chunk(bufB, ci + 1, l);
            }
            if (Wn) load_chunk(bufB, Wn, 1, l + 1);
        }
        __syncthreads();   // s_a is rewritten by the next layer's gather; every row's sum is in s_z
        if (!SINGLE && own_row_of(l)) {
            const int row = g * RPG + t;
            const float a = sigmoidf(s_z[t] + s_bias[t]);
            if (l < L) ll_store(A.ALL + (size_t)(l - 2) * A.ll_layer + ll_index(A, row), a, A.epoch);
            A.a_base[(size_t)(l - 2) * A.a_stride + row] = a;
        }
    };

    v4f buf0[RF][Q], buf1[RF][Q];
    load_chunk(buf0, wptr(0), 0, 2);
    if constexpr (!SINGLE) load_chunk(buf1, wptr(0), 1, 2);
    if constexpr (SINGLE) {
        for (int l = 2; l <= L; l += 2) {
            layer(buf0, buf1, l);
            if (l + 1 <= L) layer(buf1, buf0, l + 1);
        }
    } else {
        for (int l = 2; l <= L; ++l) layer(buf0, buf1, l);
    }
}

// ================================================================================================
// backward
// ================================================================================================
constexpr int PG = kMaxPersistentN / 1024;   // float4 column groups a thread covers in a gradient row

// Marks a loaded value as used here: the wait for it is placed here and not at its first real use.  In front of a
// loop of stores this matters: a wait inside the loop, for a value requested before the loop, is a wait for every
// store of the iterations before as well (the counter cannot tell them apart), and the stores then leave one
// group at a time.
template <typename T>
__device__ __forceinline__ void arrived(T& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void arrived(v4f (&ja)[PG]) {
#pragma unroll
    for (int p = 0; p < PG; ++p) arrived(ja[p]);
}

// Rows row .. row+n-1 of nabla_w^layer (at gw) and nabla_b^layer (at gb) from their delta values d[0..n).
// (The caller reads the two pointers from their table once per layer: read here, before every group of rows, the
// wait for the pointer would also wait for every store of the group before.)
__device__ __forceinline__ void store_gradient_rows(const PersistArgs& A, int layer, float* gw, float* gb, int row,
                                                    int n, const float d[4], const v4f (&ja)[PG]) {
    const int t = threadIdx.x, N = cols_of(A, layer), nvec = N >> 2;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (c < n) {
            float* out = gw + (size_t)(row + c) * N;
#pragma unroll
            for (int p = 0; p < PG; ++p) {
                const int v = t + kThreads * p;
                if (v < nvec) {
                    const v4f o = {d[c] * ja[p].x, d[c] * ja[p].y, d[c] * ja[p].z, d[c] * ja[p].w};
                    store_global_nt_v4f(out + 4 * v, o);
                }
            }
            if (t == 0) store_global_f32(gb + row + c, d[c]);
        }
    }
}

// The same rows with the descent step fused in: w^layer and b^layer are read, stepped and written back in
// place, the gradient entries (rounded to fp32 as they would have been stored) never reach memory.  The
// results stay in the caches: the next forward pass reads them.
__device__ __forceinline__ void step_weight_rows(const PersistArgs& A, int layer, int row, int n,
                                                 const float d[4], const v4f (&ja)[PG]) {
    const int t = threadIdx.x, N = cols_of(A, layer), nvec = N >> 2;
    float* w = const_cast<float*>(A.w[layer - 2]);
    float* b = const_cast<float*>(A.b[layer - 2]);
    const float eta = A.sgd_eta;
    v4f old[4][PG];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int p = 0; p < PG; ++p) {
            const int v = min(t + kThreads * p, nvec - 1);           // rows and groups past the end re-read
            old[c][p] = load_global_v4f(w + (size_t)(row + min(c, n - 1)) * N + 4 * v);   // valid ones
        }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (c < n) {
            float* out = w + (size_t)(row + c) * N;
#pragma unroll
            for (int p = 0; p < PG; ++p) {
                const int v = t + kThreads * p;
                if (v < nvec) {
                    const v4f g = {d[c] * ja[p].x, d[c] * ja[p].y, d[c] * ja[p].z, d[c] * ja[p].w};
                    const v4f o = {fmaf(-eta, g.x, old[c][p].x), fmaf(-eta, g.y, old[c][p].y),
                                   fmaf(-eta, g.z, old[c][p].z), fmaf(-eta, g.w, old[c][p].w)};
                    *reinterpret_cast<v4f*>(out + 4 * v) = o;
                }
            }
            if (t == 0) b[row + c] = fmaf(-eta, d[c], b[row + c]);
        }
    }
}

__device__ __forceinline__ void load_activation_groups(const PersistArgs& A, int layer, v4f (&ja)[PG]) {
    const float* ap = act_ptr(A, layer);
    const int n = A.N, first = A.n_in;
    const int nvec = (layer == 1 ? first : n) >> 2;         // (never the last layer's)
#pragma unroll
    for (int p = 0; p < PG; ++p) ja[p] = load_global_v4f(ap + 4 * min((int)threadIdx.x + kThreads * p, nvec - 1));
}

// Poll one tagged word until it carries `tag`, napping between polls.
__device__ __forceinline__ float ll_wait1(const u64* p, unsigned tag, Abort& ab, int code) {
    unsigned spin = 0;
    while (!ab.dead) {
        const u64 w = ll_load(p);
        if (ll_tag(w) == tag) return ll_val(w);
        ++spin;
        __builtin_amdgcn_s_sleep(8);
        if (spin > ab.limit) { ab.raise(code); break; }
        if ((spin & 255u) == 0u) ab.seen();
    }
    return 0.0f;
}

// Gradient workgroup: member of worker partition `part`; streams out its share of rows of
// nabla_w^l, nabla_b^l for l = L - part, L - part - k, ... as soon as delta^l's words carry this
// pass's tag.  It never feeds the chain, so the chain never waits for it.  Each of its rows' words is
// polled by one thread only (the chain's own gathers read the same lines: every further poller slows
// them down) and handed to the others through LDS.
// With the descent step fused in it rewrites w^l, which the chain reads on its way to delta^{l-1}: it then also
// waits until every chain workgroup has reported the end of its reads of w^l (one tagged word per chain
// workgroup and layer, each polled by one thread).
__device__ __forceinline__ void gradient_worker(PersistArgs& A, unsigned* s_count, int wid, int nworkers,
                                                Abort& ab) {
    __shared__ float s_wd[kThreads];
    __shared__ int s_wdead;
    const int N = A.N, L = A.L, k = A.k, t = threadIdx.x;
    const int v = worker_slot(wid, nworkers, k, A.spread != 0);
    const int part = v % k, member = v / k, members = partition_members(part, nworkers, k);
    int jb, je;
    member_rows(member, members, N, &jb, &je);
    if (t == 0) s_wdead = 0;
    __syncthreads();
    A.epoch = backward_epoch(*s_count, true);
    if (jb >= je) return;                           // (behind the barrier: its launch count is taken)
    const bool sgd = A.sgd_eta != 0.0f;
    for (int layer = L - part; layer >= 2; layer -= k) {
        const int je_l = min(je, rows_of(A, layer));  // (a narrower last layer: some workgroups have no row of it)
        if (jb >= je_l) continue;
        v4f ja[PG];
        load_activation_groups(A, layer - 1, ja);
        float* gw = A.gw[layer - 2];
        float* gb = A.gb[layer - 2];
        const u64* dl = A.DLL + (size_t)(layer - 2) * A.ll_layer;
        bool wait_reads = sgd && layer >= 3;        // the chain never reads w^2
        for (int row0 = jb; row0 < je_l; row0 += kThreads) {
            const int nb = min(kThreads, je_l - row0);
            if (t < nb) s_wd[t] = ll_wait1(dl + ll_index(A, row0 + t), A.epoch, ab, abort_code(3, layer, (int)blockIdx.x));
            if (wait_reads && t < A.GB)
                ll_wait1(A.reads_done + (size_t)(layer - 2) * kMaxGroups + t, A.epoch, ab, abort_code(3, layer, (int)blockIdx.x));
            wait_reads = false;
            if (ab.dead) s_wdead = 1;
            __syncthreads();
            if (s_wdead) return;                    // the same for every thread
            arrived(ja);
            arrived(gw);
            arrived(gb);
            // (two loops, not one with the choice inside: the loads of the descent step would otherwise be on a
            // path around the store loop, and the stores would wait for registers those loads might still owe)
            if (sgd) {
                for (int r = 0; r < nb; r += 4) {
                    float d[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) d[c] = s_wd[min(r + c, nb - 1)];
                    step_weight_rows(A, layer, row0 + r, min(4, nb - r), d, ja);
                }
            } else if (A.pace > 1) {
                // The rows go out in A.pace bursts, burst i when the chain has published delta^{layer-i} (its first
                // word is the clock).  With one burst per chain step every partition stores a k-th of its layer at
                // the start of every step: memory sees all workers write at once, briefly, and then only the
                // chain's reads, instead of a steady mix of both (L = 64, N = 4096: 1.53 -> 1.48 ms at k = 8,
                // 1.505 -> 1.47 ms at k = 4; nets that fit the cache are bound by the exchange and lose a little).
                const int per = (((nb + A.pace - 1) / A.pace) + 3) & ~3;
                for (int i = 0, r0 = 0; r0 < nb; ++i, r0 += per) {
                    if (i > 0 && layer - i >= 2) {
                        if (t == 0)
                            ll_wait1(A.DLL + (size_t)(layer - i - 2) * A.ll_layer, A.epoch, ab, abort_code(3, layer, (int)blockIdx.x));
                        if (ab.dead) s_wdead = 1;
                        __syncthreads();
                        if (s_wdead) return;
                    }
                    const int r1 = min(nb, r0 + per);
                    for (int r = r0; r < r1; r += 4) {
                        float d[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) d[c] = s_wd[min(r + c, nb - 1)];
                        store_gradient_rows(A, layer, gw, gb, row0 + r, min(4, r1 - r), d, ja);
                    }
                }
            } else {
                for (int r = 0; r < nb; r += 4) {
                    float d[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) d[c] = s_wd[min(r + c, nb - 1)];
                    store_gradient_rows(A, layer, gw, gb, row0 + r, min(4, nb - r), d, ja);
                }
            }
            __syncthreads();                        // the next batch overwrites s_wd
        }
    }
}

// Sum, in row order, of the sixteen per-row partial sums of one column (group q, element e).
template <int TPR>
__device__ __forceinline__ float strip_column_sum(const v4f (&red)[kWaves * 4][TPR], int q, int e) {
    float u = red[0][q][e];
#pragma unroll
    for (int r = 1; r < kWaves * 4; ++r) u += red[r][q][e];
    return u;
}

// Workgroups [0, GB) run the delta chain; workgroups [GB, gridDim.x) are the gradient workers
// (present when k >= 2).  TPR = threads per 16*TPR-byte row segment of the owned column strip;
// CH = float4 loads per fetched chunk (chunks after the one in use are always in flight, also across
// the exchange).  At most 256 registers per thread, so that a chain and a gradient workgroup fit one
// compute unit.
// SINGLE: the strip of a step is one chunk; otherwise a multiple of four chunks per step.
// SPLIT: a strip is shared by RS workgroups, each taking a block of rows.  A strip is then a whole
// number of 128-byte lines also for wide layers (half-line strips stream at about two thirds of the
// rate); the price is one more exchange per step: the row blocks' partial sums go out as tagged words
// and each of the RS workgroups finishes 1/RS of the strip's columns, adding the partials in row-block
// order.
// FUSED (a grid without workers): the on-chain fusion.  The thread that multiplies an entry of w^{l+1} into
// the column sums of delta^l also forms and stores the same entry of nabla_w^{l+1} = delta^{l+1} (a^l)^T,
// inside the same chunk loop (delta^{l+1} is in LDS for the product anyway, the four a^l values of the
// thread's columns sit in registers).  Layer 2, whose weights the chain never reads, is stored at the end.
template <int TPR, int CH, bool SINGLE, bool SPLIT, bool FUSED, bool NT>
__device__ __forceinline__ void backward_pass(const PersistArgs& args) {
    constexpr int CPG = 4 * TPR;              // columns per chain workgroup
    constexpr int RPP = kThreads / TPR;       // rows covered by one load of the whole workgroup
    __shared__ v4f s_delta4[2][kMaxPersistentN / 4];    // delta^{l+1}, all of it, and delta^l as it is gathered
    __shared__ v4f s_red[kWaves * 4][TPR];              // per row of 16 lanes
    __shared__ const float* s_w[kTableLds];             // w^l pointers (see the forward kernel)
    __shared__ float* s_gw[FUSED ? kTableLds : 1];      // nabla_w^l, nabla_b^l pointers (on-chain fusion only)
    __shared__ float* s_gb[FUSED ? kTableLds : 1];
    __shared__ unsigned s_count;
    // (two buffers that change roles after every step: the sequential pass still reads delta^{l+1} for its
    // gradient rows when delta^l has been gathered)
    v4f* s_delta4_cur = s_delta4[0];
    v4f* s_delta4_nxt = s_delta4[1];
    auto delta_cur = [&]() { return reinterpret_cast<const float*>(s_delta4_cur); };
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, g = blockIdx.x;
    PersistArgs A = args;
    const int N = A.N, L = A.L, GB = A.GB, nvec = N >> 2;
    Abort ab{A.abort_dev, A.abort_host, false, A.spin_limit};
    take_launch_count(A.workers ? A.counts_bwdk : A.counts_bwd1, &s_count);
    if (g >= GB) {
        gradient_worker(A, &s_count, g - GB, (int)gridDim.x - GB, ab);
        return;
    }
    for (int i = t; i < L - 1; i += kThreads) {
        s_w[i] = A.w[i];
        if constexpr (FUSED) { s_gw[i] = A.gw[i]; s_gb[i] = A.gb[i]; }
    }
    __syncthreads();
    A.epoch = backward_epoch(s_count, A.workers != 0);
    auto wptr = [&](int i) { return s_w[i]; };
    // Strips narrower than a line: strips of workgroups on one XCD (workgroups are dealt to the 8 XCDs round-robin)
    // are adjacent, so that they share their lines through that XCD's L2.
    const int RS = SPLIT ? A.RS : 1;
    // Row-block strips (whole lines): an XCD takes runs of strip_run adjacent strips, the row blocks of a strip still
    // on one XCD.  Runs of two (512 bytes of every row) are fastest in every kind of grid at N = 4096, L = 64: with
    // workers 1.461 ms at k = 8 against 1.470, 1.478, 1.493 for runs of 4, 8 (an XCD's strips all adjacent) and 1;
    // the sequential pass 1.473 against 1.508, 1.537, 1.501.  (Done by renumbering the workgroup in front of the one
    // formula below: as a second formula beside it, it cost grids that never took it 2 %.)
    int gm = g;
    if (SPLIT && A.strip_run > 0 && GB % (8 * RS) == 0 && ((GB / RS) / 8) % A.strip_run == 0) {
        const int S = GB / RS, s8 = S / 8, c = A.strip_run, j0 = g / 8, x = g % 8, i = j0 / RS, rb0 = j0 % RS;
        const int target = ((i / c) * 8 + x) * c + i % c;
        gm = 8 * ((target % s8) * RS + rb0) + target / s8;
    }
    int strip = gm, rb = 0;
    if (GB % (8 * RS) == 0) {
        const int j = gm / 8;
        rb = j % RS;
        strip = (gm % 8) * (GB / (8 * RS)) + j / RS;
    } else if constexpr (SPLIT) {
        rb = g % RS;
        strip = g / RS;
    }
    const int NR = SPLIT ? (N + RS - 1) / RS : N;        // rows of one row block
    const int row_lo = min(N, rb * NR), row_hi = min(N, row_lo + NR);
    const int col0 = strip * CPG;
    const int cg = t % TPR, rs = t / TPR;
    const int col = min(col0 + 4 * cg, N - 4);           // a partial last strip re-reads valid columns
    const int nloads = (NR + RPP - 1) / RPP;
    constexpr int NB = SINGLE ? 2 : 4;                   // chunk buffers
    const int nchunks = SINGLE ? 1 : ((nloads + CH - 1) / CH + NB - 1) / NB * NB;   // see `step` below
    // rows of the sequential pass's in-line gradients
    // (taken from my own row block: the only part of delta this workgroup gathers)
    const int nstrips = GB / RS;
    const int RPGb = (row_hi - row_lo + nstrips - 1) / nstrips;
    const int jrow0 = min(row_hi, row_lo + strip * RPGb), jrow1 = min(row_hi, jrow0 + RPGb);

    // a chunk's buffer runs from the chunk's first pass to the end of my row block: a row past that end
    // loads zeros, and the per-thread offsets are the same for every chunk
    const unsigned strip_offset = ((unsigned)(row_lo + rs) * (unsigned)N + (unsigned)col) * 4u;
    const unsigned pass_bytes = (unsigned)RPP * (unsigned)N * 4u;
    const unsigned block_bytes = (unsigned)row_hi * (unsigned)N * 4u;
    auto load_chunk_of = [&](v4f (&buf)[CH], const float* W, int ci, unsigned bytes) {
        const unsigned skip = (unsigned)(ci * CH) * pass_bytes;
        const __amdgpu_buffer_rsrc_t r = make_buffer(reinterpret_cast<const char*>(W) + skip,
                                                     bytes > skip ? bytes - skip : 0u);
#pragma unroll
        for (int u = 0; u < CH; ++u) buf[u] = buffer_load_v4f_as<NT>(r, strip_offset + (unsigned)u * pass_bytes);
    };
    // w^L may have fewer rows than N: my row block of it ends where the matrix does
    const int top_hi = min(row_hi, A.n_out);
    const unsigned top_bytes = (unsigned)top_hi * (unsigned)N * 4u;
    // k = 1: rows [jrow0, jrow1) of layer's gradients.  (What the store loop needs is requested and awaited here,
    // under the one condition the call stands under: requested at the top of the step, the compiler would see a
    // path from request to the next step without the use, and make every step wait for all loads in flight.)
    struct InlineInputs { v4f ja[PG]; float* gw; float* gb; };
    auto inline_request = [&](int layer, InlineInputs& in) {
        load_activation_groups(A, layer - 1, in.ja);
        in.gw = A.gw[layer - 2];
        in.gb = A.gb[layer - 2];
        arrived(in.ja);
        arrived(in.gw);
        arrived(in.gb);
    };
    auto inline_store = [&](int layer, int part, const InlineInputs& in) {   // part 2: all rows; 0 / 1: their first /
        const int jr1_all = min(jrow1, rows_of(A, layer)), jr0_all = min(jrow0, jr1_all);           // second half
        const int mid = min(jr1_all, jr0_all + (((jr1_all - jr0_all) / 2 + 3) & ~3));
        const int jr0 = part == 1 ? mid : jr0_all, jr1 = part == 0 ? mid : jr1_all;
        for (int row = jr0; row < jr1; row += 4) {
            const int n = min(4, jr1 - row);
            float d[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) d[c] = delta_cur()[min(row + c, N - 1)];
            store_gradient_rows(A, layer, in.gw, in.gb, row, n, d, in.ja);
        }
    };
    auto inline_grads = [&](int layer) {
        InlineInputs in;
        inline_request(layer, in);
        inline_store(layer, 2, in);
    };
    // delta^layer's rows of my row block (float4 groups [gv0, gv1)), from their tagged words, into LDS
    const int gv0 = row_lo >> 2, gv1 = (row_hi + 3) >> 2;
    auto gather_delta = [&](int layer) -> bool {
        bool missed = false;
        const u64* src = A.DLL + (size_t)(layer - 2) * A.ll_layer;
        if (nvec <= kThreads) {
            if (t >= gv0 && t < gv1) {
                float o[4];
                missed = ll_wait4(src + ll_index(A, 4 * t), 4, A.epoch, o, ab, abort_code(2, layer, g));
                s_delta4_nxt[t] = v4f{o[0], o[1], o[2], o[3]};
            }
        } else {
            for (int v0 = gv0 + t; v0 < gv1; v0 += 4 * kThreads) {
                const u64* gp[4];
                int gn[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = v0 + i * kThreads;
                    gn[i] = v < gv1 ? 4 : 0;
                    gp[i] = src + ll_index(A, 4 * min(v, gv1 - 1));
                }
                float o[4][4];
                missed |= ll_gather4x4(gp, gn, A.epoch, o, ab, abort_code(2, layer, g));
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (gn[i]) s_delta4_nxt[v0 + i * kThreads] = v4f{o[i][0], o[i][1], o[i][2], o[i][3]};
            }
        }
        return missed;
    };

    // A wait for one load also waits for every older load and store of the wave.  So nothing slow is
    // requested just before the strip loads in flight are awaited: a^{l-1} (for the next step's sigma')
    // is requested right after delta^l is published, where its latency overlaps the exchange.
    // columns whose delta this workgroup finishes and publishes: its strip, or its share of it
    const int nfin = SPLIT ? CPG / RS : CPG, fcol0 = col0 + rb * nfin;
    const bool own = t < nfin && fcol0 + t < N;
    float a_next = (own && L > 2) ? load_global_f32_here(act_ptr(A, L - 1) + fcol0 + t) : 0.0f;
    // on-chain fusion: a^l at my four columns, the second factor of my entries of nabla_w^{l+1}; requested where
    // a_next is, element by element (a load the compiler leaves in place)
    auto load_strip_activation = [&](int layer) -> v4f {
        const float* ap = act_ptr(A, layer) + col;
        return v4f{load_global_f32_here(ap), load_global_f32_here(ap + 1), load_global_f32_here(ap + 2),
                   load_global_f32_here(ap + 3)};
    };
    v4f a4_next = {0.f, 0.f, 0.f, 0.f};
    if constexpr (FUSED) { if (L > 2) a4_next = load_strip_activation(L - 1); }
    const bool bias_writer = FUSED && strip == 0 && cg == 0;
    const bool inline_bursts = !A.workers && !A.no_grads && !FUSED;    // the sequential pass's gradient bursts
    v4f buf[NB][CH];
    if (L > 2) {                                     // my strip of w^L, needed by the first chain step
        load_chunk_of(buf[0], wptr(L - 2), 0, top_bytes);
        if constexpr (!SINGLE) {
#pragma unroll
            for (int j = 1; j < NB; ++j) load_chunk_of(buf[j], wptr(L - 2), j, top_bytes);
        }
    }

    // (bp1): every chain workgroup forms all of delta^L (N cheap elements, no exchange); the owner of
    // a column block also stores and publishes it
    {
        const float* aL = act_ptr(A, L);
        for (int i = t; i < N; i += kThreads) {
            float v = 0.0f;                          // (past a narrower last layer: zeros)
            if (i < A.n_out) {
                const float a = aL[i];
                v = A.cost_scale * ((a - A.y[i]) * (a * (1.0f - a)));
            }
            reinterpret_cast<float*>(s_delta4_cur)[i] = v;
        }
        __syncthreads();
        if (own && fcol0 + t < A.n_out) {
            const float d = delta_cur()[fcol0 + t];
            ll_store(A.DLL + (size_t)(L - 2) * A.ll_layer + ll_index(A, fcol0 + t), d, A.epoch);
            A.d_base[(size_t)(L - 2) * A.d_stride + fcol0 + t] = d;
        }
    }

    // gwl, gbl, a4 (on-chain fusion only): nabla_w^{l+1}, nabla_b^{l+1}, a^l at my columns.  nabla_w^{l+1} is laid
    // out like w^{l+1}, so an entry is stored through a buffer at the very offset its weight was loaded from,
    // and rows past the end of my row block fall outside the buffer (no store).
    // (rhi, wbytes: the end of my row block of this step's matrix, as a row and in bytes)
    auto fma_chunk = [&](const v4f (&buf)[CH], int ci, v4f& acc, float* gwl, float* gbl, const v4f& a4, int rhi,
                         unsigned wbytes) {
        const unsigned gskip = (unsigned)(ci * CH) * pass_bytes;
        const __amdgpu_buffer_rsrc_t gr = make_buffer(reinterpret_cast<const char*>(gwl) + (FUSED ? gskip : 0u),
                                                      FUSED && wbytes > gskip ? wbytes - gskip : 0u);
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int row = row_lo + rs + RPP * (ci * CH + u);
            const float dv = delta_cur()[min(row, N - 1)];
            const float d = row < rhi ? dv : 0.0f;
            acc.x = fmaf(buf[u].x, d, acc.x);
            acc.y = fmaf(buf[u].y, d, acc.y);
            acc.z = fmaf(buf[u].z, d, acc.z);
            acc.w = fmaf(buf[u].w, d, acc.w);
            if constexpr (FUSED) {
                const v4f o = {d * a4.x, d * a4.y, d * a4.z, d * a4.w};
                buffer_store_nt_v4f(gr, strip_offset + (unsigned)u * pass_bytes, o);
                if (bias_writer && row < rhi) store_global_f32(gbl + row, d);
            }
        }
    };
    // One chain step, delta^{l+1} -> delta^l.  SINGLE: on entry bufA holds (possibly still in flight) my
    // strip of w^{l+1}, and the next step's is requested into bufB before this one is used.  Otherwise
    // chunk c lives in buffer c mod NB and the step has a multiple of NB chunks: on entry the first NB
    // are loaded or in flight, and as soon as a chunk has been used its buffer is requested again, for
    // chunk c + NB of this step or, past its end, of the next step -- so NB - 1 chunks stay in flight all
    // the time, also across the exchange, without any register copy.
    auto step = [&](v4f (&bufA)[CH], v4f (&bufB)[CH], int l) {
        const float a_l = a_next;
        const v4f a4 = a4_next;
        float* gwl = nullptr;
        float* gbl = nullptr;
        if constexpr (FUSED) { gwl = s_gw[l - 1]; gbl = s_gb[l - 1]; }
        const float* W = wptr(l - 1);
        const float* Wn = l > 2 ? wptr(l - 2) : nullptr;
        const int rhi = l + 1 == L ? top_hi : row_hi;
        const unsigned wbytes = l + 1 == L ? top_bytes : block_bytes;
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        if constexpr (SINGLE) {
            // (unconditional, like the refills below: past the last layer it reads an empty buffer.  With a
            // branch around it there is a path on which bufA's loads are the youngest in flight, and the waits
            // in front of the multiplications are then set for that path: they would wait for bufB as well,
            // i.e. for the next step's weights within this step.)
            load_chunk_of(bufB, Wn ? Wn : W, 0, Wn ? block_bytes : 0u);
            fma_chunk(bufA, 0, acc, gwl, gbl, a4, rhi, wbytes);
        } else {
            // every refill is one unconditional load: past the last layer it reads an empty buffer
            // (zeros, no memory traffic), so a buffer's registers are never carried around a branch
            const float* Wnext = Wn ? Wn : W;
            const unsigned next_bytes = Wn ? block_bytes : 0u;
            for (int ci = 0; ci < nchunks; ci += NB) {
                const bool same = ci + NB < nchunks;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    fma_chunk(buf[j], ci + j, acc, gwl, gbl, a4, rhi, wbytes);
                    load_chunk_of(buf[j], same ? W : Wnext, same ? ci + j + NB : j, same ? wbytes : next_bytes);
                }
            }
        }
        // add the threads that share a column group: within each row of 16 lanes by rotation; the sixteen
        // rows of the workgroup are then added in order by the thread that finishes the column
        acc.x = row_class_sum<TPR>(acc.x);
        acc.y = row_class_sum<TPR>(acc.y);
        acc.z = row_class_sum<TPR>(acc.z);
        acc.w = row_class_sum<TPR>(acc.w);
        if ((lane & 15) < TPR) s_red[wave * 4 + (lane >> 4)][lane & 15] = acc;
        __syncthreads();
        // every load of w^{l+1} by this workgroup has been used: tell the workers, who are about to rewrite it
        if (A.sgd_eta != 0.0f && t == 0) ll_store(A.reads_done + (size_t)(l - 1) * kMaxGroups + g, 1.0f, A.epoch);
        if constexpr (SPLIT) {
            // my row block's partial sums of the strip go out; the partials of my share of its columns
            // come in, from every row block (mine included), and are added in row-block order
            u64* pl = A.PLL + (size_t)(l - 2) * N * RS;
            if (t < CPG && col0 + t < N) {
                const int q = t >> 2, e = t & 3;
                const float u = strip_column_sum(s_red, q, e);
                ll_store(pl + (size_t)(col0 + t) * RS + rb, u, A.epoch);
            }
            auto finish_my_columns = [&]() {
                if (own) {
                    float p[4];
                    ll_wait4(pl + (size_t)(fcol0 + t) * RS, RS, A.epoch, p, ab, abort_code(0, l, g));
                    const float u = ((p[0] + p[1]) + p[2]) + p[3];      // slots past RS hold zeros
                    const float d = u * (a_l * (1.0f - a_l));
                    ll_store(A.DLL + (size_t)(l - 2) * A.ll_layer + ll_index(A, fcol0 + t), d, A.epoch);
                    A.d_base[(size_t)(l - 2) * A.d_stride + fcol0 + t] = d;
                    if (l > 2) a_next = load_global_f32_here(act_ptr(A, l - 1) + fcol0 + t);
                }
            };
            if (inline_bursts) {
                // the sequential pass stores half of its rows of layer l+1's gradients while the partial sums are
                // under way, the other half while delta^l is (one request of what the stores need, one branch)
                InlineInputs in;
                inline_request(l + 1, in);
                inline_store(l + 1, 0, in);
                finish_my_columns();
                inline_store(l + 1, 1, in);
            } else {
                finish_my_columns();
            }
            if constexpr (FUSED) { if (l > 2) a4_next = load_strip_activation(l - 1); }
        } else {
            if (own) {
                const int q = t >> 2, e = t & 3;
                const float u = strip_column_sum(s_red, q, e);
                const float d = u * (a_l * (1.0f - a_l));
                ll_store(A.DLL + (size_t)(l - 2) * A.ll_layer + ll_index(A, col0 + t), d, A.epoch);
                A.d_base[(size_t)(l - 2) * A.d_stride + col0 + t] = d;
                if (l > 2) a_next = load_global_f32_here(act_ptr(A, l - 1) + col0 + t);
            }
            if constexpr (FUSED) { if (l > 2) a4_next = load_strip_activation(l - 1); }
        }
        // exchange: all of delta^l, into the other buffer.  The sequential pass stores its rows of layer l+1's
        // gradients between publishing and gathering, from delta^{l+1} in the buffer the step has just used: the
        // stores fill the time the peers' words are under way.
        if constexpr (!SPLIT) {
            if (inline_bursts) inline_grads(l + 1);
        }
        if (!inline_bursts) nap(A.nap);
        gather_delta(l);
        __syncthreads();
        v4f* const was = s_delta4_cur;
        s_delta4_cur = s_delta4_nxt;
        s_delta4_nxt = was;
    };

    if constexpr (SINGLE) {
        for (int l = L - 1; l >= 2; l -= 2) {
            step(buf[0], buf[1], l);
            if (l - 1 >= 2) step(buf[1], buf[0], l - 1);
        }
    } else {
        for (int l = L - 1; l >= 2; --l) step(buf[0], buf[1], l);
    }
    if (!A.workers && !A.no_grads) inline_grads(2);
}

template <int Q, int RF, bool SINGLE, bool NT = false>
__global__ __launch_bounds__(kThreads, 2) void k_fwd_persistent(const PersistArgs args) {
    forward_pass<Q, RF, SINGLE, NT>(args);
}
// The backward kernel runs with two grids: chain workgroups only (k = 1 without the descent step, the on-chain
// fusion, the chain alone), or chain + gradient workers.  Each grid has its own launch counts and its own
// tags (see persistent_epoch.h), so the words of one can never pass for the other's.
// (The fused grid has no worker workgroups to share a compute unit with: one wave per SIMD, hence twice the
// registers, which the extra stores of its multi-chunk loops need.)
template <int TPR, int CH, bool SINGLE, bool SPLIT, bool FUSED, bool NT = false>
__global__ __launch_bounds__(kThreads, FUSED ? 1 : 2) void k_bwd_persistent(const PersistArgs args) {
    static_assert(!NT || SPLIT, "non-temporal weight loads are instantiated for the wide-layer instances only");
    backward_pass<TPR, CH, SINGLE, SPLIT, FUSED, NT>(args);
}

__global__ __launch_bounds__(kThreads) void k_fill_u64(u64* p, size_t n, u64 v) {
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads)
        p[i] = v;
}

}  // namespace

size_t persistent_ll_layer_words(int N, int ll_shift) {
    return ((size_t)((N + 7) >> 3) << ll_shift);
}

bool persistent_supported(int L, int N) {
    return N % 4 == 0 && N >= 4 && N <= kMaxPersistentN && L >= 2 && L <= kMaxPersistentDepth;
}

// Forward: G workgroups, each owning rpg rows; every workgroup owns at least one row.
void persistent_forward_shape(int N, int num_cus, int requested, int* G, int* rpg) {
    // up to two workgroups per compute unit (each needs at most 256 registers per thread)
    int g = requested > 0 ? requested : kMaxGroups;
    if (g > (N + 3) / 4) g = (N + 3) / 4;
    if (g > 2 * kMaxGroups) g = 2 * kMaxGroups;
    if (num_cus > 0 && g > 2 * num_cus) g = 2 * num_cus;
    if (g < 1) g = 1;
    *rpg = (N + g - 1) / g;
    *G = (N + *rpg - 1) / *rpg;
}

// Backward chain: strips of 4*tpr columns, tpr in {1, 2, 4, 8} (16 with four row blocks), each shared by
// rs row blocks;
// GB = strips * rs workgroups.  Wide layers (N > 2048) take 256-byte strips in four row blocks.
void persistent_backward_shape(int N, int num_cus, int requested, int row_split, int* GB, int* tpr, int* rs) {
    int split = (row_split == 1 || row_split == 2 || row_split == 4) ? row_split : (N > 2048 ? 4 : 1);
    while (split > 1 && N < 4 * split) split >>= 1;      // every row block holds rows
    int cap = requested > 0 ? requested : (N <= 2048 ? 128 : kMaxGroups);
    if (cap > kMaxGroups) cap = kMaxGroups;
    if (num_cus > 0 && cap > num_cus) cap = num_cus;
    if (cap < 1) cap = 1;
    const int groups4 = (N + 3) / 4;                    // float4 column groups
    for (;; split >>= 1) {
        const int aim = cap / split > 0 ? cap / split : 1;   // strips aimed at
        int need = (groups4 + aim - 1) / aim, tp = 1;
        const int tp_max = split == 4 ? 16 : 8;              // strips of up to 128 bytes, 256 in four blocks
        while (tp < need && tp < tp_max) tp <<= 1;
        while (split > 1 && 4 * tp % split != 0) tp <<= 1;   // a strip's columns divide among its row blocks
        *tpr = tp;
        *rs = split;
        *GB = (groups4 + tp - 1) / tp * split;
        // more workgroups than aimed at: only acceptable when nothing is left to give (tp capped at 8)
        if (*GB <= cap || split == 1) return;
    }
}

hipError_t launch_fill_u64(void* p, size_t n_words, unsigned long long v, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    k_fill_u64<<<1024, kThreads, 0, s>>>(static_cast<u64*>(p), n_words, v);
    return hipGetLastError();
}

typedef void (*persist_kernel_t)(const PersistArgs);

// The forward kernel instance for this shape (nullptr: none).
static bool edge_widths_ok(const PersistArgs& A) {
    return A.n_in >= 4 && A.n_in <= A.N && A.n_in % 4 == 0 && A.n_out >= 4 && A.n_out <= A.N && A.n_out % 4 == 0;
}

static persist_kernel_t forward_kernel(const PersistArgs& A) {
    if (!persistent_supported(A.L, A.N) || !edge_widths_ok(A) || A.G > kMaxLaunchGroups) return nullptr;
    const int q = (A.N / 4 + 63) / 64;                       // float4 groups per lane and row
    const int rw = (A.RPG + kWaves - 1) / kWaves;            // rows per wave
    if (q <= 4) {
        if (rw == 1) return k_fwd_persistent<4, 1, true>;
        if (rw == 2) return k_fwd_persistent<4, 2, true>;
        if (rw <= 4) return k_fwd_persistent<4, 4, true>;
        return k_fwd_persistent<4, 4, false>;
    }
    if (q <= 8) {
        if (rw == 1) return k_fwd_persistent<8, 1, true>;
        if (rw == 2) return k_fwd_persistent<8, 2, true>;
        return k_fwd_persistent<8, 2, false>;
    }
    if (q <= 16) {
        if (rw == 1) return A.stream_weights ? k_fwd_persistent<16, 1, true, true> : k_fwd_persistent<16, 1, true>;
        return A.stream_weights ? k_fwd_persistent<16, 1, false, true> : k_fwd_persistent<16, 1, false>;
    }
    return nullptr;
}

template <int TPR, bool FUSED>
static persist_kernel_t backward_kernel_tpr(const PersistArgs& A) {
    const int nloads = (A.N + kThreads / TPR - 1) / (kThreads / TPR);
    // (row-block strips: chunks of eight loads beside gradient workers; chunks of two for the sequential pass, whose
    // stores then have memory more to themselves -- with eight loads in flight per thread instead of thirty-two
    // fewer of the next step's reads fall among them: 1.58 against 1.65 ms at L = 64, N = 4096; beside workers the
    // short chunks lose, 1.76 against 1.67 ms)
    if constexpr (!FUSED) {
        if (A.RS > 1 && !A.workers)
            return A.stream_weights ? k_bwd_persistent<TPR, 2, false, true, false, true>
                                    : k_bwd_persistent<TPR, 2, false, true, false>;
    }
    if (A.RS > 1)
        return A.stream_weights ? k_bwd_persistent<TPR, 8, false, true, FUSED, true>
                                : k_bwd_persistent<TPR, 8, false, true, FUSED>;
    if (nloads <= 4) return k_bwd_persistent<TPR, 4, true, false, FUSED>;
    if (nloads <= 8) return k_bwd_persistent<TPR, 8, true, false, FUSED>;
    return k_bwd_persistent<TPR, 8, false, false, FUSED>;
}

template <bool FUSED>
static persist_kernel_t backward_kernel_of(const PersistArgs& A) {
    switch (A.TPR) {
        case 1: return backward_kernel_tpr<1, FUSED>(A);
        case 2: return backward_kernel_tpr<2, FUSED>(A);
        case 4: return backward_kernel_tpr<4, FUSED>(A);
        case 8: return backward_kernel_tpr<8, FUSED>(A);
        case 16: return A.RS == 4 ? backward_kernel_tpr<16, FUSED>(A) : nullptr;
        default: return nullptr;
    }
}

// The backward kernel instance for this shape and variant (nullptr: none).
static persist_kernel_t backward_kernel(const PersistArgs& A) {
    if (A.GB > kMaxGroups * 2 || !persistent_supported(A.L, A.N) || !edge_widths_ok(A)) return nullptr;
    if (A.RS != 1 && A.RS != 2 && A.RS != 4) return nullptr;
    if (A.GB % A.RS != 0 || (4 * A.TPR) % A.RS != 0) return nullptr;
    if (A.GB > kMaxGroups || kMaxGroups > kThreads) return nullptr;   // one polling thread per chain workgroup
    return A.fused ? backward_kernel_of<true>(A) : backward_kernel_of<false>(A);
}

// How many workgroups of each kernel instance one compute unit holds at a time, by the runtime's own
// occupancy calculation for that instance (registers, LDS, waves).
hipError_t persistent_resident_per_cu(const PersistArgs& A, int* forward, int* backward, int* backward_fused) {
    PersistArgs B = A;
    const persist_kernel_t kf = forward_kernel(A);
    B.fused = 0;
    const persist_kernel_t kb = backward_kernel(B);
    B.fused = 1;
    const persist_kernel_t kbf = backward_kernel(B);
    if (!kf || !kb || !kbf) return hipErrorInvalidValue;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(forward, kf, kThreads, 0);
    if (e != hipSuccess) return e;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(backward, kb, kThreads, 0);
    if (e != hipSuccess) return e;
    // (the grids with and without workers may take different instances: the smaller figure serves both)
    B.fused = 0;
    B.workers = A.workers ? 0 : 1;
    const persist_kernel_t kb2 = backward_kernel(B);
    if (!kb2) return hipErrorInvalidValue;
    int other = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&other, kb2, kThreads, 0);
    if (e != hipSuccess) return e;
    if (other < *backward) *backward = other;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(backward_fused, kbf, kThreads, 0);
}

hipError_t launch_fwd_persistent(const PersistArgs& A, hipStream_t s) {
    const persist_kernel_t k = forward_kernel(A);
    if (!k) return hipErrorInvalidValue;
    k<<<A.G, kThreads, 0, s>>>(A);
    return hipGetLastError();
}

hipError_t launch_bwd_persistent(const PersistArgs& A, hipStream_t s) {
    const persist_kernel_t k = backward_kernel(A);
    if (!k) return hipErrorInvalidValue;
    if ((A.k > 1 || A.sgd_eta != 0.0f) != (A.workers != 0)) {
        if (!(A.workers == 0 && (A.fused || A.no_grads))) return hipErrorInvalidValue;
    }
    if (A.workers && (A.fused || A.no_grads)) return hipErrorInvalidValue;
    if (A.fused && A.sgd_eta != 0.0f) return hipErrorInvalidValue;
    const int grid = A.GB + (A.workers ? A.GW : 0);  // chain workgroups, then the gradient workers
    if (grid > kMaxLaunchGroups) return hipErrorInvalidValue;
    k<<<grid, kThreads, 0, s>>>(A);
    return hipGetLastError();
}

}  // namespace lf
