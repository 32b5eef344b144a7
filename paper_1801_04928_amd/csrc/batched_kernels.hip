// Minibatch (B > 1) kernels: the three per-layer contractions of the pass as LDS-tiled MFMA GEMMs.
//
//   forward (z),(a):  A_out[b][j] = sigma( sum_k A_in[b][k]  W[j][k]  + bias[j] )
//   chain   (bp2):    D_l[b][k]   = ( sum_j D_next[b][j] W_next[j][k] ) * A_l[b][k] (1 - A_l[b][k])
//   grads   (bp4):    nabla_w[j][k] = sum_b D[b][j] A_prev[b][k]        (bp3): nabla_b[j] = sum_b D[b][j]
//
// All three are  C[m][n] = sum_q P(m,q) Q(n,q)  with operands that are either contiguous along the
// contraction index q ("QC": element (i,q) at p[i*ld + q]) or along their own index ("IC": element
// (i,q) at p[q*ld + i]).  forward: P = A_in (QC), Q = W (QC).  chain: P = D_next (QC), Q = W_next (IC).
// grads: P = D (IC), Q = A_prev (IC).  Accumulation is fp32 in the MFMA accumulators, in an order fixed
// by (N, B) alone, so results do not depend on k or on the launch.
#include "lf_internal.h"

namespace lf {
namespace {

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128;          // output tile of a workgroup; 2 x 2 waves of 64 x 64

__host__ __device__ constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }

enum Epilogue { EPI_RAW = 0, EPI_SIGMOID = 1, EPI_SIGMA_PRIME = 2, EPI_GRAD = 3 };

template <typename T> struct Tile;
template <> struct Tile<float> {
    static constexpr int BK = 32;
    static constexpr int LDA = BM + 4;     // LDS is [q][i]: a lane reads one float per MFMA, lanes along i
    static constexpr int ELEMS = BK * LDA;
};
template <> struct Tile<__bf16> {
    static constexpr int BK = 64;
    static constexpr int LDA = BK + 8;     // QC operand: LDS is [i][q], a lane reads 8 consecutive q (16 bytes)
    static constexpr int LDI = BM + 32;    // IC operand: LDS is [q][i] as in memory; read with the transposing
                                           // ds_read_b64_tr_b16, which hands each lane 4 consecutive q.  A half
                                           // wave reads 4 rows x 64 bytes: with a row stride of 16 banks more than
                                           // a multiple of 64 the four rows fill the 64 banks exactly (measured:
                                           // no bank conflicts; +16 elements gave one conflict cycle in three)
    static constexpr int ELEMS = BM * LDA > BK * LDI ? BM * LDA : BK * LDI;
};

struct GemmArgs {
    const void* P;  int ldp;               // rows of P index m
    const void* Q;  int ldq;               // rows of Q index n
    unsigned p_bytes, q_bytes;             // sizes of the two operand matrices (< 4 GiB each)
    int M, Nn, K;                          // C is M x Nn, contraction length K
    int k_tiles_per_split;                 // split-K: blockIdx.z handles this many BK tiles
    float* raw;                            // EPI_RAW: [splits][M][Nn] fp32
    const float* bias;                     // EPI_SIGMOID: [Nn]
    const void* act;                       // EPI_SIGMA_PRIME: A_l [M][Nn], type T
    void* out;                             // EPI_SIGMOID: T [M][Nn]; EPI_SIGMA_PRIME / EPI_GRAD: float [M][Nn]
    void* out_bf;                          // EPI_SIGMA_PRIME with bf16: bfloat16 copy of out (or null);
                                           // EPI_GRAD with sgd_eta: the bfloat16 weights to rewrite (or null)
    float sgd_eta;                         // EPI_GRAD: != 0 = out holds w^l in fp32 and receives w - eta * C
};

// ---- global -> register staging ---------------------------------------------------------------
// Each thread stages 4 x 16 bytes per operand and tile.  The operand is addressed as one buffer: a
// vector that lies outside the matrix (row past the end, or past the contraction length) is given an
// offset past the end of the buffer and loads zeros.  No branch surrounds a load, so the compiler can
// count the loads in flight and the prefetch depth below is real.
constexpr unsigned kOutside = 0xFFFFFFF0u;

template <typename T, bool IC> struct Stage;

template <> struct Stage<float, false> {   // [i][q], float4 along q; 8 threads cover 32 q of one row
    v4f r[4];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int I, int Kq) {
        const int t = threadIdx.x, qv = (t & 7) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = (t >> 3) + 32 * u;
            const bool ok = (i0 + i < I) && (q0 + qv < Kq);
            const unsigned off = ((unsigned)(i0 + i) * (unsigned)ld + (unsigned)(q0 + qv)) * 4u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(float* s) const {
        const int t = threadIdx.x, qv = (t & 7) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = (t >> 3) + 32 * u;
#pragma unroll
            for (int c = 0; c < 4; ++c) s[(qv + c) * Tile<float>::LDA + i] = r[u][c];
        }
    }
};
template <> struct Stage<float, true> {    // [q][i], float4 along i; 32 threads cover 128 i of one q
    v4f r[4];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int I, int Kq) {
        const int t = threadIdx.x, iv = (t & 31) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = (t >> 5) + 8 * u;
            const bool ok = (q0 + q < Kq) && (i0 + iv < I);
            const unsigned off = ((unsigned)(q0 + q) * (unsigned)ld + (unsigned)(i0 + iv)) * 4u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(float* s) const {
        const int t = threadIdx.x, iv = (t & 31) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = (t >> 5) + 8 * u;
            *reinterpret_cast<v4f*>(s + q * Tile<float>::LDA + iv) = r[u];
        }
    }
};
template <> struct Stage<__bf16, false> {  // [i][q], 8 bf16 along q; 8 threads cover 64 q of one row
    v4f r[4];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int I, int Kq) {
        const int t = threadIdx.x, qv = (t & 7) * 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = (t >> 3) + 32 * u;
            const bool ok = (i0 + i < I) && (q0 + qv < Kq);
            const unsigned off = ((unsigned)(i0 + i) * (unsigned)ld + (unsigned)(q0 + qv)) * 2u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(__bf16* s) const {
        const int t = threadIdx.x, qv = (t & 7) * 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = (t >> 3) + 32 * u;
            *reinterpret_cast<v4f*>(s + i * Tile<__bf16>::LDA + qv) = r[u];
        }
    }
};
template <> struct Stage<__bf16, true> {   // [q][i], 8 bf16 along i; 16 threads cover 128 i of one q
    v4f r[4];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int I, int Kq) {
        const int t = threadIdx.x, iv = (t & 15) * 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = (t >> 4) * 4 + u;            // a thread holds 4 consecutive q of its 8 i
            const bool ok = (q0 + q < Kq) && (i0 + iv < I);
            const unsigned off = ((unsigned)(q0 + q) * (unsigned)ld + (unsigned)(i0 + iv)) * 2u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(__bf16* s) const {   // LDS keeps the memory layout [q][i]
        const int t = threadIdx.x, iv = (t & 15) * 8, q = (t >> 4) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) *reinterpret_cast<v4f*>(s + (q + u) * Tile<__bf16>::LDI + iv) = r[u];
    }
};

// MFMA operand (8 consecutive q for row i = lane % 32, starting at q0 + 8 (lane / 32)) from an LDS tile kept
// as [q][i].  ds_read_b64_tr_b16 works on groups of 16 lanes: source lane s supplies the address of four
// consecutive i, result lane r receives element (r % 4) of source lanes r/4, 4 + r/4, 8 + r/4, 12 + r/4.
// With source lane s pointing at row q = s/4, columns 4 (s % 4) .. +3, result lane r holds q = 0..3 at
// column r: four consecutive q of its own row.  Two such loads give the eight values.
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
__device__ __forceinline__ v8bf lds_operand_transposed(const __bf16* tile, int ld, int i_base, int q0) {
    const int lane = threadIdx.x & 63, s16 = lane & 15;
    const int q = q0 + 8 * (lane >> 5) + (s16 >> 2);
    const int i = i_base + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);
    typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(tile + q * ld + i));
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(tile + (q + 4) * ld + i));
    const v8s both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(v8bf, both);
}

// ---- the kernel -------------------------------------------------------------------------------
template <typename T, bool P_IC, bool Q_IC, int EPI>
__global__ __launch_bounds__(kThreads) void k_gemm(const GemmArgs g) {
    using TL = Tile<T>;
    // one block: the two operand tiles, and afterwards the staging area of the gradient epilogue
    constexpr int kOperandBytes = 2 * TL::ELEMS * (int)sizeof(T);
    constexpr int kEpilogueBytes = 4 * 32 * (64 + 4) * 4;       // 4 waves x 32 rows x (64+4) floats
    __shared__ __attribute__((aligned(16))) char s_block[kOperandBytes > kEpilogueBytes ? kOperandBytes : kEpilogueBytes];
    T* s_p = reinterpret_cast<T*>(s_block);
    T* s_q = s_p + TL::ELEMS;

    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int r32 = lane & 31, half = lane >> 5;

    const int kt_total = ceil_div(g.K, TL::BK);
    const int kt_begin = blockIdx.z * g.k_tiles_per_split;
    const int kt_end = min(kt_total, kt_begin + g.k_tiles_per_split);

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Global -> register -> LDS with a prefetch distance of three k-tiles: tile kt+3 is requested while
    // tile kt is multiplied, which covers the memory latency even when only one or two workgroups share
    // a compute unit.  The three register stages rotate by a 3-way unrolled loop (static indexing).
    Stage<T, P_IC> sp[3];
    Stage<T, Q_IC> sq[3];
    const __amdgpu_buffer_rsrc_t P = make_buffer(g.P, g.p_bytes);
    const __amdgpu_buffer_rsrc_t Q = make_buffer(g.Q, g.q_bytes);
#pragma unroll
    for (int u = 0; u < 3; ++u)
        if (kt_begin + u < kt_end) {
            sp[u].load(P, g.ldp, m0, (kt_begin + u) * TL::BK, g.M, g.K);
            sq[u].load(Q, g.ldq, n0, (kt_begin + u) * TL::BK, g.Nn, g.K);
        }
    __builtin_amdgcn_sched_barrier(0);   // keep the requests up here: the scheduler would sink them to their uses
    auto multiply_tile = [&]() {
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int kk = 0; kk < TL::BK; kk += 2) {
                float a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i] = s_p[(kk + half) * TL::LDA + wm + i * 32 + r32];
#pragma unroll
                for (int j = 0; j < 2; ++j) b[j] = s_q[(kk + half) * TL::LDA + wn + j * 32 + r32];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < TL::BK; kk += 16) {
                v8bf a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    if constexpr (P_IC) a[i] = lds_operand_transposed(s_p, TL::LDI, wm + i * 32, kk);
                    else a[i] = *reinterpret_cast<const v8bf*>(&s_p[(wm + i * 32 + r32) * TL::LDA + kk + half * 8]);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if constexpr (Q_IC) b[j] = lds_operand_transposed(s_q, TL::LDI, wn + j * 32, kk);
                    else b[j] = *reinterpret_cast<const v8bf*>(&s_q[(wn + j * 32 + r32) * TL::LDA + kk + half * 8]);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
            }
        }
    };
    for (int kt = kt_begin; kt < kt_end; kt += 3) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            if (kt + u < kt_end) {
                sp[u].store(s_p);
                sq[u].store(s_q);
                __syncthreads();
                if (kt + u + 3 < kt_end) {
                    sp[u].load(P, g.ldp, m0, (kt + u + 3) * TL::BK, g.M, g.K);
                    sq[u].load(Q, g.ldq, n0, (kt + u + 3) * TL::BK, g.Nn, g.K);
                }
                __builtin_amdgcn_sched_barrier(0);   // requests stay ahead of the multiplications
                multiply_tile();
                __syncthreads();
            }
        }
    }

    // Accumulator element e of lane (r32, half) in tile (i, j) is
    // C[m0 + wm + 32 i + 8 (e/4) + 4 half + e%4][n0 + wn + 32 j + r32].
    if constexpr (EPI == EPI_GRAD) {
        // nabla_w is the one large output (N x N fp32): each wave turns its accumulators through a private
        // LDS area so that a lane stores 16 contiguous bytes and a wave 4 rows x 256 contiguous bytes.
        constexpr int LDE = 64 + 4;
        float* stage = reinterpret_cast<float*>(s_block) + wave * 32 * LDE;
        float* out = static_cast<float*>(g.out);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    stage[(8 * (e >> 2) + 4 * half + (e & 3)) * LDE + j * 32 + r32] = acc[i][j][e];
            // the area is private to the wave: no barrier, LDS operations of a wave complete in order
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int row = 4 * it + (lane >> 4), c4 = (lane & 15) * 4;
                const v4f v = *reinterpret_cast<const v4f*>(&stage[row * LDE + c4]);
                const int m = m0 + wm + i * 32 + row, n = n0 + wn + c4;
                if (m < g.M && n < g.Nn) {
                    float* dst = out + (size_t)m * g.Nn + n;
                    if (g.sgd_eta != 0.0f) {       // the descent step fused in: one more read of the same line
                        const v4f w = *reinterpret_cast<const v4f*>(dst);
                        const v4f o = {fmaf(-g.sgd_eta, v.x, w.x), fmaf(-g.sgd_eta, v.y, w.y),
                                       fmaf(-g.sgd_eta, v.z, w.z), fmaf(-g.sgd_eta, v.w, w.w)};
                        *reinterpret_cast<v4f*>(dst) = o;
                        if (g.out_bf) {            // bfloat16 storage: the weights the next pass multiplies with
                            const v4bf ob = {(__bf16)o.x, (__bf16)o.y, (__bf16)o.z, (__bf16)o.w};
                            *reinterpret_cast<v4bf*>(static_cast<__bf16*>(g.out_bf) + (size_t)m * g.Nn + n) = ob;
                        }
                    } else {
                        store_global_nt_v4f(dst, v);
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn + j * 32 + r32;
            if (n >= g.Nn) continue;
            float bias = 0.0f;
            if constexpr (EPI == EPI_SIGMOID) bias = g.bias[n];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm + i * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                if (m >= g.M) continue;
                const size_t o = (size_t)m * g.Nn + n;
                const float v = acc[i][j][e];
                if constexpr (EPI == EPI_RAW) {
                    g.raw[(size_t)blockIdx.z * g.M * g.Nn + o] = v;
                } else if constexpr (EPI == EPI_SIGMOID) {
                    static_cast<T*>(g.out)[o] = (T)sigmoidf(v + bias);
                } else if constexpr (EPI == EPI_SIGMA_PRIME) {
                    const float a = (float)static_cast<const T*>(g.act)[o];
                    const float d = v * (a * (1.0f - a));
                    static_cast<float*>(g.out)[o] = d;
                    if constexpr (sizeof(T) == 2) static_cast<__bf16*>(g.out_bf)[o] = (__bf16)d;
                } else {
                    __builtin_nontemporal_store(v, static_cast<float*>(g.out) + o);
                }
            }
        }
}


// ================================================================================================
// bf16, large shapes: 256 x 256 tile, 512 threads
// ================================================================================================
// With 64 x 64 wave tiles one K = 16 step reads 4 KB of LDS per wave for 4 MFMAs (128 cycles): four
// busy SIMDs would need 128 bytes per clock, all the LDS has -- the matrix cores wait for operands half
// of the time.  Here a wave owns 64 x 128 (6 KB per 8 MFMAs: 96 bytes per clock), eight waves (4 x 2)
// share a 256 x 256 tile (128 flops per operand byte fetched, against 64), and LDS is double-buffered:
// tile t is multiplied while tile t+1 goes from registers to the other buffer and tile t+2 is
// requested, with one barrier per tile.  Two waves per SIMD cover each other's waits.
namespace big {
constexpr int kThreadsBig = 512;
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int LDA = TK + 8;                // QC operand in LDS: [i][q]
constexpr int LDI = TM + 32;               // IC operand in LDS: [q][i]
constexpr int ELEMS = TM * LDA > TK * LDI ? TM * LDA : TK * LDI;     // per operand and buffer

// 16-byte pieces of one operand tile, four per thread
template <bool IC> struct StageBig;
template <> struct StageBig<false> {       // [i][q]: 8 threads cover the 64 q of one row
    v4f r[4];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int I, int Kq, bool live) {
        const int t = threadIdx.x, qv = (t & 7) * 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = (t >> 3) + 64 * u;
            const bool ok = live && (i0 + i < I) && (q0 + qv < Kq);
            const unsigned off = ((unsigned)(i0 + i) * (unsigned)ld + (unsigned)(q0 + qv)) * 2u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(__bf16* s) const {
        const int t = threadIdx.x, qv = (t & 7) * 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) *reinterpret_cast<v4f*>(s + ((t >> 3) + 64 * u) * LDA + qv) = r[u];
    }
};
template <> struct StageBig<true> {        // [q][i]: 32 threads cover the 256 i of one q
    v4f r[4];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int I, int Kq, bool live) {
        const int t = threadIdx.x, iv = (t & 31) * 8;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = (t >> 5) * 4 + u;
            const bool ok = live && (q0 + q < Kq) && (i0 + iv < I);
            const unsigned off = ((unsigned)(q0 + q) * (unsigned)ld + (unsigned)(i0 + iv)) * 2u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(__bf16* s) const {
        const int t = threadIdx.x, iv = (t & 31) * 8, q = (t >> 5) * 4;
#pragma unroll
        for (int u = 0; u < 4; ++u) *reinterpret_cast<v4f*>(s + (q + u) * LDI + iv) = r[u];
    }
};

// Issue order of one tile's block, as scheduling groups (mask: 0x008 MFMA, 0x020 memory read, 0x100 LDS
// read, 0x200 LDS write).  A k = 16 step is 8 MFMAs; its operands (6 fragments, one or two LDS reads
// each) are read during the step before; the 8 LDS writes and the 8 requests alternate, two of each per
// step.
template <int R, int I>      // I = 8 * step + index of the MFMA within the step
__device__ __forceinline__ void interleave_from() {
    if constexpr (I < 32) {
        constexpr int step = I / 8, m = I % 8, per = (R + 7) / 8;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (step < 3 && m * per < R) __builtin_amdgcn_sched_group_barrier(0x100, per, 0);
        // a staged vector goes to LDS and its registers are requested again right away: every request
        // then has a whole tile's multiplications to come back
        if constexpr (m % 4 == 1) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        if constexpr (m % 4 == 3) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        interleave_from<R, I + 1>();
    }
}
template <bool P_IC, bool Q_IC>
__device__ __forceinline__ void interleave() {
    constexpr int R = (P_IC ? 4 : 2) + (Q_IC ? 8 : 4);     // LDS reads per step (6, 10 or 12)
    __builtin_amdgcn_sched_group_barrier(0x100, R, 0);      // operands of step 0
    interleave_from<R, 0>();
}

template <bool P_IC, bool Q_IC, int EPI>
__global__ __launch_bounds__(kThreadsBig) void k_gemm_big(const GemmArgs g) {
    // Two buffers of two operand tiles; afterwards the staging areas of the epilogue.  Four separate arrays:
    // that writes to one buffer and reads of the other cannot touch the same memory is then visible to
    // the compiler, which may interleave them.
    __shared__ __attribute__((aligned(16))) __bf16 s_p0[ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_q0[ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_p1[ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_q1[ELEMS];

    // Which tile column and which split this workgroup takes.  Workgroups are dealt to the 8 XCDs round-robin
    // in x-first order, so with a multiple of 8 tile columns the XCD is x % 8: the split is taken from x (x % S
    // for S = 2, 4 or 8 splits), so that one XCD's workgroups all work in one range of the contraction and its L2
    // fetches only that part of the operand every tile column shares (P); the workgroups of one tile column and
    // split (they share Q's tiles) stay on one XCD, as before.  Only a matter of which workgroup does what.
    int tile_x = blockIdx.x, split = blockIdx.z;
    {
        const int S = gridDim.z;
        if (S > 1 && S <= 8 && (S & (S - 1)) == 0 && gridDim.x % 8 == 0) {
            split = (int)blockIdx.x % S;
            tile_x = (int)blockIdx.x / S + (int)(gridDim.x / S) * (int)blockIdx.z;
        }
    }
    const int m0 = blockIdx.y * TM, n0 = tile_x * TN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
    const int r32 = lane & 31, half = lane >> 5;

    const int kt_total = ceil_div(g.K, TK);
    const int kt_begin = split * g.k_tiles_per_split;
    const int kt_end = min(kt_total, kt_begin + g.k_tiles_per_split);
    const int T = kt_end - kt_begin;

    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    StageBig<P_IC> sp;
    StageBig<Q_IC> sq;
    const __amdgpu_buffer_rsrc_t P = make_buffer(g.P, g.p_bytes);
    const __amdgpu_buffer_rsrc_t Q = make_buffer(g.Q, g.q_bytes);
    auto request = [&](int t) {       // tiles past the end load zeros: no branch around a request
        sp.load(P, g.ldp, m0, (kt_begin + t) * TK, g.M, g.K, t < T);
        sq.load(Q, g.ldq, n0, (kt_begin + t) * TK, g.Nn, g.K, t < T);
    };
    auto multiply = [&](const __bf16* tp, const __bf16* tq) {
#pragma unroll
        for (int kk = 0; kk < TK; kk += 16) {
            v8bf a[2], b[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if constexpr (P_IC) a[i] = lds_operand_transposed(tp, LDI, wm + i * 32, kk);
                else a[i] = *reinterpret_cast<const v8bf*>(&tp[(wm + i * 32 + r32) * LDA + kk + half * 8]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (Q_IC) b[j] = lds_operand_transposed(tq, LDI, wn + j * 32, kk);
                else b[j] = *reinterpret_cast<const v8bf*>(&tq[(wn + j * 32 + r32) * LDA + kk + half * 8]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };

    // One straight-line block per tile: tile t+1 goes from the registers to the other buffer (last read
    // before the barrier that ended the previous iteration), tile t+2 is requested, tile t is multiplied.
    // The order below is only the data flow; the instructions are interleaved by the groups declared after
    // it, so that the matrix cores run while LDS and memory instructions issue.
    auto tile_block = [&](const __bf16* cur_p, const __bf16* cur_q, __bf16* nxt_p, __bf16* nxt_q, int t) {
        sp.store(nxt_p);
        sq.store(nxt_q);
        request(t + 2);
        multiply(cur_p, cur_q);
        interleave<P_IC, Q_IC>();
        __syncthreads();
    };
    if (T > 0) {
        request(0);
        sp.store(s_p0);
        sq.store(s_q0);
        request(1);
        __syncthreads();
        for (int t = 0; t < T; t += 2) {
            tile_block(s_p0, s_q0, s_p1, s_q1, t);
            if (t + 1 < T) tile_block(s_p1, s_q1, s_p0, s_q0, t + 1);
        }
    }

    // Accumulator element e of lane (r32, half) in tile (i, j) is
    // C[m0 + wm + 32 i + 8 (e/4) + 4 half + e%4][n0 + wn + 32 j + r32].
    // Every epilogue turns the wave's accumulators through a private LDS area (all operand reads are behind
    // the last barrier), so that a lane handles 4 consecutive columns and a wave 2 rows x 512 contiguous
    // bytes per store instruction.  LDS operations of a wave complete in order: no barrier is needed.
    constexpr int LDE = 128 + 4;
    static_assert(2 * 32 * LDE * 4 <= ELEMS * 2, "two waves' staging areas fit one operand buffer");
    __bf16* const area = wave < 2 ? s_p0 : (wave < 4 ? s_q0 : (wave < 6 ? s_p1 : s_q1));
    float* stage = reinterpret_cast<float*>(area) + (wave & 1) * 32 * LDE;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                stage[(8 * (e >> 2) + 4 * half + (e & 3)) * LDE + j * 32 + r32] = acc[i][j][e];
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int row = 2 * it + (lane >> 5), c4 = (lane & 31) * 4;
            const v4f v = *reinterpret_cast<const v4f*>(&stage[row * LDE + c4]);
            const int m = m0 + wm + i * 32 + row, n = n0 + wn + c4;
            if (m >= g.M || n >= g.Nn) continue;              // Nn is a multiple of 4
            const size_t o = (size_t)m * g.Nn + n;
            if constexpr (EPI == EPI_GRAD) {
                float* dst = static_cast<float*>(g.out) + o;
                if (g.sgd_eta != 0.0f) {           // the descent step fused in: fp32 master weights stepped in
                    const v4f w = *reinterpret_cast<const v4f*>(dst);     // place, the bfloat16 weights rewritten
                    const v4f s = {fmaf(-g.sgd_eta, v.x, w.x), fmaf(-g.sgd_eta, v.y, w.y),
                                   fmaf(-g.sgd_eta, v.z, w.z), fmaf(-g.sgd_eta, v.w, w.w)};
                    *reinterpret_cast<v4f*>(dst) = s;
                    const v4bf sb = {(__bf16)s.x, (__bf16)s.y, (__bf16)s.z, (__bf16)s.w};
                    *reinterpret_cast<v4bf*>(static_cast<__bf16*>(g.out_bf) + o) = sb;
                } else {
                    store_global_nt_v4f(dst, v);
                }
            } else if constexpr (EPI == EPI_RAW) {
                *reinterpret_cast<v4f*>(g.raw + (size_t)split * g.M * g.Nn + o) = v;
            } else if constexpr (EPI == EPI_SIGMOID) {
                const v4f bs = *reinterpret_cast<const v4f*>(g.bias + n);
                const v4bf a = {(__bf16)sigmoidf(v.x + bs.x), (__bf16)sigmoidf(v.y + bs.y),
                                (__bf16)sigmoidf(v.z + bs.z), (__bf16)sigmoidf(v.w + bs.w)};
                *reinterpret_cast<v4bf*>(static_cast<__bf16*>(g.out) + o) = a;
            } else {
                const v4bf ab = *reinterpret_cast<const v4bf*>(static_cast<const __bf16*>(g.act) + o);
                v4f d;
                v4bf db;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float a = (float)ab[c];
                    d[c] = v[c] * (a * (1.0f - a));
                    db[c] = (__bf16)d[c];
                }
                *reinterpret_cast<v4f*>(static_cast<float*>(g.out) + o) = d;
                *reinterpret_cast<v4bf*>(static_cast<__bf16*>(g.out_bf) + o) = db;
            }
        }
    }
}

// The gradient product nabla_w = D^T A_prev as one stream of k-tiles over several output tiles.
// Its contraction (the minibatch) is short -- 8 k-tiles at B = 512 -- so a workgroup per output tile spends
// more time starting up (launch, first operands from memory) and storing its 256 KB of fp32 results than
// multiplying.  Here a workgroup is resident for the whole product and walks its tiles: the k-tiles of all of
// them form one stream through the same double-buffered pipeline, so the first operands of the next tile are
// requested, and written to LDS, while the current tile is still being multiplied.  At a tile's end every wave
// stores its accumulators straight to memory (for a fixed accumulator element a half wave holds 32
// consecutive columns of one row: one 128-byte line per row and store instruction; no LDS staging, which
// would collide with the next tile's operands) and goes on multiplying with operands that arrived before
// the stores were issued.
template <int DUMMY>
__global__ __launch_bounds__(kThreadsBig) void k_grad_stream(const GemmArgs g, int tiles_x, int tiles_total) {
    __shared__ __attribute__((aligned(16))) __bf16 s_p0[ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_q0[ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_p1[ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_q1[ELEMS];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
    const int r32 = lane & 31, half = lane >> 5;
    const int T = ceil_div(g.K, TK);                         // k-tiles per output tile
    // my tiles: blockIdx.x, blockIdx.x + gridDim.x, ...  (with a multiple of 8 tile columns and a grid that is a
    // multiple of 8, all of them lie in tile columns of one residue mod 8: the operands of one XCD's L2)
    const int first = blockIdx.x, stride = gridDim.x;
    const int mine = first < tiles_total ? (tiles_total - first + stride - 1) / stride : 0;

    v16f acc[2][4];
    auto clear = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    };
    clear();

    StageBig<true> sp, sq;
    const __amdgpu_buffer_rsrc_t P = make_buffer(g.P, g.p_bytes);
    const __amdgpu_buffer_rsrc_t Q = make_buffer(g.Q, g.q_bytes);
    const __amdgpu_buffer_rsrc_t OUT = make_buffer(g.out, (unsigned)((size_t)g.M * g.Nn * 4u));
    // the k-tile the next request fetches: tile number req_tile of mine, k-tile req_kt of it
    int req_tile = 0, req_kt = 0;
    auto request = [&]() {          // past my last tile: loads of zeros, no branch around a request
        const bool live = req_tile < mine;
        const int t = first + req_tile * stride;
        const int m0 = (t / tiles_x) * TM, n0 = (t % tiles_x) * TN;
        sp.load(P, g.ldp, m0, req_kt * TK, g.M, g.K, live);
        sq.load(Q, g.ldq, n0, req_kt * TK, g.Nn, g.K, live);
        if (++req_kt == T) { req_kt = 0; ++req_tile; }
    };
    auto multiply = [&](const __bf16* tp, const __bf16* tq) {
#pragma unroll
        for (int kk = 0; kk < TK; kk += 16) {
            v8bf a[2], b[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = lds_operand_transposed(tp, LDI, wm + i * 32, kk);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = lds_operand_transposed(tq, LDI, wn + j * 32, kk);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };
    // Accumulator element e of lane (r32, half) in tile (i, j) is
    // C[m0 + wm + 32 i + 8 (e/4) + 4 half + e%4][n0 + wn + 32 j + r32].  The whole byte offset of a store goes
    // into the bounds-checked vector offset (a scalar offset would not be checked): a row past the end of the
    // matrix then lies outside the buffer (no store; the launcher guarantees the sum cannot wrap), a column
    // past the end is given an offset outside it.
    auto store_tile = [&](int tile_no) {
        const int t = first + tile_no * stride;
        const int m0 = (t / tiles_x) * TM, n0 = (t % tiles_x) * TN;
        const int n = n0 + wn + r32;
        const unsigned lane_off = ((unsigned)(m0 + wm + 4 * half) * (unsigned)g.Nn + (unsigned)n) * 4u;
        const unsigned row_bytes = (unsigned)g.Nn * 4u;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool col_ok = n + 32 * j < g.Nn;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const unsigned off = lane_off + 128u * j + (unsigned)(32 * i + 8 * (e >> 2) + (e & 3)) * row_bytes;
                    const float v = acc[i][j][e];      // (a copy: a bit cast of the vector element itself reads element 0)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), OUT, col_ok ? off : kOutside, 0, 2);
                }
            }
    };
    int kt_in_tile = 0, tile_no = 0;
    auto tile_block = [&](const __bf16* cur_p, const __bf16* cur_q, __bf16* nxt_p, __bf16* nxt_q) {
        sp.store(nxt_p);
        sq.store(nxt_q);
        request();
        multiply(cur_p, cur_q);
        interleave<true, true>();
        __syncthreads();
        if (++kt_in_tile == T) {
            store_tile(tile_no);
            clear();
            kt_in_tile = 0;
            ++tile_no;
        }
    };
    if (mine > 0) {
        request();
        sp.store(s_p0);
        sq.store(s_q0);
        request();
        __syncthreads();
        const int total = mine * T;
        for (int it = 0; it < total; it += 2) {
            tile_block(s_p0, s_q0, s_p1, s_q1);
            if (it + 1 < total) tile_block(s_p1, s_q1, s_p0, s_q0);
        }
    }
}

static_assert(TK == Tile<__bf16>::BK, "both bf16 kernels count k-tiles of the same length");
static_assert(2 * 2 * ELEMS * 2 <= 160 * 1024, "LDS of one compute unit");
}  // namespace big

// ================================================================================================
// bf16, large shapes: 128 x 256 tile, 256 threads, two workgroups per compute unit
// ================================================================================================
// The leapfrog schedule runs the chain product of one layer beside the gradient products of the layers
// above it.  The two are complementary -- the chain product is bound by the matrix cores, the gradient
// product by its N x N fp32 store stream -- but kernels whose workgroups fill a compute unit (the
// 256 x 256 kernel above: 512 threads, 147 KB of LDS) cannot share one: they take turns.  This kernel is
// sized for half a compute unit (256 threads, 60 KB of LDS, 256 registers), so that a workgroup of the
// chain product and one of a gradient product -- or two of one product in different phases -- are
// resident together: one multiplies while the other stores, loads or waits at a barrier.
// Same wave tile (64 x 128: 8 matrix instructions per 6 operand fragments), 2 x 2 waves, k-tiles of 32,
// LDS double-buffered, one barrier per k-tile; tile t is multiplied while tile t+1 goes from registers to
// the other buffer and tile t+2 is requested.  The epilogues store straight from the accumulators: for a
// fixed accumulator element the 32 lanes of a half wave hold 32 consecutive columns of one row, a whole
// 128-byte line of fp32 output.
namespace half {
constexpr int kThreadsHalf = 256;
constexpr int TM = 128, TN = 256, TK = 32;
constexpr int LDA = TK + 8;                // QC operand in LDS: [i][q]; 80-byte rows: 16 lanes' 16-byte reads
                                           // fall on 16 different bank groups
constexpr int LDI_P = TM + 32;             // IC operand in LDS: [q][i], rows 16 banks past a multiple of 64
constexpr int LDI_Q = TN + 32;
constexpr int P_ELEMS = TM * LDA > TK * LDI_P ? TM * LDA : TK * LDI_P;
constexpr int Q_ELEMS = TN * LDA > TK * LDI_Q ? TN * LDA : TK * LDI_Q;

// 16-byte pieces of one operand tile of I rows (of its own index), I / 64 per thread
template <int I, bool IC> struct StageHalf;
template <int I> struct StageHalf<I, false> {     // [i][q]: 4 threads cover the 32 q of one row
    v4f r[I / 64];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int Imax, int Kq, bool live) {
        const int t = threadIdx.x, qv = (t & 3) * 8;
#pragma unroll
        for (int u = 0; u < I / 64; ++u) {
            const int i = (t >> 2) + 64 * u;
            const bool ok = live && (i0 + i < Imax) && (q0 + qv < Kq);
            const unsigned off = ((unsigned)(i0 + i) * (unsigned)ld + (unsigned)(q0 + qv)) * 2u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(__bf16* s) const {
        const int t = threadIdx.x, qv = (t & 3) * 8;
#pragma unroll
        for (int u = 0; u < I / 64; ++u) *reinterpret_cast<v4f*>(s + ((t >> 2) + 64 * u) * LDA + qv) = r[u];
    }
};
template <int I> struct StageHalf<I, true> {      // [q][i]: I / 8 threads cover the I entries of one q
    static constexpr int TPQ = I / 8, QPP = kThreadsHalf / TPQ, LDI = I + 32;
    v4f r[I / 64];
    __device__ void load(__amdgpu_buffer_rsrc_t buf, int ld, int i0, int q0, int Imax, int Kq, bool live) {
        const int t = threadIdx.x, iv = (t % TPQ) * 8;
#pragma unroll
        for (int u = 0; u < I / 64; ++u) {
            const int q = t / TPQ + QPP * u;
            const bool ok = live && (q0 + q < Kq) && (i0 + iv < Imax);
            const unsigned off = ((unsigned)(q0 + q) * (unsigned)ld + (unsigned)(i0 + iv)) * 2u;
            r[u] = buffer_load_v4f(buf, ok ? off : kOutside);
        }
    }
    __device__ void store(__bf16* s) const {
        const int t = threadIdx.x, iv = (t % TPQ) * 8;
#pragma unroll
        for (int u = 0; u < I / 64; ++u) *reinterpret_cast<v4f*>(s + (t / TPQ + QPP * u) * LDI + iv) = r[u];
    }
};

// Issue order of one k-tile's block (see big::interleave_from): 16 matrix instructions in two k = 16 steps;
// the second step's operands are read from LDS during the first; each of the six staged vectors is written
// to LDS and requested again back to back, one LDS write or one request after every matrix instruction.
template <int R, int I>
__device__ __forceinline__ void interleave_from() {
    if constexpr (I < 16) {
        constexpr int step = I / 8, m = I % 8, per = (R + 7) / 8;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (step < 1 && m * per < R) __builtin_amdgcn_sched_group_barrier(0x100, per, 0);
        if constexpr (I >= 1 && I <= 12 && I % 2 == 1) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        if constexpr (I >= 1 && I <= 12 && I % 2 == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        interleave_from<R, I + 1>();
    }
}
template <bool P_IC, bool Q_IC>
__device__ __forceinline__ void interleave() {
    constexpr int R = (P_IC ? 4 : 2) + (Q_IC ? 8 : 4);
    __builtin_amdgcn_sched_group_barrier(0x100, R, 0);
    interleave_from<R, 0>();
}

template <bool P_IC, bool Q_IC, int EPI>
__global__ __launch_bounds__(kThreadsHalf, 2) void k_gemm_half(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) __bf16 s_p0[P_ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_q0[Q_ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_p1[P_ELEMS];
    __shared__ __attribute__((aligned(16))) __bf16 s_q1[Q_ELEMS];

    // (Workgroups are dealt to the 8 XCDs, each with an L2 of its own, round-robin by linear index, x fastest.
    // With a multiple of 8 tile columns an XCD therefore owns every 8th tile column and walks it row by row:
    // the workgroups resident on it together share a few operand tiles of either kind, which its L2 holds.)
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 128;
    const int r32 = lane & 31, half = lane >> 5;

    const int kt_total = ceil_div(g.K, TK);
    const int kt_begin = blockIdx.z * g.k_tiles_per_split;
    const int kt_end = min(kt_total, kt_begin + g.k_tiles_per_split);
    const int T = kt_end - kt_begin;

    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    StageHalf<TM, P_IC> sp;
    StageHalf<TN, Q_IC> sq;
    const __amdgpu_buffer_rsrc_t P = make_buffer(g.P, g.p_bytes);
    const __amdgpu_buffer_rsrc_t Q = make_buffer(g.Q, g.q_bytes);
    auto request = [&](int t) {       // tiles past the end load zeros: no branch around a request
        sp.load(P, g.ldp, m0, (kt_begin + t) * TK, g.M, g.K, t < T);
        sq.load(Q, g.ldq, n0, (kt_begin + t) * TK, g.Nn, g.K, t < T);
    };
    auto multiply = [&](const __bf16* tp, const __bf16* tq) {
#pragma unroll
        for (int kk = 0; kk < TK; kk += 16) {
            v8bf a[2], b[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if constexpr (P_IC) a[i] = lds_operand_transposed(tp, LDI_P, wm + i * 32, kk);
                else a[i] = *reinterpret_cast<const v8bf*>(&tp[(wm + i * 32 + r32) * LDA + kk + half * 8]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (Q_IC) b[j] = lds_operand_transposed(tq, LDI_Q, wn + j * 32, kk);
                else b[j] = *reinterpret_cast<const v8bf*>(&tq[(wn + j * 32 + r32) * LDA + kk + half * 8]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };
    auto tile_block = [&](const __bf16* cur_p, const __bf16* cur_q, __bf16* nxt_p, __bf16* nxt_q, int t) {
        sp.store(nxt_p);
        sq.store(nxt_q);
        request(t + 2);
        multiply(cur_p, cur_q);
        interleave<P_IC, Q_IC>();
        __syncthreads();
    };
    if (T > 0) {
        request(0);
        sp.store(s_p0);
        sq.store(s_q0);
        request(1);
        __syncthreads();
        for (int t = 0; t < T; t += 2) {
            tile_block(s_p0, s_q0, s_p1, s_q1, t);
            if (t + 1 < T) tile_block(s_p1, s_q1, s_p0, s_q0, t + 1);
        }
    }

    // Accumulator element e of lane (r32, half) in tile (i, j) is
    // C[m0 + wm + 32 i + 8 (e/4) + 4 half + e%4][n0 + wn + 32 j + r32]: for a fixed e a half wave holds 32
    // consecutive columns of one row, so every store instruction writes two whole 128-byte lines of fp32.
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn + j * 32 + r32;
            if (n >= g.Nn) continue;
            float bias = 0.0f;
            if constexpr (EPI == EPI_SIGMOID) bias = g.bias[n];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm + i * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                if (m >= g.M) continue;
                const size_t o = (size_t)m * g.Nn + n;
                const float v = acc[i][j][e];
                if constexpr (EPI == EPI_GRAD) {
                    float* dst = static_cast<float*>(g.out) + o;
                    if (g.sgd_eta != 0.0f) {       // the descent step fused in: fp32 master weights stepped in
                        const float w = fmaf(-g.sgd_eta, v, *dst);       // place, the bfloat16 weights rewritten
                        *dst = w;
                        static_cast<__bf16*>(g.out_bf)[o] = (__bf16)w;
                    } else {
                        __builtin_nontemporal_store(v, (__attribute__((address_space(1))) float*)dst);
                    }
                } else if constexpr (EPI == EPI_RAW) {
                    g.raw[(size_t)blockIdx.z * g.M * g.Nn + o] = v;
                } else if constexpr (EPI == EPI_SIGMOID) {
                    static_cast<__bf16*>(g.out)[o] = (__bf16)sigmoidf(v + bias);
                } else {
                    const float a = (float)static_cast<const __bf16*>(g.act)[o];
                    const float d = v * (a * (1.0f - a));
                    static_cast<float*>(g.out)[o] = d;
                    static_cast<__bf16*>(g.out_bf)[o] = (__bf16)d;
                }
            }
        }
}

static_assert(2 * (P_ELEMS + Q_ELEMS) * 2 <= 80 * 1024, "two workgroups' LDS fit one compute unit");
}  // namespace half

// Split-K second stage: sum the raw partials in split order, then the layer's epilogue.  A thread takes four
// consecutive outputs (one row: every width is a multiple of 4), 16 bytes per load.
template <typename T, int EPI>
__global__ __launch_bounds__(kThreads) void k_split_finish(const float* __restrict__ raw, int splits,
                                                           size_t count, int Nn,
                                                           const float* __restrict__ bias,
                                                           const T* __restrict__ act, void* out,
                                                           __bf16* out_bf) {
    const size_t o = ((size_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (o >= count) return;
    v4f v = *reinterpret_cast<const v4f*>(raw + o);
    for (int z = 1; z < splits; ++z) v += *reinterpret_cast<const v4f*>(raw + (size_t)z * count + o);
    if constexpr (EPI == EPI_SIGMOID) {
        const v4f bs = *reinterpret_cast<const v4f*>(bias + o % Nn);
        typedef T v4t __attribute__((ext_vector_type(4)));
        const v4t r = {(T)sigmoidf(v[0] + bs[0]), (T)sigmoidf(v[1] + bs[1]), (T)sigmoidf(v[2] + bs[2]),
                       (T)sigmoidf(v[3] + bs[3])};
        *reinterpret_cast<v4t*>(static_cast<T*>(out) + o) = r;
    } else {
        typedef T v4t __attribute__((ext_vector_type(4)));
        const v4t av = *reinterpret_cast<const v4t*>(act + o);
        v4f d;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float a = (float)av[c];
            d[c] = v[c] * (a * (1.0f - a));
        }
        *reinterpret_cast<v4f*>(static_cast<float*>(out) + o) = d;
        if constexpr (sizeof(T) == 2) {
            const v4bf db = {(__bf16)d[0], (__bf16)d[1], (__bf16)d[2], (__bf16)d[3]};
            *reinterpret_cast<v4bf*>(out_bf + o) = db;
        }
    }
}

// eq. (bp3) for a minibatch: nabla_b[j] = sum_b D[b][j].  A workgroup owns 32 columns; its 8 row groups
// each add every 8th sample in ascending order, then the 8 partial sums are added in group order.
// sgd_eta != 0: nabla_b is b^l itself and receives b - eta * sum.
__global__ __launch_bounds__(kThreads) void k_bias_grad(const float* __restrict__ D, float* nabla_b, int N,
                                                        int B, float sgd_eta) {
    __shared__ float s_part[8][32];
    const int c = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int j = blockIdx.x * 32 + c;
    float s = 0.0f;
    if (j < N) {
        // eight rows requested at a time, added in ascending order
        int b = rg;
        for (; b + 56 < B; b += 64) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = D[(size_t)(b + 8 * u) * N + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; b < B; b += 8) s += D[(size_t)b * N + j];
    }
    s_part[rg][c] = s;
    __syncthreads();
    if (rg == 0 && j < N) {
        float t = s_part[0][c];
#pragma unroll
        for (int q = 1; q < 8; ++q) t += s_part[q][c];
        nabla_b[j] = sgd_eta != 0.0f ? fmaf(-sgd_eta, t, nabla_b[j]) : t;
    }
}

template <typename T, bool P_IC, bool Q_IC, int EPI>
hipError_t run(GemmArgs g, int splits, hipStream_t s) {
    // operand sizes for the buffer addressing: P is (P_IC ? K x M : M x K), Q likewise with Nn
    const unsigned long long pb = (unsigned long long)(P_IC ? g.K : g.M) * g.ldp * sizeof(T);
    const unsigned long long qb = (unsigned long long)(Q_IC ? g.K : g.Nn) * g.ldq * sizeof(T);
    if (pb >= 0xFFFFFFF0ull || qb >= 0xFFFFFFF0ull) return hipErrorInvalidValue;
    g.p_bytes = (unsigned)pb;
    g.q_bytes = (unsigned)qb;
    const dim3 grid(ceil_div(g.Nn, BN), ceil_div(g.M, BM), splits);
    k_gemm<T, P_IC, Q_IC, EPI><<<grid, kThreads, 0, s>>>(g);
    return hipGetLastError();
}

template <bool P_IC, bool Q_IC, int EPI>
hipError_t run_big(GemmArgs g, int splits, hipStream_t s) {
    const unsigned long long pb = (unsigned long long)(P_IC ? g.K : g.M) * g.ldp * 2ull;
    const unsigned long long qb = (unsigned long long)(Q_IC ? g.K : g.Nn) * g.ldq * 2ull;
    if (pb >= 0xFFFFFFF0ull || qb >= 0xFFFFFFF0ull) return hipErrorInvalidValue;
    g.p_bytes = (unsigned)pb;
    g.q_bytes = (unsigned)qb;
    const dim3 grid(ceil_div(g.Nn, big::TN), ceil_div(g.M, big::TM), splits);
    big::k_gemm_big<P_IC, Q_IC, EPI><<<grid, big::kThreadsBig, 0, s>>>(g);
    return hipGetLastError();
}

// The streamed gradient product (big::k_grad_stream): `groups` resident workgroups walk all output tiles.
hipError_t run_grad_stream(GemmArgs g, int groups, hipStream_t s) {
    const unsigned long long pb = (unsigned long long)g.K * g.ldp * 2ull, qb = (unsigned long long)g.K * g.ldq * 2ull;
    // (the result is addressed with 32-bit offsets that may point up to one tile of rows past its end)
    const unsigned long long ob = (unsigned long long)(g.M + big::TM) * g.Nn * 4ull;
    if (pb >= 0xFFFFFFF0ull || qb >= 0xFFFFFFF0ull || ob >= 0xFFFFFFF0ull) return hipErrorInvalidValue;
    g.p_bytes = (unsigned)pb;
    g.q_bytes = (unsigned)qb;
    const int tiles_x = ceil_div(g.Nn, big::TN), tiles = tiles_x * ceil_div(g.M, big::TM);
    big::k_grad_stream<0><<<groups < tiles ? groups : tiles, big::kThreadsBig, 0, s>>>(g, tiles_x, tiles);
    return hipGetLastError();
}

template <bool P_IC, bool Q_IC, int EPI>
hipError_t run_half(GemmArgs g, int splits, hipStream_t s) {
    const unsigned long long pb = (unsigned long long)(P_IC ? g.K : g.M) * g.ldp * 2ull;
    const unsigned long long qb = (unsigned long long)(Q_IC ? g.K : g.Nn) * g.ldq * 2ull;
    if (pb >= 0xFFFFFFF0ull || qb >= 0xFFFFFFF0ull) return hipErrorInvalidValue;
    g.p_bytes = (unsigned)pb;
    g.q_bytes = (unsigned)qb;
    const dim3 grid(ceil_div(g.Nn, half::TN), ceil_div(g.M, half::TM), splits);
    half::k_gemm_half<P_IC, Q_IC, EPI><<<grid, half::kThreadsHalf, 0, s>>>(g);
    return hipGetLastError();
}

}  // namespace

// Which kernels a minibatch net takes, decided once per net from its widest layer.  bf16 nets whose forward
// product has at least 64 tiles of 256 x 256 take the wide-net kernels: by default the 256 x 256-tile kernel for
// all three products (measured faster than the 128 x 256 one, alone and beside each other).
// How such a net shares the chip between the chain and the workers: a kernel of either kind fills every compute
// unit it gets (registers, LDS), so two of them never share one; what can be shared is the set of compute
// units.  The chain product is split only two ways along K -- 128 workgroups, half the chip (and half the
// split's partial-sum traffic) -- the streamed gradient product keeps 96 workgroups resident, and the k workers
// run on two streams (worker j on stream j mod 2), so that at most two gradient products are in flight and the
// next chain kernel always finds compute units.  Measured at L = 48, N = 8192, B = 512, k = 8: 7.0 ms per backward
// pass against 8.0 ms with every kernel spread over the whole chip.  (The split does not depend on k: the
// gradients must be the same bits for every k.  A sequential pass, k = 1, would be faster with four splits.)
// Overrides for tests and A/B runs, read when the plan is made:
// LF_GEMM_BIG=0/1 forces the narrow / wide-net kernels; LF_GEMM_CHAIN_TILE = "big" or "half" picks the wide-net
// kernel of the forward and chain products, LF_GEMM_GRAD_TILE = "stream" (default), "big" or "half" that of the
// gradient product; LF_GEMM_SPLIT_TARGET = workgroups the split of a chain-side product aims at (both products),
// LF_GEMM_CHAIN_SPLIT_TARGET = the same for the backward chain product alone; LF_GEMM_STREAM_GROUPS = resident
// workgroups of the streamed gradient product; LF_WORKER_STREAMS (read by the schedule) = streams the workers share.
GemmPlan gemm_plan(int N, int B, bool bf16) {
    // (narrow kernels: one stream for all workers -- at L = 32, N = 4096, B = 256, k = 4 the backward pass takes
    // 4.4-4.5 ms with one worker stream and 4.6-4.7 ms with four: gradient products that queue behind each other
    // leave the chain its compute units)
    GemmPlan p{GEMM_128, GEMM_128, 512, 512, 256, 1};
    bool wide = bf16 && ceil_div(B, big::TM) * ceil_div(N, big::TN) >= 64;
    if (const char* e = getenv("LF_GEMM_BIG")) {
        if (e[0] == '0') wide = false;
        if (e[0] == '1') wide = bf16;
    }
    if (wide) {
        p.chain = GEMM_BIG;
        p.grad = GEMM_STREAM;
        p.split_target = 256;
        p.chain_split_target = 128;
        p.stream_groups = 96;
        p.worker_streams = 2;
        if (const char* e = getenv("LF_GEMM_CHAIN_TILE")) p.chain = e[0] == 'b' ? GEMM_BIG : GEMM_HALF;
        if (const char* e = getenv("LF_GEMM_GRAD_TILE")) p.grad = e[0] == 'b' ? GEMM_BIG : (e[0] == 's' ? GEMM_STREAM : GEMM_HALF);
    }
    if (const char* e = getenv("LF_GEMM_STREAM_GROUPS")) {
        const int t = atoi(e);
        if (t >= 8 && t <= 1024) p.stream_groups = t;
    }
    if (const char* e = getenv("LF_GEMM_SPLIT_TARGET")) {
        const int t = atoi(e);
        if (t >= 64 && t <= 2048) p.split_target = p.chain_split_target = t;
    }
    if (const char* e = getenv("LF_GEMM_CHAIN_SPLIT_TARGET")) {
        const int t = atoi(e);
        if (t >= 64 && t <= 2048) p.chain_split_target = t;
    }
    return p;
}

int chain_splits(int n_out, int K, int B, bool bf16, int kernel, int target) {
    if (kernel == GEMM_HALF) {
        const int tiles = ceil_div(n_out, half::TN) * ceil_div(B, half::TM);
        const int kt = ceil_div(K, half::TK);
        int s = 1;
        while (tiles * s < target && s < 16 && kt / (s * 2) >= 8) s *= 2;
        return s;
    }
    if (kernel == GEMM_BIG) {
        const int tiles = ceil_div(n_out, big::TN) * ceil_div(B, big::TM);
        const int kt = ceil_div(K, big::TK);
        int s = 1;
        while (tiles * s < target && s < 16 && kt / (s * 2) >= 4) s *= 2;   // one workgroup per compute unit
        return s;
    }
    const int tiles = ceil_div(n_out, BN) * ceil_div(B, BM);
    const int kt = ceil_div(K, bf16 ? Tile<__bf16>::BK : Tile<float>::BK);
    int s = 1;
    while (tiles * s < target && s < 16 && kt / (s * 2) >= 4) s *= 2;
    return s;
}

size_t split_workspace_floats(int n_out, int K, int B, bool bf16) {      // enough for any plan
    (void)K; (void)bf16;
    return (size_t)16 * B * n_out;                                       // no plan splits more than 16 ways
}

size_t split_scratch_floats(int n_out, int K, int B, bool bf16, const GemmPlan& plan, bool chain_product) {
    const int s = chain_splits(n_out, K, B, bf16, plan.chain, chain_product ? plan.chain_split_target : plan.split_target);
    return s > 1 ? (size_t)s * B * n_out : 0;
}

template <typename T>
static hipError_t fwd_impl(const void* W, const float* bias, const void* A_in, void* A_out, float* raw,
                           int n_out, int n_in, int B, const GemmPlan& plan, hipStream_t s) {
    constexpr bool bf = sizeof(T) == 2;
    const int splits = chain_splits(n_out, n_in, B, bf, plan.chain, plan.split_target);
    GemmArgs g{};
    g.P = A_in; g.ldp = n_in; g.Q = W; g.ldq = n_in; g.M = B; g.Nn = n_out; g.K = n_in;
    g.k_tiles_per_split = ceil_div(ceil_div(n_in, Tile<T>::BK), splits);
    g.bias = bias; g.out = A_out; g.raw = raw;
    hipError_t e;
    if constexpr (bf) {
        if (plan.chain == GEMM_HALF) {
            g.k_tiles_per_split = ceil_div(ceil_div(n_in, half::TK), splits);
            if (splits == 1) return run_half<false, false, EPI_SIGMOID>(g, 1, s);
            e = run_half<false, false, EPI_RAW>(g, splits, s);
        } else if (plan.chain == GEMM_BIG) {
            if (splits == 1) return run_big<false, false, EPI_SIGMOID>(g, 1, s);
            e = run_big<false, false, EPI_RAW>(g, splits, s);
        } else {
            if (splits == 1) return run<T, false, false, EPI_SIGMOID>(g, 1, s);
            e = run<T, false, false, EPI_RAW>(g, splits, s);
        }
    } else {
        if (splits == 1) return run<T, false, false, EPI_SIGMOID>(g, 1, s);
        e = run<T, false, false, EPI_RAW>(g, splits, s);
    }
    if (e != hipSuccess) return e;
    const size_t count = (size_t)B * n_out;
    k_split_finish<T, EPI_SIGMOID><<<(unsigned)((count / 4 + kThreads - 1) / kThreads), kThreads, 0, s>>>(
        raw, splits, count, n_out, bias, nullptr, A_out, nullptr);
    return hipGetLastError();
}

template <typename T>
static hipError_t chain_impl(const void* W_next, const void* D_next_op, const void* A_l, float* D_l,
                             void* D_l_bf, float* raw, int n_l, int n_next, int B, const GemmPlan& plan,
                             hipStream_t s) {
    constexpr bool bf = sizeof(T) == 2;
    const int splits = chain_splits(n_l, n_next, B, bf, plan.chain, plan.chain_split_target);
    GemmArgs g{};
    g.P = D_next_op; g.ldp = n_next; g.Q = W_next; g.ldq = n_l; g.M = B; g.Nn = n_l; g.K = n_next;
    g.k_tiles_per_split = ceil_div(ceil_div(n_next, Tile<T>::BK), splits);
    g.act = A_l; g.out = D_l; g.out_bf = D_l_bf; g.raw = raw;
    hipError_t e;
    if constexpr (bf) {
        if (plan.chain == GEMM_HALF) {
            g.k_tiles_per_split = ceil_div(ceil_div(n_next, half::TK), splits);
            if (splits == 1) return run_half<false, true, EPI_SIGMA_PRIME>(g, 1, s);
            e = run_half<false, true, EPI_RAW>(g, splits, s);
        } else if (plan.chain == GEMM_BIG) {
            if (splits == 1) return run_big<false, true, EPI_SIGMA_PRIME>(g, 1, s);
            e = run_big<false, true, EPI_RAW>(g, splits, s);
        } else {
            if (splits == 1) return run<T, false, true, EPI_SIGMA_PRIME>(g, 1, s);
            e = run<T, false, true, EPI_RAW>(g, splits, s);
        }
    } else {
        if (splits == 1) return run<T, false, true, EPI_SIGMA_PRIME>(g, 1, s);
        e = run<T, false, true, EPI_RAW>(g, splits, s);
    }
    if (e != hipSuccess) return e;
    const size_t count = (size_t)B * n_l;
    k_split_finish<T, EPI_SIGMA_PRIME><<<(unsigned)((count / 4 + kThreads - 1) / kThreads), kThreads, 0, s>>>(
        raw, splits, count, n_l, nullptr, static_cast<const T*>(A_l), D_l, static_cast<__bf16*>(D_l_bf));
    return hipGetLastError();
}

hipError_t launch_fwd_gemm(const void* W, const float* bias, const void* A_in, void* A_out, float* raw,
                           int n_out, int n_in, int B, bool bf16, const GemmPlan& plan, hipStream_t s) {
    return bf16 ? fwd_impl<__bf16>(W, bias, A_in, A_out, raw, n_out, n_in, B, plan, s)
                : fwd_impl<float>(W, bias, A_in, A_out, raw, n_out, n_in, B, plan, s);
}

hipError_t launch_chain_gemm(const void* W_next, const float* D_next, const void* D_next_bf,
                             const void* A_l, float* D_l, void* D_l_bf, float* raw, int n_l, int n_next,
                             int B, bool bf16, const GemmPlan& plan, hipStream_t s) {
    return bf16 ? chain_impl<__bf16>(W_next, D_next_bf, A_l, D_l, D_l_bf, raw, n_l, n_next, B, plan, s)
                : chain_impl<float>(W_next, D_next, A_l, D_l, nullptr, raw, n_l, n_next, B, plan, s);
}

hipError_t launch_grad_gemm(const float* D, const void* D_bf, const void* A_prev, float* nabla_w,
                            float* nabla_b, int n_l, int n_prev, int B, bool bf16, const GemmPlan& plan,
                            bool whole_chip, float sgd_eta, void* w_bf, hipStream_t s) {
    if (sgd_eta != 0.0f && bf16 != (w_bf != nullptr)) return hipErrorInvalidValue;
    k_bias_grad<<<ceil_div(n_l, 32), kThreads, 0, s>>>(D, nabla_b, n_l, B, sgd_eta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    GemmArgs g{};
    g.ldp = n_l; g.Q = A_prev; g.ldq = n_prev; g.M = n_l; g.Nn = n_prev; g.K = B;
    g.out = nabla_w;
    g.sgd_eta = sgd_eta;
    g.out_bf = sgd_eta != 0.0f ? w_bf : nullptr;
    if (bf16) {
        g.P = D_bf;
        g.k_tiles_per_split = ceil_div(B, Tile<__bf16>::BK);
        if (plan.grad == GEMM_HALF) {
            g.k_tiles_per_split = ceil_div(B, half::TK);
            return run_half<true, true, EPI_GRAD>(g, 1, s);
        }
        // the streamed kernel stores gradients only (the descent step keeps the tile-per-workgroup kernel) and
        // addresses the result through one 32-bit buffer
        if (plan.grad == GEMM_STREAM && sgd_eta == 0.0f &&
            (unsigned long long)(n_l + big::TM) * n_prev * 4ull < 0xFFFFFFF0ull)
            return run_grad_stream(g, whole_chip ? 256 : plan.stream_groups, s);
        if (plan.grad == GEMM_BIG || plan.grad == GEMM_STREAM) return run_big<true, true, EPI_GRAD>(g, 1, s);
        return run<__bf16, true, true, EPI_GRAD>(g, 1, s);
    }
    g.P = D;
    g.k_tiles_per_split = ceil_div(B, Tile<float>::BK);
    return run<float, true, true, EPI_GRAD>(g, 1, s);
}

}  // namespace lf
