// Internal interface between the C-ABI layer (lf_api.hip) and the kernel files.
// Every launcher only enqueues work on `s` and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "device_helpers.h"

namespace lf {

// ---- single-sample (B = 1) fp32 path: HBM-bound GEMV / outer-product kernels --------------------

// Row blocks the transposed GEMV of eq. (bp2) is split into (size of its partial buffer, [P][N]).
int chain_partial_blocks(int N);

// eqs. (z),(a): a_out = sigma(W a_in + b)
hipError_t launch_fwd_gemv_f32(const float* W, const float* b, const float* a_in, float* a_out,
                               int N, hipStream_t s);
// eq. (bp2): delta_l = (W_next^T delta_next) (.) a_l (1 - a_l); partial: [chain_partial_blocks(N)][N]
hipError_t launch_chain_gemvT_f32(const float* W_next, const float* delta_next, const float* a_l,
                                  float* delta_l, float* partial, int N, hipStream_t s);
// eqs. (bp3),(bp4): nabla_b = delta; nabla_w[j][k] = delta[j] a_prev[k]
hipError_t launch_grad_outer_f32(const float* delta, const float* a_prev, float* nabla_w,
                                 float* nabla_b, int N, hipStream_t s);

// ---- any B, either storage type ----------------------------------------------------------------

// eq. (bp1): delta_L = scale * (a_L - y) (.) a_L (1 - a_L) over count = B*N elements (scale: a power
// of two, see lf_set_cost_scale).  delta_bf (may be NULL) receives a bfloat16 copy of delta_L for the
// bf16 matrix kernels.
hipError_t launch_output_error(const void* a_L, const void* y, float* delta_L, void* delta_bf,
                               size_t count, bool bf16, float scale, hipStream_t s);

// ---- minibatch path: MFMA contractions ----------------------------------------------------------

// Floats of scratch the split-K stage of the forward / chain contractions needs (0 = no split).
size_t split_workspace_floats(int N, int B, bool bf16);
// Whether a net of this shape takes the 256 x 256-tile bf16 kernel (decided once per net; `big_tiles` below).
bool gemm_use_big(int N, int B, bool bf16);

// eqs. (z),(a) for a minibatch: A_out[b][j] = sigma(sum_k A_in[b][k] W[j][k] + bias[j])
// `raw` is the split-K scratch, split_workspace_floats(N, B, bf16) floats (may be NULL when that is 0).
hipError_t launch_fwd_gemm(const void* W, const float* bias, const void* A_in, void* A_out, float* raw,
                           int N, int B, bool bf16, bool big_tiles, hipStream_t s);
// eq. (bp2) for a minibatch: D_l[b][k] = (sum_j D_next[b][j] W_next[j][k]) A_l[b][k] (1 - A_l[b][k]).
// For bf16, D_next_bf / D_l_bf are the bfloat16 copies used as matrix operands.
hipError_t launch_chain_gemm(const void* W_next, const float* D_next, const void* D_next_bf,
                             const void* A_l, float* D_l, void* D_l_bf, float* raw,
                             int N, int B, bool bf16, bool big_tiles, hipStream_t s);
// eqs. (bp3),(bp4) for a minibatch: nabla_w[j][k] = sum_b D[b][j] A_prev[b][k];
// nabla_b[j] = sum_b D[b][j] (fixed summation order).
hipError_t launch_grad_gemm(const float* D, const void* D_bf, const void* A_prev, float* nabla_w,
                            float* nabla_b, int N, int B, bool bf16, bool big_tiles, hipStream_t s);

}  // namespace lf
