// Internal interface between the C-ABI layer (lf_api.hip) and the kernel files.
// Every launcher only enqueues work on `s` and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "device_helpers.h"

namespace lf {

// ---- single-sample (B = 1) fp32 path: HBM-bound GEMV / outer-product kernels --------------------
// Matrices are rows x cols, row-major: w^l has n_l rows and n_{l-1} columns.

// Row blocks the transposed GEMV of eq. (bp2) is split into (its partial buffer is [P][cols]).
int chain_partial_blocks(int rows);

// eqs. (z),(a): a_out = sigma(W a_in + b)
hipError_t launch_fwd_gemv_f32(const float* W, const float* b, const float* a_in, float* a_out,
                               int rows, int cols, hipStream_t s);
// eq. (bp2): delta_l = (W_next^T delta_next) (.) a_l (1 - a_l); W_next is rows x cols, delta_next has rows
// entries, delta_l and a_l cols; partial: [chain_partial_blocks(rows)][cols]
hipError_t launch_chain_gemvT_f32(const float* W_next, const float* delta_next, const float* a_l,
                                  float* delta_l, float* partial, int rows, int cols, hipStream_t s);
// eqs. (bp3),(bp4): nabla_b = delta (rows entries); nabla_w[j][k] = delta[j] a_prev[k] (rows x cols).
// sgd_eta != 0: the descent step fused in -- nabla_w and nabla_b are then w^l and b^l themselves and receive
// w - eta nabla_w, b - eta nabla_b; the gradients are not stored.
hipError_t launch_grad_outer_f32(const float* delta, const float* a_prev, float* nabla_w,
                                 float* nabla_b, int rows, int cols, float sgd_eta, hipStream_t s);

// ---- any B, either storage type ----------------------------------------------------------------

// eq. (bp1): delta_L = scale * (a_L - y) (.) a_L (1 - a_L) over count = B*N elements (scale: a power
// of two, see lf_set_cost_scale).  delta_bf (may be NULL) receives a bfloat16 copy of delta_L for the
// bf16 matrix kernels.
hipError_t launch_output_error(const void* a_L, const void* y, float* delta_L, void* delta_bf,
                               size_t count, bool bf16, float scale, hipStream_t s);

// ---- minibatch path: MFMA contractions ----------------------------------------------------------

// Floats of scratch the split-K stage of a forward / chain contraction with a B x n_out result and
// contraction length K needs (0 = no split).
size_t split_workspace_floats(int n_out, int K, int B, bool bf16);
struct GemmPlan;
// Floats of split-K scratch the forward (chain_product = false) or chain product actually uses under a plan.
size_t split_scratch_floats(int n_out, int K, int B, bool bf16, const GemmPlan& plan, bool chain_product);
// Which matrix kernel a product takes: 128 x 128 tiles (fp32; bf16 nets of moderate width), or one of the two
// wide-net bf16 kernels -- 256 x 256 tiles filling a compute unit, or 128 x 256 tiles sized so that two
// workgroups (of one product or of two) share a compute unit; the gradient product also as resident workgroups
// that stream through all their 256 x 256 tiles.
enum GemmKernel { GEMM_128 = 0, GEMM_BIG = 1, GEMM_HALF = 2, GEMM_STREAM = 3 };   // STREAM: gradient product only
struct GemmPlan {
    int chain;          // GemmKernel of the forward and chain products
    int grad;           // GemmKernel of the gradient product
    int split_target;   // workgroups the K split of the forward product aims at
    int chain_split_target;   // the same for the chain product of the backward pass
    int stream_groups;  // resident workgroups of the streamed gradient product
    int worker_streams; // streams the k workers share (worker j runs on stream j mod this)
};
// The plan of a net whose widest layer has N neurons (decided once per net).
GemmPlan gemm_plan(int N, int B, bool bf16);

// eqs. (z),(a) for a minibatch: A_out[b][j] = sigma(sum_k A_in[b][k] W[j][k] + bias[j]); W is n_out x n_in.
// `raw` is the split-K scratch, split_workspace_floats(n_out, n_in, B, bf16) floats (may be NULL when that is 0).
hipError_t launch_fwd_gemm(const void* W, const float* bias, const void* A_in, void* A_out, float* raw,
                           int n_out, int n_in, int B, bool bf16, const GemmPlan& plan, hipStream_t s);
// eq. (bp2) for a minibatch: D_l[b][k] = (sum_j D_next[b][j] W_next[j][k]) A_l[b][k] (1 - A_l[b][k]);
// W_next is n_next x n_l.  For bf16, D_next_bf / D_l_bf are the bfloat16 copies used as matrix operands.
// raw: split_workspace_floats(n_l, n_next, B, bf16) floats.
hipError_t launch_chain_gemm(const void* W_next, const float* D_next, const void* D_next_bf,
                             const void* A_l, float* D_l, void* D_l_bf, float* raw,
                             int n_l, int n_next, int B, bool bf16, const GemmPlan& plan, hipStream_t s);
// eqs. (bp3),(bp4) for a minibatch: nabla_w[j][k] = sum_b D[b][j] A_prev[b][k] (n_l x n_prev);
// nabla_b[j] = sum_b D[b][j] (fixed summation order).
// sgd_eta != 0: the descent step fused into the epilogues -- nabla_w and nabla_b are then w^l (in fp32) and b^l
// themselves and receive w - eta nabla_w, b - eta nabla_b; the gradients are not stored.  With bfloat16 storage
// nabla_w is the fp32 master copy of w^l, and w_bf, the bfloat16 weights, are rewritten as its rounding (w_bf
// is NULL exactly when the storage is fp32).  whole_chip: nothing runs beside this product (the sequential
// pass), so the streamed kernel keeps a workgroup on every compute unit instead of the plan's share.
hipError_t launch_grad_gemm(const float* D, const void* D_bf, const void* A_prev, float* nabla_w,
                            float* nabla_b, int n_l, int n_prev, int B, bool bf16, const GemmPlan& plan,
                            bool whole_chip, float sgd_eta, void* w_bf, hipStream_t s);

}  // namespace lf
